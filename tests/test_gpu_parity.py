"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Needs a real MI355X."""
import numpy as np
import pytest

import oracle
from paper_2312_17530_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


AUTO, FULL_MAP = 0, 1     # ranking paths of the library (same result, different traffic)


@pytest.fixture(params=[False, True], ids=["two_arenas", "in_place"])
def in_place(request):
    """Where the new residual goes: a second arena (the form bench.py times) or the same one."""
    return request.param


def _session(shapes, p, alpha, ratios, p_per_layer=None, path=AUTO, in_place=False, work_feed=0):
    from paper_2312_17530_amd.session import Session
    return Session(shapes, p, alpha, ratios, p_per_layer, path=path, in_place=in_place, work_feed=work_feed)


FEED_AUTO, FEED_OFF, FEED_ON = 0, 1, 2


def run_and_check(shapes, p_list, alpha, ratios, grads_per_iter, name="case", check_nsi=True,
                  path=AUTO, in_place=False, work_feed=FEED_AUTO):
    """Runs every iteration on GPU and oracle from identical state and applies the parity rule.
    Returns (number of layer-iterations compared, number that matched the oracle exactly)."""
    import torch
    sess = _session(shapes, p_list[0], alpha, ratios, p_list, path, in_place, work_feed)
    name = f"{name}/{'in_place' if in_place else 'two_arenas'}"
    L = len(shapes)
    resid = [np.zeros(sh, dtype=np.float32) for sh in shapes]
    n_cmp = n_exact = 0
    for t, grads in enumerate(grads_per_iter):
        sess.set_grad(grads)
        sess.set_residual(resid)
        if check_nsi:
            gpu_nsi = sess.nsi(use_residual=True)
        sess.compress()
        torch.cuda.synchronize()
        res = sess.results()
        gpu_r = sess.unpack(sess.residual)
        dense = sess.unpack(sess.decompress(accumulate=False))
        new_resid = []
        for l in range(L):
            o = oracle.compress_layer(grads[l], resid[l], p_list[l], alpha, ratios[l])
            tag = f"{name}[t={t},l={l},{shapes[l]},p={p_list[l]}]"
            assert sess.plan.layer_k(l) == o.k, tag
            if check_nsi:
                ok = parity.nsi_close(gpu_nsi[l], o.nsi)
                assert ok.all(), f"{tag}: {int((~ok).sum())} scores outside tolerance"
            gi, gv, gc, gn = res[l]
            exact = parity.check_layer(tag, shapes[l], p_list[l], o.k, o.tau, o.nsi, o.centres,
                                       o.idx, o.val, o.r_new, o.v, gi, gv, gc, gn, gpu_r[l])
            # decompress(accumulate=0) + residual == v, bitwise
            d = dense[l].reshape(-1)
            want = np.zeros(d.size, dtype=np.float32)
            want[gi] = gv
            assert np.array_equal(d.view(np.uint32), want.view(np.uint32)), f"{tag}: decompress"
            n_cmp += 1
            n_exact += int(exact)
            # continue from the oracle's state (identical unless the tolerance band was used)
            new_resid.append(o.r_new)
        resid = new_resid
    return n_cmp, n_exact


def run_and_check_momentum(shapes, p_list, alpha, ratios, m, grads_per_iter, name, u0=None, r0=None,
                           work_feed=FEED_AUTO):
    """Eq. 12 in full: every iteration on GPU and oracle from identical (u, r) state."""
    import torch
    from paper_2312_17530_amd.session import Session
    sess = Session(shapes, p_list[0], alpha, ratios, p_list, momentum=m, work_feed=work_feed)
    L = len(shapes)
    mom = u0 if u0 is not None else [np.zeros(sh, dtype=np.float32) for sh in shapes]
    resid = r0 if r0 is not None else [np.zeros(sh, dtype=np.float32) for sh in shapes]
    n_cmp = n_exact = 0
    for t, grads in enumerate(grads_per_iter):
        sess.set_grad(grads)
        sess.set_residual(resid)
        sess.set_momentum(mom)
        sess.compress()
        torch.cuda.synchronize()
        res = sess.results()
        gpu_r = sess.unpack(sess.residual)
        gpu_u = sess.unpack(sess.momentum_buf)
        new_resid, new_mom = [], []
        for l in range(L):
            om = oracle.compress_layer_momentum(grads[l], mom[l], resid[l], m, p_list[l], alpha, ratios[l])
            o = om.layer
            tag = f"{name}[momentum,t={t},l={l},{shapes[l]},p={p_list[l]}]"
            gi, gv, gc, gn = res[l]
            exact = parity.check_layer(tag, shapes[l], p_list[l], o.k, o.tau, o.nsi, o.centres, o.idx,
                                       o.val, o.r_new, o.v, gi, gv, gc, gn, gpu_r[l])
            # the momentum: m*u + g where nothing was sent, +0 where something was (the GPU's own set)
            un, _ = oracle.momentum_accumulate(mom[l], grads[l], resid[l], m)
            want_u = un.reshape(-1).copy()
            want_u[gi] = 0.0
            assert np.array_equal(gpu_u[l].reshape(-1).view(np.uint32), want_u.view(np.uint32)), f"{tag}: momentum"
            if exact:
                assert np.array_equal(gpu_u[l].view(np.uint32), om.u_new.view(np.uint32)), f"{tag}: momentum vs oracle"
            n_cmp += 1
            n_exact += int(exact)
            new_resid.append(o.r_new)
            new_mom.append(om.u_new)
        resid, mom = new_resid, new_mom
    return n_cmp, n_exact


def test_momentum_ragged_shapes_three_iterations():
    shapes = RAGGED
    p_list = [1, 3, 5, 7, 3, 5, 3, 3, 7, 5, 3, 1, 3, 5]
    ratios = [1.0, 0.1, 0.1, 1.0, 0.02, 0.05, 0.02, 0.01, 0.3, 0.001, 0.5, 0.07, 0.0, 1.0]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 17, t, l) for l, sh in enumerate(shapes)] for t in range(3)]
    n, ex = run_and_check_momentum(shapes, p_list, 0.5, ratios, 0.9, its, "ragged")
    assert n == 3 * len(shapes) and ex >= n - 2


@pytest.mark.parametrize("m", [0.9, 0.0, 1.0, 0.5])
def test_momentum_resnet18_two_iterations(m):
    w = synth.config(1)
    its = [synth.gradients(w, t) for t in range(2)]
    rng = np.random.default_rng(5)
    u0 = [(rng.standard_normal(sh) * 1e-3).astype(np.float32) for sh in w.shapes]
    r0 = [(rng.standard_normal(sh) * 1e-3).astype(np.float32) for sh in w.shapes]
    n, ex = run_and_check_momentum(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, m, its, w.name, u0, r0)
    assert n == 2 * w.n_layers and ex >= n - 2


def test_momentum_zero_equals_the_plain_call():
    import torch
    from paper_2312_17530_amd.session import Session
    w = synth.scaled_down(synth.config(2), 256, 512)
    grads = synth.gradients(w, 0)
    a = Session(w.shapes, w.p, w.alpha, w.ratios)
    b = Session(w.shapes, w.p, w.alpha, w.ratios, momentum=0.0)
    for sess in (a, b):
        sess.set_grad(grads)
        sess.compress()
    torch.cuda.synchronize()
    assert torch.equal(a.out_counts, b.out_counts)
    assert torch.equal(a.residual.view(torch.int32), b.residual.view(torch.int32))
    for (i1, v1, c1, n1), (i2, v2, c2, n2) in zip(a.results(), b.results()):
        assert np.array_equal(i1, i2) and np.array_equal(v1.view(np.uint32), v2.view(np.uint32)) and np.array_equal(c1, c2)


def test_momentum_refuses_overlapping_arenas():
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import Session
    sess = Session([(64, 64)], 3, 0.5, [0.1], momentum=0.9)
    args = dict(out_idx=sess.out_idx, out_val=sess.out_val, out_counts=sess.out_counts, workspace=sess.workspace)
    for bad in ((sess.grad, sess.momentum_buf, sess.momentum_buf, sess.residual, sess.residual_next),
                (sess.grad, sess.momentum_buf, sess.momentum_next, sess.residual, sess.residual),
                (sess.grad, sess.momentum_buf, sess.residual_next, sess.residual, sess.residual_next),
                (sess.grad, sess.momentum_buf, sess.grad, sess.residual, sess.residual_next)):
        with pytest.raises(binding.RsdgcError):
            binding.rsdgc_compress_momentum(sess.plan, bad[0], bad[1], bad[2], 0.9, bad[3], bad[4], **args)
    with pytest.raises(binding.RsdgcError):
        binding.rsdgc_compress_momentum(sess.plan, sess.grad, sess.momentum_buf, sess.momentum_next, 1.5,
                                        sess.residual, sess.residual_next, **args)
    torch.cuda.synchronize()


def _gpu_dynamic_ratios(shapes, weights, rho):
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import Session
    sess = Session(shapes, 3, 0.5, [0.01] * len(shapes))
    arena = torch.empty_like(sess.grad)
    # the padding between layers holds huge values: it must not count
    host = np.full(sess.plan.total_elems, 1e30, dtype=np.float32)
    for a, off, sz in zip(weights, sess.offsets, sess.sizes):
        host[off:off + sz] = np.asarray(a, dtype=np.float32).reshape(-1)
    arena.copy_(torch.from_numpy(host))
    return sess, binding.rsdgc_dynamic_ratios(sess.plan, arena, rho, sess.workspace)


@pytest.mark.parametrize("rho", [0.0, 0.001, 0.02, 0.3, 0.97, 1.0])
def test_dynamic_ratios_match_the_oracle(rho):
    """Eqs. 3-5 on the GPU (radix select of |w| over all layers) against the oracle's full sort."""
    rng = np.random.default_rng(41)
    shapes = RAGGED + [(300, 700), (129, 64)]
    weights = [(rng.standard_normal(sh) * 10.0 ** rng.uniform(-2, 0)).astype(np.float32) for sh in shapes]
    weights[3][:] = 0.0                                # a dead layer
    weights[5][:] = np.float32(-0.125)                 # a layer of equal weights (ties inside one layer)
    weights[7][:] = np.float32(0.125)                  # ... and the same |w| in a later layer (ties across layers)
    _, got = _gpu_dynamic_ratios(shapes, weights, rho)
    want = oracle.dynamic_ratios(weights, rho)
    assert got == want


def test_dynamic_ratios_all_weights_equal_fall_back_to_layer_order():
    shapes = [(40, 50), (30, 30), (64, 128)]
    weights = [np.full(sh, 0.5 if l != 1 else -0.5, dtype=np.float32) for l, sh in enumerate(shapes)]
    for rho in (0.1, 0.2, 0.5, 0.9):
        _, got = _gpu_dynamic_ratios(shapes, weights, rho)
        assert got == oracle.dynamic_ratios(weights, rho)


def test_dynamic_ratios_feed_the_plan():
    """The per-epoch step of Algorithm 1 end to end: ratios from the weights, then one iteration."""
    import torch
    from paper_2312_17530_amd import binding
    w = synth.scaled_down(synth.config(2), 256, 512)
    rng = np.random.default_rng(43)
    weights = [(rng.standard_normal(sh) * np.sqrt(2.0 / sh[1])).astype(np.float32) for sh in w.shapes]
    sess, ratios = _gpu_dynamic_ratios(w.shapes, weights, 0.02)
    assert ratios == oracle.dynamic_ratios(weights, 0.02)
    sess.set_ratios(ratios)                            # (output buffers grow with the new capacities)
    grads = synth.gradients(w, 0)
    sess.set_grad(grads)
    sess.compress()
    torch.cuda.synchronize()
    res = sess.results()
    gpu_r = sess.unpack(sess.residual)
    for l, sh in enumerate(w.shapes):
        o = oracle.compress_layer(grads[l], np.zeros(sh, np.float32), w.p, w.alpha, ratios[l])
        gi, gv, gc, gn = res[l]
        assert sess.plan.layer_k(l) == o.k
        parity.check_layer(f"dynamic[l={l}]", sh, w.p, o.k, o.tau, o.nsi, o.centres, o.idx, o.val, o.r_new,
                           o.v, gi, gv, gc, gn, gpu_r[l])


def test_apply_messages_of_three_nodes_matches_the_oracle():
    """Eq. 12, third line: three nodes compress their own gradients (one GPU plays all three in
    turn); the receiving side sums their messages in order and steps the weights.  Two rounds, so
    the second one runs on the accumulator the first one left behind."""
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import Session
    shapes = [(1, 40), (33, 129), (200, 45), (64, 256), (300, 700), (7, 1000)]
    p_list = [3, 3, 5, 3, 3, 7]
    ratios = [0.5, 0.05, 0.1, 0.2, 0.02, 0.3]
    sess = Session(shapes, 3, 0.5, ratios, p_list)
    rng = np.random.default_rng(61)
    weights = [rng.standard_normal(sh).astype(np.float32) for sh in shapes]
    w_dev = torch.empty_like(sess.grad)
    sess.pack(weights, w_dev)
    eta = 0.05
    for rnd in range(2):
        msgs_dev, msgs_host = [], []
        for node in range(3):
            grads = [synth.layer_gradient(sh, 1e-2, 70 + node, rnd, l) for l, sh in enumerate(shapes)]
            sess.set_grad(grads)
            sess.residual.zero_()
            sess.compress()
            torch.cuda.synchronize()
            msgs_dev.append((sess.out_idx.clone(), sess.out_val.clone(), sess.out_counts.clone()))
            msgs_host.append([(i.copy(), v.copy()) for i, v, _, _ in sess.results()])
        binding.rsdgc_apply(sess.plan, msgs_dev, w_dev, eta, sess.workspace)
        torch.cuda.synchronize()
        got = sess.unpack(w_dev)
        for l, sh in enumerate(shapes):
            want = oracle.apply_messages(weights[l], [m[l] for m in msgs_host], eta)
            assert np.array_equal(got[l].view(np.uint32), want.view(np.uint32)), (rnd, l)
        weights = got


def run_and_check_blocks(shapes, p_list, alpha, ratios, grads_per_iter, name, in_place=False, work_feed=0,
                         m=None, u0=None):
    """The block reading on GPU and oracle from identical state; returns (compared, exact).
    With m: Eq. 12's momentum carried beside the residual (u0: momentum before the first call)."""
    import torch
    from paper_2312_17530_amd.session import BlockSession
    sess = BlockSession(shapes, p_list[0], alpha, ratios, p_list, in_place=in_place, work_feed=work_feed,
                        momentum=m)
    resid = [np.zeros(sh, dtype=np.float32) for sh in shapes]
    mom = None if m is None else (u0 if u0 is not None else [np.zeros(sh, dtype=np.float32) for sh in shapes])
    n_cmp = n_exact = 0
    for t, grads in enumerate(grads_per_iter):
        sess.set_grad(grads)
        sess.set_residual(resid)
        if m is not None:
            sess.set_momentum(mom)
        sess.compress()
        torch.cuda.synchronize()
        res = sess.results()
        gpu_r = sess.unpack(sess.residual)
        gpu_u = sess.unpack(sess.momentum_buf) if m is not None else None
        dense = sess.unpack(sess.decompress(accumulate=False))
        new_resid, new_mom = [], []
        for l, sh in enumerate(shapes):
            p = p_list[l]
            if m is None:
                o = oracle.compress_layer_blocks(grads[l], resid[l], p, alpha, ratios[l])
            else:
                om = oracle.compress_layer_blocks_momentum(grads[l], mom[l], resid[l], m, p, alpha, ratios[l])
                o = om.layer
            tag = f"{name}[blocks,t={t},l={l},{sh},p={p},m={m}]"
            gb, gv = res[l]
            assert sess.plan.layer_k(l) == o.k and len(gb) == o.k, tag
            assert np.all(np.diff(gb.astype(np.int64)) > 0), tag
            # ranking: every block clearly above the threshold is kept, none clearly below
            s = o.nsi.ravel().astype(np.float64)
            kept = np.zeros(s.size, dtype=bool)
            kept[gb] = True
            if 0 < o.k < s.size:
                tau = float(o.tau)
                assert not np.any(~kept & (s > tau * (1 + parity.EPS))), tag
                assert not np.any(kept & (s < tau * (1 - parity.EPS))), tag
            # wire format and residual follow from the GPU's own kept set, bit for bit
            R, C = sh
            BC = -(-C // p)
            v = o.v
            want_r = v.copy()
            want_val = np.zeros(len(gb) * p * p, dtype=np.float32)
            for j, b in enumerate(gb):
                bx, by = divmod(int(b), BC)
                x1, y1 = min(R, bx * p + p), min(C, by * p + p)
                blk = np.zeros((p, p), dtype=np.float32)
                blk[:x1 - bx * p, :y1 - by * p] = v[bx * p:x1, by * p:y1]
                want_val[j * p * p:(j + 1) * p * p] = blk.ravel()
                want_r[bx * p:x1, by * p:y1] = 0.0
            assert np.array_equal(gv.view(np.uint32), want_val.view(np.uint32)), f"{tag}: values"
            assert np.array_equal(gpu_r[l].view(np.uint32), want_r.view(np.uint32)), f"{tag}: residual"
            assert np.array_equal((dense[l] + gpu_r[l]).view(np.uint32), v.view(np.uint32)) or \
                np.array_equal(dense[l] + gpu_r[l], v), f"{tag}: decompress"
            if m is not None:
                # u_new = m*u + g in two roundings, +0 on the slots of the GPU's own kept blocks
                want_u = np.float32(m) * mom[l] + grads[l]
                want_u[want_r.view(np.uint32) != v.view(np.uint32)] = 0.0      # (slots the residual cleared)
                for b in gb:
                    bx, by = divmod(int(b), BC)
                    want_u[bx * p:bx * p + p, by * p:by * p + p] = 0.0
                assert np.array_equal(gpu_u[l].view(np.uint32), want_u.view(np.uint32)), f"{tag}: momentum"
            exact = np.array_equal(gb, o.blocks)
            if exact:
                assert np.array_equal(gv.view(np.uint32), o.val.view(np.uint32)), tag
                assert np.array_equal(gpu_r[l].view(np.uint32), o.r_new.view(np.uint32)), tag
                if m is not None:
                    assert np.array_equal(gpu_u[l].view(np.uint32), om.u_new.view(np.uint32)), tag
            n_cmp += 1
            n_exact += int(exact)
            new_resid.append(o.r_new)
            if m is not None:
                new_mom.append(om.u_new)
        resid = new_resid
        mom = new_mom
    return n_cmp, n_exact


def test_blocks_ragged_shapes_mixed_p_two_iterations(in_place):
    shapes = RAGGED + [(300, 700), (512, 1152)]
    p_list = [1, 3, 5, 7, 3, 5, 3, 3, 7, 5, 3, 1, 3, 5, 3, 3]
    ratios = [1.0, 0.1, 0.1, 1.0, 0.02, 0.05, 0.02, 0.01, 0.3, 0.001, 0.5, 0.07, 0.0, 1.0, 0.02, 0.01]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 19, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    n, ex = run_and_check_blocks(shapes, p_list, 0.5, ratios, its, "ragged", in_place=in_place)
    assert n == 2 * len(shapes) and ex >= n - 2


@pytest.mark.parametrize("m", [0.9, 0.0, 1.0])
def test_blocks_momentum_ragged_shapes_mixed_p_three_iterations(m, in_place):
    """Eq. 12 in full under the block reading: u and r carried over three iterations from a
    non-zero momentum, every neighbourhood side, ragged shapes, both arena forms."""
    shapes = RAGGED + [(300, 700), (512, 1152)]
    p_list = [1, 3, 5, 7, 3, 5, 3, 3, 7, 5, 3, 1, 3, 5, 3, 3]
    ratios = [1.0, 0.1, 0.1, 1.0, 0.02, 0.05, 0.02, 0.01, 0.3, 0.001, 0.5, 0.07, 0.0, 1.0, 0.02, 0.01]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 23, t, l) for l, sh in enumerate(shapes)] for t in range(3)]
    u0 = [synth.layer_gradient(sh, 2e-3, 24, 0, l) for l, sh in enumerate(shapes)]
    n, ex = run_and_check_blocks(shapes, p_list, 0.5, ratios, its, "ragged_momentum", in_place=in_place, m=m, u0=u0)
    assert n == 3 * len(shapes) and ex >= n - 3


def test_blocks_momentum_resnet18_shapes_with_the_work_feed():
    w = synth.scaled_down(synth.config(1), 256, 1024)
    its = [synth.gradients(w, t) for t in range(2)]
    for feed in (FEED_AUTO, FEED_ON):
        n, ex = run_and_check_blocks(w.shapes, [w.p] * len(w.shapes), w.alpha, w.ratios, its, "resnet18_momentum",
                                     m=0.9, work_feed=feed)
        assert ex >= n - 2


def test_blocks_momentum_zero_gives_the_plain_block_message_and_refuses_overlapping_arenas():
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import BlockSession
    shapes, ratios = [(64, 100), (40, 52), (31, 29)], [0.1, 0.2, 0.1]
    grads = [synth.layer_gradient(sh, 1e-2, 86, 0, l) for l, sh in enumerate(shapes)]
    a = BlockSession(shapes, 3, 0.5, ratios)
    b = BlockSession(shapes, 3, 0.5, ratios, momentum=0.0)
    for s in (a, b):
        s.set_grad(grads)
    b.set_momentum([synth.layer_gradient(sh, 1.0, 87, 0, l) for l, sh in enumerate(shapes)])
    a.compress()
    b.compress()
    for (b1, v1), (b2, v2) in zip(a.results(), b.results()):
        assert np.array_equal(b1, b2) and np.array_equal(v1.view(np.uint32), v2.view(np.uint32))
    assert torch.equal(a.residual, b.residual)
    # overlapping arenas (other than an output on its own input) are refused before any launch
    s = b
    bad = [dict(momentum_out=s.grad), dict(momentum_out=s.residual), dict(residual_out=s.momentum_buf),
           dict(momentum=s.residual_next), dict(m=1.5), dict(m=float("nan"))]
    for change in bad:
        args = dict(grad=s.grad, momentum=s.momentum_buf, momentum_out=s.momentum_next, m=0.5,
                    residual=s.residual, residual_out=s.residual_next)
        args.update(change)
        with pytest.raises(binding.RsdgcError):
            binding.rsdgc_compress_blocks_momentum(s.plan, args["grad"], args["momentum"], args["momentum_out"],
                                                   args["m"], args["residual"], args["residual_out"],
                                                   s.out_blocks, s.out_val, s.out_counts, s.workspace)


def test_blocks_degenerate_inputs_follow_index_tie_break():
    shapes = [(40, 70), (64, 128), (33, 40), (16, 300)]
    zeros = np.zeros(shapes[0], dtype=np.float32)
    const = np.full(shapes[1], -0.375, dtype=np.float32)
    xs, ys = np.meshgrid(np.arange(33), np.arange(40), indexing="ij")
    checker = np.where((xs + ys) % 2 == 0, 0.5, -0.5).astype(np.float32)
    ints = np.random.default_rng(98).integers(-3, 4, size=shapes[3]).astype(np.float32)
    grads = [zeros, const, checker, ints]
    for p in (3, 5, 1):
        n, ex = run_and_check_blocks(shapes, [p] * 4, 0.5, [0.3, 0.2, 0.1, 0.15], [grads, grads], f"degenerate(p={p})")
        assert ex == n, "exact ties must resolve exactly like the oracle (lower block index wins)"


def test_blocks_large_layers_with_masses_of_exact_ties():
    """The block reading on layers of about a million elements whose block scores are all equal
    or take few values: the threshold bucket holds most of the grid, far more than the small
    second list, so the last digits come from the bucket list itself."""
    shapes = [(1024, 1024), (768, 1536), (1000, 1100), (600, 2048)]
    rng = np.random.default_rng(4243)
    zeros = np.zeros(shapes[0], dtype=np.float32)
    const = np.full(shapes[1], 0.0625, dtype=np.float32)
    ints = rng.integers(-2, 3, size=shapes[2]).astype(np.float32)
    noise = (rng.standard_normal(shapes[3]) * 1e-3).astype(np.float32)
    grads = [zeros, const, ints, noise]
    for p in (3, 1):
        n, ex = run_and_check_blocks(shapes, [p] * 4, 0.5, [0.05, 0.02, 0.03, 0.02], [grads, grads],
                                     f"large_ties(p={p})")
        assert n == 8 and ex >= 7


def test_blocks_receiving_side_skips_what_a_malformed_message_names():
    """As for element messages: a block index at or beyond the layer's block count is skipped,
    a count beyond k_l is read as k_l, a negative one as zero; the arena's padding is not written."""
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import BlockSession
    shapes, ratios, p = [(64, 100), (40, 50), (31, 29)], [0.1, 0.2, 0.1], 3
    sess = BlockSession(shapes, p, 0.5, ratios)
    sess.set_grad([synth.layer_gradient(sh, 1e-2, 85, 0, l) for l, sh in enumerate(shapes)])
    sess.compress()
    torch.cuda.synchronize()
    plan = sess.plan
    n_blocks = [-(-r // p) * -(-c // p) for r, c in shapes]
    ks = [plan.layer_k(l) for l in range(3)]
    counts = sess.out_counts.cpu().numpy().copy()
    blocks = sess.out_blocks.cpu().numpy().view(np.uint32).copy()
    val = sess.out_val.cpu().numpy().copy()
    assert list(counts) == ks and ks[0] >= 3
    b0 = plan.centre_offset(0)
    picks = np.array([0, ks[0] // 2, ks[0] - 1])
    blocks[b0 + picks] = np.array([n_blocks[0], 0xffffffff, n_blocks[0] + 77], dtype=np.uint32)
    counts[1] = ks[1] + 100000
    counts[2] = -1
    dev = sess.grad.device
    dense = torch.full_like(sess.grad, 7.0)
    binding.rsdgc_decompress_blocks(plan, torch.from_numpy(blocks.view(np.int32)).to(dev),
                                    torch.from_numpy(val).to(dev), torch.from_numpy(counts.astype(np.int32)).to(dev),
                                    dense, False, sess.workspace)
    torch.cuda.synchronize()
    want = np.full(dense.numel(), 7.0, dtype=np.float32)
    for l, (R, C) in enumerate(shapes):
        n = min(max(int(counts[l]), 0), ks[l])
        bo, vo = plan.centre_offset(l), plan.out_offset(l)
        b = blocks[bo:bo + n]
        v = val[vo:vo + n * p * p].reshape(n, p * p)
        ok = b < n_blocks[l]
        o = plan.layer_offset(l)
        want[o:o + R * C] = oracle.decompress_blocks(b[ok], v[ok].reshape(-1), R, C, p).reshape(-1)
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_blocks_apply_messages_of_three_nodes_matches_the_oracle():
    """Eq. 12, third line, with block messages: three nodes compress their own gradients in the
    block reading; the receiving side sums the messages in order and steps the weights.  Two
    rounds, so the second runs on the accumulator the first left behind; a tampered message at
    the end (block index beyond the grid, counts beyond k_l and negative) must be skipped."""
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import BlockSession
    shapes = [(1, 40), (33, 129), (200, 45), (64, 256), (300, 700), (7, 1000)]
    p_list = [3, 3, 5, 3, 1, 7]
    ratios = [0.5, 0.05, 0.1, 0.2, 0.02, 0.3]
    sess = BlockSession(shapes, 3, 0.5, ratios, p_list)
    rng = np.random.default_rng(62)
    weights = [rng.standard_normal(sh).astype(np.float32) for sh in shapes]
    w_dev = torch.full_like(sess.grad, 3.0)
    for l, w in enumerate(weights):
        o = sess.plan.layer_offset(l)
        w_dev[o:o + w.size] = torch.from_numpy(w.reshape(-1)).to(w_dev.device)
    eta = 0.05
    for rnd in range(2):
        msgs_dev, msgs_host = [], []
        for node in range(3):
            sess.set_grad([synth.layer_gradient(sh, 1e-2, 90 + node, rnd, l) for l, sh in enumerate(shapes)])
            sess.residual.zero_()
            sess.compress()
            torch.cuda.synchronize()
            msgs_dev.append((sess.out_blocks.clone(), sess.out_val.clone(), sess.out_counts.clone()))
            msgs_host.append(sess.results())
        binding.rsdgc_apply_blocks(sess.plan, msgs_dev, w_dev, eta, sess.workspace)
        torch.cuda.synchronize()
        arena = w_dev.cpu().numpy()
        got = []
        for l, (R, C) in enumerate(shapes):
            o = sess.plan.layer_offset(l)
            got.append(arena[o:o + R * C].reshape(R, C).copy())
            want = oracle.apply_block_messages(weights[l], [m[l] for m in msgs_host], p_list[l], eta)
            assert np.array_equal(got[l].view(np.uint32), want.view(np.uint32)), (rnd, l)
        weights = got
    # a tampered copy of the last message: nothing it names wrongly is followed
    blocks, val, counts = (t.clone() for t in msgs_dev[-1])
    n_blocks = [-(-r // p) * -(-c // p) for (r, c), p in zip(shapes, p_list)]
    ks = [sess.plan.layer_k(l) for l in range(len(shapes))]
    host_blocks = blocks.cpu().numpy().view(np.uint32).copy()
    host_counts = counts.cpu().numpy().copy()
    l_bad = 4
    host_blocks[sess.plan.centre_offset(l_bad)] = n_blocks[l_bad] + 3
    host_counts[1] = ks[1] + 1000
    host_counts[2] = -7
    blocks.copy_(torch.from_numpy(host_blocks.view(np.int32)))
    counts.copy_(torch.from_numpy(host_counts))
    before = w_dev.cpu().numpy().copy()
    binding.rsdgc_apply_blocks(sess.plan, [(blocks, val, counts)], w_dev, eta, sess.workspace)
    torch.cuda.synchronize()
    arena = w_dev.cpu().numpy()
    last = msgs_host[-1]
    want_arena = before.copy()
    for l, (R, C) in enumerate(shapes):
        b, v = last[l]
        pp = p_list[l] ** 2
        if l == 2:
            b, v = b[:0], v[:0]
        if l == l_bad:
            b, v = b[1:], v[pp:]
        o = sess.plan.layer_offset(l)
        want_arena[o:o + R * C] = oracle.apply_block_messages(weights[l], [(b, v)], p_list[l], eta).reshape(-1)
    assert np.array_equal(arena.view(np.uint32), want_arena.view(np.uint32))     # padding (3.0) included


def test_blocks_resnet18_shapes():
    w = synth.config(1)
    its = [synth.gradients(w, t) for t in range(2)]
    n, ex = run_and_check_blocks(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, its, w.name)
    assert n == 2 * w.n_layers and ex >= n - 2


@pytest.mark.parametrize("in_place", [False, True], ids=["two_arenas", "in_place"])
def test_blocks_with_the_work_feed_forced_on(in_place):
    """The block-score pass with its tiles handed out through the work counters (by default only
    for launches of many thousand tiles): ragged shapes with mixed p, and ResNet-18."""
    shapes = RAGGED
    p_list = [1, 3, 5, 7, 3, 5, 3, 3, 7, 5, 3, 1, 3, 5]
    ratios = [1.0, 0.1, 0.1, 1.0, 0.02, 0.05, 0.02, 0.01, 0.3, 0.001, 0.5, 0.07, 0.0, 1.0]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 23, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    n, ex = run_and_check_blocks(shapes, p_list, 0.5, ratios, its, "blocks/feed/ragged", in_place=in_place, work_feed=2)
    assert n == 2 * len(shapes) and ex >= n - 2
    w = synth.config(1)
    its = [synth.gradients(w, t) for t in range(2)]
    n, ex = run_and_check_blocks(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, its, "blocks/feed/" + w.name,
                                 in_place=in_place, work_feed=2)
    assert n == 2 * w.n_layers and ex >= n - 2


def test_block_plan_and_element_plan_do_not_mix():
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import BlockSession, Session
    b = BlockSession([(64, 64)], 3, 0.5, [0.1])
    e = Session([(64, 64)], 3, 0.5, [0.1])
    with pytest.raises(binding.RsdgcError):
        binding.rsdgc_compress(b.plan, b.grad, b.residual, b.residual_next, b.out_blocks, b.out_val,
                               b.out_counts, b.workspace)
    with pytest.raises(binding.RsdgcError):
        binding.rsdgc_compress_blocks(e.plan, e.grad, e.residual, e.residual_next, e.out_idx, e.out_val,
                                      e.out_counts, e.workspace)
    torch.cuda.synchronize()


def test_config0_single_layer_512(in_place):
    w = synth.config(0)
    n, ex = run_and_check(w.shapes, [w.p], w.alpha, w.ratios, [synth.gradients(w, 0)], w.name,
                          in_place=in_place)
    assert n == 1 and ex == 1


RAGGED = [(1, 1), (1, 40), (40, 1), (2, 2), (33, 129), (45, 61), (64, 27), (200, 45), (31, 257),
          (100, 300), (32, 128), (64, 256), (65, 130), (7, 1000)]


@pytest.mark.parametrize("alpha", [0.5, 0.0, 1.0, 0.25])
def test_ragged_shapes_mixed_p_two_iterations(alpha, in_place):
    rng = np.random.default_rng(int(alpha * 100) + 7)
    shapes = RAGGED
    p_list = [1, 3, 5, 7, 3, 5, 3, 3, 7, 5, 3, 1, 3, 5]
    ratios = [1.0, 0.1, 0.1, 1.0, 0.02, 0.05, 0.02, 0.01, 0.3, 0.001, 0.5, 0.07, 0.0, 1.0]
    its = []
    for t in range(2):
        its.append([synth.layer_gradient(sh, 1e-3 * (l + 1), 11, t, l) for l, sh in enumerate(shapes)])
    n, ex = run_and_check(shapes, p_list, alpha, ratios, its, "ragged", in_place=in_place)
    assert n == 2 * len(shapes)
    assert ex >= n - 2          # the tolerance band is allowed, but should hardly ever be needed


@pytest.mark.parametrize("path", [AUTO, FULL_MAP])
def test_long_vectors_and_narrow_layers(path):
    """One-dimensional parameters given as a column or as a row, and tall layers of a few columns:
    three iterations against the oracle on each ranking path (a column is handled as a row inside
    the library; the flat indices are the same), and a workspace that stays in proportion -- the
    tile slots of such layers are as short as their tiles."""
    shapes = [(50000, 1), (1, 50000), (30000, 7), (3, 40000), (2500, 20)]
    p_list = [3, 3, 5, 3, 7]
    ratios = [0.02, 0.02, 0.01, 0.05, 0.02]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 23, t, l) for l, sh in enumerate(shapes)] for t in range(3)]
    n, ex = run_and_check(shapes, p_list, 0.5, ratios, its, "vectors", path=path)
    assert n == 3 * len(shapes) and ex >= n - 2
    G = sum(r * c for r, c in shapes)
    ws = _session(shapes, 3, 0.5, ratios, p_list, path=path).plan.workspace_bytes
    assert ws <= 20 * G + (4 << 20), ws
    # the column and the row of the same values give the same pairs
    g = synth.layer_gradient((50000, 1), 1e-3, 23, 0, 0)
    col = _session([(50000, 1)], 3, 0.5, [0.02], path=path)
    row = _session([(1, 50000)], 3, 0.5, [0.02], path=path)
    col.set_grad([g])
    row.set_grad([g.reshape(1, -1)])
    col.compress()
    row.compress()
    (ci, cv, cc, cn), (ri, rv, rc, rn) = col.results()[0], row.results()[0]
    assert cn == rn and np.array_equal(cc, rc) and np.array_equal(ci, ri)
    assert np.array_equal(cv.view(np.uint32), rv.view(np.uint32))


def _draw_small(seed):
    """A seeded small plan: 1-5 layers of up to 90 x 400 elements, a neighbourhood side per
    layer, keep ratios from 0 to 1, a mix from 0 to 1, two iterations of ordinary noise or of
    inputs with five distinct values (scores tie in masses)."""
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 6))
    shapes = [(int(rng.integers(1, 91)), int(rng.integers(1, 401))) for _ in range(L)]
    p_list = [int(rng.choice([1, 3, 5, 7])) for _ in range(L)]
    ratios = [float(rng.choice([0.0, 0.003, 0.02, 0.1, 0.3, 0.8, 1.0])) for _ in range(L)]
    alpha = float(rng.choice([0.0, 0.25, 0.5, 1.0]))
    its = []
    for t in range(2):
        grads = []
        for sh in shapes:
            if rng.random() < 0.3:
                grads.append(rng.integers(-2, 3, size=sh).astype(np.float32) * np.float32(0.125))
            else:
                grads.append((rng.standard_normal(sh) * 10.0 ** rng.uniform(-4, 0)).astype(np.float32))
        its.append(grads)
    return shapes, p_list, ratios, alpha, its


def test_drawn_small_configurations(in_place):
    """Twenty seeded draws (see _draw_small), two iterations carrying the residual."""
    n_total = ex_total = 0
    for seed in range(20):
        shapes, p_list, ratios, alpha, its = _draw_small(seed)
        n, ex = run_and_check(shapes, p_list, alpha, ratios, its, f"drawn{seed}", in_place=in_place)
        n_total += n
        ex_total += ex
    assert ex_total >= n_total - 2


def test_drawn_small_configurations_with_momentum_and_in_the_block_reading():
    """The same draws through rsdgc_compress_momentum (m drawn too) and rsdgc_compress_blocks."""
    n_total = ex_total = 0
    for seed in range(20, 32):
        shapes, p_list, ratios, alpha, its = _draw_small(seed)
        m = [0.9, 0.5, 0.0, 1.0][seed % 4]
        n, ex = run_and_check_momentum(shapes, p_list, alpha, ratios, m, its, f"drawn{seed}")
        n_total += n
        ex_total += ex
        n, ex = run_and_check_blocks(shapes, p_list, alpha, ratios, its, f"drawn{seed}", in_place=bool(seed % 2))
        n_total += n
        ex_total += ex
    assert ex_total >= n_total - 3


def test_drawn_large_configurations(in_place):
    """Six seeded draws of 2-3 layers of 0.1 to 4 million elements with odd row lengths: most take
    the candidate path (with and without the work feed), some the full map; sides, ratios, mixes
    and the noise scale (down to 1e-6, up to 1e3) are drawn per layer."""
    n_total = ex_total = 0
    for seed in range(6):
        rng = np.random.default_rng(2000 + seed)
        L = int(rng.integers(2, 4))
        shapes = [(int(rng.integers(300, 1501)), int(rng.integers(300, 3001))) for _ in range(L)]
        p_list = [int(rng.choice([1, 3, 3, 5, 7])) for _ in range(L)]
        ratios = [float(rng.choice([0.003, 0.02, 0.05, 0.2])) for _ in range(L)]
        alpha = float(rng.choice([0.0, 0.25, 0.5, 0.5, 1.0]))
        its = [[synth.layer_gradient(sh, 10.0 ** rng.uniform(-6, 3), 2000 + seed, t, l) for l, sh in enumerate(shapes)]
               for t in range(2)]
        feed = FEED_ON if seed % 2 else FEED_AUTO
        n, ex = run_and_check(shapes, p_list, alpha, ratios, its, f"drawn_large{seed}", in_place=in_place,
                              work_feed=feed)
        n_total += n
        ex_total += ex
    assert ex_total >= n_total - 2


def test_subnormal_and_huge_magnitudes(in_place):
    """Gradients in float32's subnormal range (their scores are subnormal floats too, and must
    not be flushed to zero: the ranking would collapse into index order) and near its upper end
    (squares far beyond float32, within double)."""
    shapes = [(40, 300), (64, 129), (700, 1100)]
    rng = np.random.default_rng(77)
    for scale in (1e-41, 3e-39, 1e18):
        its = [[(rng.standard_normal(sh) * scale).astype(np.float32) for sh in shapes] for _ in range(2)]
        assert all(np.isfinite(g).all() and np.count_nonzero(g) > g.size // 2 for g in its[0])
        n, ex = run_and_check(shapes, [3, 5, 3], 0.5, [0.05, 0.1, 0.02], its, f"magnitude{scale}", in_place=in_place)
        assert n == 6 and ex >= 5


def _near_constant_layers(shapes, seed):
    """Inputs on which a one-pass variance (sum of squares minus squared sum) loses all its
    digits: values a few float32 ulps apart (c (1 + j 2^-23), small j), a ramp on a large offset,
    small noise on a large offset, and a constant with a few single-ulp dents."""
    rng = np.random.default_rng(seed)
    out = []
    for i, sh in enumerate(shapes):
        kind = i % 4
        if kind == 0:
            c = np.float32(0.7310791)
            bits = np.full(sh, c.view(np.uint32), dtype=np.uint32) + rng.integers(0, 4, size=sh).astype(np.uint32)
            g = bits.view(np.float32)
        elif kind == 1:
            g = np.float32(1000.0) + np.float32(1e-3) * np.arange(sh[0] * sh[1], dtype=np.float32).reshape(sh)
        elif kind == 2:
            g = (np.float32(-5.0) + np.float32(1e-6) * rng.standard_normal(sh)).astype(np.float32)
        else:
            c = np.float32(3.1415927)
            bits = np.full(sh, c.view(np.uint32), dtype=np.uint32)
            dents = rng.random(sh) < 0.01
            bits[dents] += np.uint32(1)
            g = bits.view(np.float32)
        out.append(np.ascontiguousarray(g, dtype=np.float32))
    return out


@pytest.mark.parametrize("alpha", [0.0, 0.5])
def test_near_constant_windows_where_a_one_pass_variance_cancels(alpha):
    """Eq. 10 on windows whose standard deviation is 1e-7 of their mean.  With alpha = 0 the score
    is that standard deviation alone, so any loss of digits in the variance shows at once: the
    scores must still agree with the oracle's two-pass value to 1e-5 relative (no absolute floor)."""
    shapes = [(40, 70), (33, 130), (64, 27), (50, 300), (17, 23), (90, 45), (128, 256), (1, 500)]
    grads = _near_constant_layers(shapes, 31)
    for p in (3, 5, 7):
        ratios = [0.1, 0.05, 0.3, 0.02, 0.5, 0.1, 0.05, 0.2]
        n, ex = run_and_check(shapes, [p] * len(shapes), alpha, ratios, [grads, grads],
                              f"near_constant(p={p},alpha={alpha})")
        assert n == 2 * len(shapes) and ex >= n - 2
    n, ex = run_and_check_blocks(shapes, [3, 5, 7, 3, 5, 7, 3, 5], alpha, [0.1] * len(shapes), [grads, grads],
                                 f"near_constant_blocks(alpha={alpha})")
    assert ex >= n - 2


@pytest.mark.parametrize("p", [3, 5, 7])
def test_near_constant_windows_at_a_million_elements(p, in_place):
    """The same at sizes that take the main (candidate) pass: alpha = 0, layers of a million elements."""
    shapes = [(1024, 1024), (600, 2048), (768, 1536), (1000, 1100)]
    grads = _near_constant_layers(shapes, 32 + p)
    n, ex = run_and_check(shapes, [p] * 4, 0.0, [0.02, 0.01, 0.03, 0.02], [grads, grads],
                          f"near_constant_large(p={p})", in_place=in_place)
    assert n == 8 and ex >= 6


def test_degenerate_inputs_follow_index_tie_break():
    shapes = [(40, 70), (64, 128), (50, 50), (33, 40), (16, 300), (90, 45)]
    zeros = np.zeros(shapes[0], dtype=np.float32)
    const = np.full(shapes[1], -0.375, dtype=np.float32)
    impulse = np.zeros(shapes[2], dtype=np.float32)
    impulse[20, 31] = 3.0
    impulse[5, 5] = -3.0
    xs, ys = np.meshgrid(np.arange(33), np.arange(40), indexing="ij")
    checker = np.where((xs + ys) % 2 == 0, 0.5, -0.5).astype(np.float32)
    rng = np.random.default_rng(99)
    ints = rng.integers(-3, 4, size=shapes[4]).astype(np.float32)       # masses of exact ties
    ramp = (np.arange(90 * 45, dtype=np.float32).reshape(90, 45) * np.float32(1e-3) + np.float32(5.0))
    grads = [zeros, const, impulse, checker, ints, ramp]
    for p, alpha in [(3, 0.5), (5, 0.5), (3, 1.0), (3, 0.0), (1, 1.0)]:
        ratios = [0.3, 0.2, 0.05, 0.1, 0.15, 0.25]
        n, ex = run_and_check(shapes, [p] * len(shapes), alpha, ratios, [grads, grads],
                              f"degenerate(p={p},alpha={alpha})")
        assert ex == n, "exact ties must resolve exactly like the oracle (lower index wins)"


def test_large_layers_with_masses_of_exact_ties(in_place):
    """Layers large enough for the candidate path whose scores are all equal, or take a handful
    of values (a frozen layer's all-zero gradient is the everyday case): the candidate bound
    cannot separate anything, the layer falls back to the full map, its threshold bucket holds
    far more keys than the bucket list, and the last radix digits -- those of the index -- are
    found by streaming the score map.  The lower index must win exactly as in the oracle."""
    shapes = [(1024, 1024), (768, 1536), (1000, 1100), (600, 2048)]
    rng = np.random.default_rng(4242)
    zeros = np.zeros(shapes[0], dtype=np.float32)
    const = np.full(shapes[1], 0.0625, dtype=np.float32)
    ints = rng.integers(-2, 3, size=shapes[2]).astype(np.float32)
    noise = (rng.standard_normal(shapes[3]) * 1e-3).astype(np.float32)     # an ordinary layer beside them
    grads = [zeros, const, ints, noise]
    for p, ratios in [(3, [0.05, 0.02, 0.03, 0.02]), (5, [0.3, 0.01, 0.2, 0.05])]:
        n, ex = run_and_check(shapes, [p] * 4, 0.5, ratios, [grads, grads], f"large_ties(p={p})",
                              in_place=in_place)
        assert n == 8 and ex >= 7, "exact ties must resolve exactly like the oracle"
    if not in_place:        # the same fallback with Eq. 12's momentum: the full-map pass forms m*u + g again
        n, ex = run_and_check_momentum(shapes, [3] * 4, 0.5, [0.05, 0.02, 0.03, 0.02], 0.9, [grads, grads],
                                       "large_ties")
        assert n == 8 and ex >= 7


def test_large_layers_with_high_keep_ratios(in_place):
    """Keep ratios far above the benchmark's (up to 1, where Eq. 11 selects G/p^2 centres, and
    with p = 1 every element): the layers are ranked on the full map and the threshold bucket of
    an ordinary noise layer outgrows the bucket list."""
    shapes = [(1000, 1100), (600, 2048), (900, 1000)]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 43, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    for p_list, ratios in [([3, 3, 3], [1.0, 0.5, 0.25]), ([1, 1, 5], [1.0, 0.4, 1.0])]:
        n, ex = run_and_check(shapes, p_list, 0.5, ratios, its, f"high_ratio{p_list}", in_place=in_place)
        assert n == 6 and ex >= 5


@pytest.mark.parametrize("path", [AUTO, FULL_MAP])
def test_config1_resnet18_two_iterations(path, in_place):
    w = synth.config(1)
    its = [synth.gradients(w, t) for t in range(w.iterations)]
    n, ex = run_and_check(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, its, w.name, path=path,
                          in_place=in_place)
    assert n == 2 * w.n_layers
    assert ex >= n - 2


@pytest.mark.parametrize("path", [AUTO, FULL_MAP])
def test_config2_resnet50_dynamic_ratios(path):
    w = synth.config(2)
    its = [synth.gradients(w, 0)]
    n, ex = run_and_check(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, its, w.name, path=path)
    assert n == w.n_layers
    assert ex >= n - 2


def test_large_layers_with_rows_that_are_not_whole_mask_words(in_place):
    """Layers large enough for the candidate path whose row length is not a multiple of 32:
    their tiles share mask words, so marking goes through atomics instead of tile-owned words.
    A layer with C % 32 == 0 sits between them (tile-owned words)."""
    shapes = [(700, 1100), (1000, 2570), (640, 1536), (2100, 333)]
    p_list = [3, 5, 3, 7]
    ratios = [0.02, 0.01, 0.03, 0.05]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 31, t, l) for l, sh in enumerate(shapes)]
           for t in range(2)]
    from paper_2312_17530_amd import binding
    n, ex = run_and_check(shapes, p_list, 0.5, ratios, its, "large_unaligned", in_place=in_place)
    assert n == 2 * len(shapes) and ex >= n - 1
    sess = _session(shapes, 3, 0.5, ratios, p_list)
    sess.set_grad(its[0])
    sess.compress()
    paths = binding.rsdgc_last_paths(sess.plan, sess.workspace)
    assert paths[0] == 0 and paths[3] == 0, "expected the candidate path"


@pytest.mark.parametrize("path", [AUTO, FULL_MAP])
def test_wide_layers_whose_rows_span_many_chunks(path):
    """Rows of 65536 and 40000 elements: the 16 rows of a tile lie in sixteen different groups of
    chunks, further apart than the kernels that count kept elements as they mark them keep
    counters for in LDS (those go to the global counters one by one).  One aligned layer, one whose
    rows are no whole mask words; candidate path and full map."""
    shapes = [(40, 65536), (33, 40000), (64, 256)]
    ratios = [0.02, 0.03, 0.05]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 61, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    n, ex = run_and_check(shapes, [3, 5, 3], 0.5, ratios, its, "wide_rows", path=path)
    assert n == 6 and ex >= 5


@pytest.mark.parametrize("in_place", [False, True], ids=["two_arenas", "in_place"])
def test_work_feed_on_small_launches(in_place):
    """The main pass can hand out its tiles through per-XCD work counters; by default it does so
    only for launches of many thousand tiles.  Forced on here, so that the small cases meet it
    too: ragged shapes with mixed p (launches of a few tiles, most domains empty), large layers
    with unaligned rows, ResNet-18, the fallback inputs, and the momentum form."""
    shapes = RAGGED
    p_list = [1, 3, 5, 7, 3, 5, 3, 3, 7, 5, 3, 1, 3, 5]
    ratios = [1.0, 0.1, 0.1, 1.0, 0.02, 0.05, 0.02, 0.01, 0.3, 0.001, 0.5, 0.07, 0.0, 1.0]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 19, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    n, ex = run_and_check(shapes, p_list, 0.5, ratios, its, "feed/ragged", in_place=in_place, work_feed=FEED_ON)
    assert n == 2 * len(shapes) and ex >= n - 2
    shapes = [(700, 1100), (1000, 2570), (640, 1536), (2100, 333)]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 31, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    n, ex = run_and_check(shapes, [3, 1, 3, 3], 0.5, [0.02, 0.01, 0.03, 0.05], its, "feed/large_unaligned",
                          in_place=in_place, work_feed=FEED_ON)
    assert n == 2 * len(shapes) and ex >= n - 1
    # large layers with the wide neighbourhoods: their main pass rules centres out before the square root
    shapes = [(1500, 2100), (1200, 1800), (900, 2048)]
    its = [[synth.layer_gradient(sh, 1e-3 * (l + 1), 37, t, l) for l, sh in enumerate(shapes)] for t in range(2)]
    n, ex = run_and_check(shapes, [7, 5, 5], 0.5, [0.01, 0.02, 0.003], its, "feed/wide", in_place=in_place,
                          work_feed=FEED_ON)
    assert n == 2 * len(shapes) and ex >= n - 1
    for alpha in (0.0, 1.0):
        n, ex = run_and_check(shapes[1:], [5, 7], alpha, [0.02, 0.01], its[:1] and [[g for g in its[0][1:]]],
                              f"feed/wide/alpha{alpha}", in_place=in_place, work_feed=FEED_ON)
        assert n == 2 and ex >= 1
    w = synth.config(1)
    its = [synth.gradients(w, t) for t in range(2)]
    n, ex = run_and_check(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, its, "feed/" + w.name,
                          in_place=in_place, work_feed=FEED_ON)
    assert n == 2 * w.n_layers and ex >= n - 2
    if not in_place:
        n, ex = run_and_check_momentum(w.shapes, [w.p] * w.n_layers, w.alpha, w.ratios, 0.9, its,
                                       "feed/momentum/" + w.name, work_feed=FEED_ON)
        assert n == 2 * w.n_layers and ex >= n - 2


def _tile_is_sampled(t):
    """The library samples one tile in 16 (layers below 4096 tiles) by this hash of the tile's
    index inside its layer."""
    return ((t * 2654435761) & 0xFFFFFFFF) >> 28 == 0


def test_candidate_path_falls_back_when_its_bound_fails(in_place):
    """Large layers rank only the centres above a bound estimated from sampled tiles.  Inputs
    built to defeat that estimate must still give the oracle's result (through the full map)."""
    R, C = 512, 4608                      # 32 x 18 tiles of 16 x 256
    TR, TC = 16, 256                      # the library's NSI tile
    rng = np.random.default_rng(123)
    base = (rng.standard_normal((R, C)) * 1e-3).astype(np.float32)
    tiles_x = C // TC
    # (a) the sampled tiles carry far larger values than the rest: the bound comes out too high
    hot_sampled = base.copy()
    # (b) one region holds thousands of top-ranked centres: candidate slots overflow
    hot_tile = base.copy()
    hot_tile[64:96, 256:384] *= np.float32(50.0)
    n_sampled = 0
    for t in range((R // TR) * tiles_x):
        if _tile_is_sampled(t):
            n_sampled += 1
            tr, tc = divmod(t, tiles_x)
            hot_sampled[tr * TR:(tr + 1) * TR, tc * TC:(tc + 1) * TC] *= np.float32(30.0)
    assert n_sampled >= 8, "the layer must be large enough to take the candidate path"
    # (c) a well-behaved layer next to them keeps using the candidate path
    shapes = [(R, C), (R, C), (R, C)]
    grads = [hot_sampled, hot_tile, base]
    for ratios in ([0.3, 0.02, 0.02], [0.02, 0.2, 0.01]):
        for feed in (FEED_AUTO, FEED_ON):
            n, ex = run_and_check(shapes, [3, 3, 3], 0.5, ratios, [grads, grads], "fallback",
                                  in_place=in_place, work_feed=feed)
            assert n == 6 and ex >= 5


def test_candidate_bound_is_predicted_from_earlier_calls_and_recovers_from_failures():
    """The first calls of a large layer take a bound sampled from that call's scores (path 0); once
    two thresholds lie close together the bound is predicted from them (path 3) and no tile is
    sampled.  A call whose bound fails -- here an input with thousands of winners in one tile, and
    a gradient that suddenly shrinks so that the predicted bound lies above everything -- is redone
    through the full map within the call (path 1) and the layer goes back to sampled bounds for a
    few calls; it is never parked on the full map.  Every call gives the oracle's result."""
    import torch
    from paper_2312_17530_amd import binding
    R, C = 512, 4608
    rng = np.random.default_rng(124)
    base = (rng.standard_normal((R, C)) * 1e-3).astype(np.float32)
    hot_tile = base.copy()
    hot_tile[64:96, 256:384] *= np.float32(50.0)          # thousands of winners in one tile: slots overflow
    other = (rng.standard_normal((R, C)) * 1e-3).astype(np.float32)
    shapes, ratios = [(R, C), (R, C)], [0.02, 0.02]
    sess = _session(shapes, 3, 0.5, ratios)
    zero = [np.zeros((R, C), np.float32)] * 2

    def call(grads, tag):
        sess.set_grad(grads)
        sess.set_residual(zero)
        sess.compress()
        torch.cuda.synchronize()
        paths = binding.rsdgc_last_paths(sess.plan, sess.workspace)
        res = sess.results()
        gpu_r = sess.unpack(sess.residual)
        for l in range(2):
            o = oracle.compress_layer(grads[l], zero[l], 3, 0.5, ratios[l])
            gi, gv, gc, gn = res[l]
            assert parity.check_layer(f"{tag}[l={l},path={paths[l]}]", shapes[l], 3, o.k, o.tau, o.nsi, o.centres,
                                      o.idx, o.val, o.r_new, o.v, gi, gv, gc, gn, gpu_r[l])
        return list(paths)

    assert call([base, other], "first") == [0, 0]          # no history: sampled bounds
    assert call([base, other], "second") == [0, 0]         # one threshold is not a trend
    assert call([base, other], "third") == [3, 3]          # two equal thresholds: predicted
    assert call([hot_tile, other], "hot tile") == [1, 3]   # slots overflow: redone through the full map
    seen = [call([base, other], f"after failure {i}") for i in range(6)]
    assert all(p[1] == 3 for p in seen)
    assert all(p[0] in (0, 3) for p in seen), "a layer whose bound failed is not parked on the full map"
    assert seen[0][0] == 0 and seen[-1][0] == 3            # sampled for a few calls, then predicted again
    # the gradient shrinks tenfold from one call to the next: the predicted bound lies far too high
    small = [g * np.float32(0.1) for g in (base, other)]
    assert call(small, "shrunk") == [1, 1]
    # the call after a failed bound does not extend the jump into a trend: its bound is sampled or
    # taken from the last threshold alone, and holds
    assert all(p in (0, 3) for p in call(small, "shrunk again"))
    # and grows a hundredfold: the bound is far too low, every tile overflows -- or the sample decides
    big = [g * np.float32(10.0) for g in (base, other)]
    for i in range(8):
        paths = call(big if i % 2 == 0 else small, f"alternating {i}")
        assert all(p in (0, 1, 3) for p in paths)
    binding.rsdgc_plan_forget_workspace(sess.plan)         # a prepared-again workspace starts afresh
    assert call([base, other], "fresh workspace") == [0, 0]


def test_thirty_calls_from_a_zero_residual_hardly_ever_fall_back():
    """The benchmark's situation: the same workspace over many calls while the residual builds up
    from zero (the VGG-19 recipe on matrices clipped to 1024 x 4608, so that every large layer
    keeps its tile structure).  With the same gradient every call the threshold grows fast at
    first and ever more slowly later; with a fresh gradient every call it grows like a random
    walk.  At most one call of one layer may need the full map in either run."""
    import torch
    from paper_2312_17530_amd import binding
    w = synth.scaled_down(synth.config(3), 1024, 4608)
    for fresh in (False, True):
        sess = _session(w.shapes, w.p, w.alpha, w.ratios)
        g0 = synth.gradients(w, 0)
        sess.set_grad(g0)
        history = []
        for t in range(30):
            if fresh and t > 0:
                sess.set_grad(synth.gradients(w, t))
            sess.compress()
            torch.cuda.synchronize()
            history.append(binding.rsdgc_last_paths(sess.plan, sess.workspace))
        large = [l for l in range(w.n_layers) if any(h[l] in (0, 3) for h in history)]
        assert len(large) >= 8
        fallbacks = [(t, l) for t, h in enumerate(history) for l in large if h[l] == 1]
        assert len(fallbacks) <= 1, f"fresh={fresh}: {fallbacks}"
        # (with the same gradient every call the threshold still moves by more than the prediction
        # accepts until about the thirteenth call)
        predicted = sum(1 for h in history[10:] for l in large if h[l] == 3)
        assert predicted >= 0.7 * 20 * len(large), f"fresh={fresh}: bounds are still sampled late in the run"
        assert all(h[l] == 3 for h in history[20:] for l in large), f"fresh={fresh}"


def test_heavy_tailed_gradients_fed_in_turn_do_not_cost_failed_bounds():
    """The stress recipe (Student-t noise, p = 5, 0.1 % kept) on a 4096 x 4096 layer, four gradients
    fed in turn over 40 calls: the threshold jumps with the gradient's turn, and the layer has to
    learn that from its forecasts while bounds are still sampled -- after the ten calls that
    sample, at most one bound may fail."""
    import torch
    from paper_2312_17530_amd import binding
    w = synth.scaled_down(synth.config(4), 4096, 4096)
    sess = _session(w.shapes, w.p, w.alpha, w.ratios)
    arenas = []
    for t in range(4):
        sess.set_grad(synth.gradients(w, t))
        arenas.append(sess.grad.clone())
    history = []
    for t in range(40):
        sess.grad = arenas[t % 4]
        sess.compress()
        torch.cuda.synchronize()
        history.append(binding.rsdgc_last_paths(sess.plan, sess.workspace)[0])
    assert all(h in (0, 1, 3) for h in history)
    assert history[16:].count(1) <= 1, history
    assert history[20:].count(3) >= 19, history


def test_a_bound_that_fails_because_a_tile_overflows_does_not_widen_the_margin():
    """A 64 x 576 layer with p = 7 and k_l = 25: the scores of neighbouring centres share most of
    their 49 elements, so hundreds of centres of one tile lie within a few per cent of the
    threshold.  A bound set further below the threshold after such a tile overflowed would overflow
    again, call after call; the margin has to shrink instead, and the layer comes back to predicted
    bounds.  Every call gives the oracle's result, carried residual included."""
    import torch
    from paper_2312_17530_amd import binding
    w = synth.config(3)
    shape, ratio, p = w.shapes[1], w.ratios[1], 7
    assert shape == (64, 576)
    grads = [synth.gradients(w, t)[1] for t in range(4)]
    sess = _session([shape], p, w.alpha, [ratio])
    r = np.zeros(shape, np.float32)
    history = []
    for t in range(40):
        g = grads[t % 4]
        sess.set_grad([g])
        sess.compress()
        torch.cuda.synchronize()
        path = binding.rsdgc_last_paths(sess.plan, sess.workspace)[0]
        history.append(path)
        o = oracle.compress_layer(g, r, p, w.alpha, ratio)
        assert o.k == 25
        gi, gv, gc, gn = sess.results()[0]
        gpu_r = sess.unpack(sess.residual)[0]
        assert parity.check_layer(f"call {t}, path {path}", shape, p, o.k, o.tau, o.nsi, o.centres,
                                  o.idx, o.val, o.r_new, o.v, gi, gv, gc, gn, gpu_r)
        r = gpu_r.copy()     # (equal to the oracle's where the selections agree; the next call starts from the same state)
        sess.set_residual([r])
    assert all(h in (0, 1, 3) for h in history)
    assert history[24:].count(1) <= 4, history
    assert history[24:].count(3) >= 12, history


def test_gradients_at_the_edges_of_the_range_of_candidate_bounds():
    """The main pass tests scores against a layer's bound in float32, which its error bounds allow
    for bounds between 2^-40 and 2^40; a layer whose bound would lie outside is ranked on the full
    map.  Gradients scaled to either side of both ends: the oracle's result at every scale, the
    candidate path (predicted bounds by the third call) inside the range, the full map outside."""
    import torch
    from paper_2312_17530_amd import binding
    R, C, p, ratio = 256, 2304, 3, 0.02
    rng = np.random.default_rng(91)
    base = rng.standard_normal((R, C)).astype(np.float32)
    zero = np.zeros((R, C), np.float32)
    for scale, inside in [(2.0 ** -42, False), (2.0 ** -41.5, False), (2.0 ** -39, True), (2.0 ** -36, True),
                          (2.0 ** 36, True), (2.0 ** 38.5, True), (2.0 ** 40.5, False), (2.0 ** 43, False)]:
        g = (base * np.float32(scale)).astype(np.float32)
        sess = _session([(R, C)], p, 0.5, [ratio])
        o = oracle.compress_layer(g, zero, p, 0.5, ratio)
        assert (2.0 ** -40 <= float(o.tau) <= 2.0 ** 40) == inside, (scale, float(o.tau))
        for call in range(3):
            sess.set_grad([g])
            sess.set_residual([zero])
            sess.compress()
            torch.cuda.synchronize()
            path = binding.rsdgc_last_paths(sess.plan, sess.workspace)[0]
            gi, gv, gc, gn = sess.results()[0]
            parity.check_layer(f"scale 2^{np.log2(scale):.1f}, call {call}, path {path}", (R, C), p, o.k, o.tau, o.nsi,
                               o.centres, o.idx, o.val, o.r_new, o.v, gi, gv, gc, gn, sess.unpack(sess.residual)[0])
        assert path == (3 if inside else 1), (scale, path)


def _same_floats(a, b):
    a, b = np.asarray(a, np.float32).reshape(-1), np.asarray(b, np.float32).reshape(-1)
    return a.shape == b.shape and bool(np.all((a.view(np.uint32) == b.view(np.uint32)) | (np.isnan(a) & np.isnan(b))))


@pytest.mark.parametrize("path", [AUTO, FULL_MAP])
def test_non_finite_gradients_give_a_well_formed_result_and_leave_no_trace(path):
    """NaN and infinite gradient values are not detected and which centres win next to them is
    unspecified -- but a call on them must still be well formed (k_l centres per layer, ascending
    indices inside the layer, the kept elements exactly the windows of those centres, values and
    residual copied bit for bit), and the thresholds it leaves in the workspace (infinite, NaN)
    must not spoil later calls: those give the oracle's result again."""
    import torch
    shapes, ratios, p = [(512, 4608), (64, 576), (300, 77)], [0.02, 0.05, 0.03], 3
    rng = np.random.default_rng(77)
    clean = [(rng.standard_normal(sh) * 1e-3).astype(np.float32) for sh in shapes]
    zero = [np.zeros(sh, np.float32) for sh in shapes]
    sess = _session(shapes, p, 0.5, ratios, path=path)

    def oracle_call(tag):
        sess.set_grad(clean)
        sess.set_residual(zero)
        sess.compress()
        torch.cuda.synchronize()
        res, gpu_r = sess.results(), sess.unpack(sess.residual)
        for l, sh in enumerate(shapes):
            o = oracle.compress_layer(clean[l], zero[l], p, 0.5, ratios[l])
            gi, gv, gc, gn = res[l]
            parity.check_layer(f"{tag}[l={l}]", sh, p, o.k, o.tau, o.nsi, o.centres, o.idx, o.val, o.r_new, o.v,
                               gi, gv, gc, gn, gpu_r[l])

    for _ in range(3):
        oracle_call("before")                  # (three calls: the candidate path now predicts its bounds)
    scattered = [g.copy() for g in clean]
    for g in scattered:
        flat = g.reshape(-1)
        at = rng.choice(flat.size, size=max(4, flat.size // 5000), replace=False)
        flat[at[0::4]] = np.nan
        flat[at[1::4]] = np.inf
        flat[at[2::4]] = -np.inf
        flat[at[3::4]] = np.float32(3e38)      # squares overflow float32, not the sums kept in double
    tile_of_inf = [g.copy() for g in clean]
    tile_of_inf[0][32:64, 1024:1536] = np.inf
    all_nan = [g.copy() for g in clean]
    all_nan[1][:] = np.nan
    all_nan[2][:] = np.inf
    for tag, grads in [("scattered", scattered), ("tile of inf", tile_of_inf), ("whole layers", all_nan),
                       ("scattered again", scattered)]:
        sess.set_grad(grads)
        sess.set_residual(zero)
        sess.compress()
        torch.cuda.synchronize()
        res, gpu_r = sess.results(), sess.unpack(sess.residual)
        for l, (R, C) in enumerate(shapes):
            gi, gv, gc, gn = res[l]
            k = int(np.ceil(R * C / (p * p) * ratios[l]))
            assert gn == k and len(gc) == k, f"{tag}[l={l}]"
            assert np.all(np.diff(gc.astype(np.int64)) > 0) and int(gc[-1]) < R * C
            want = np.flatnonzero(parity.dilate_np(gc, R, C, p)).astype(np.uint32)
            assert np.array_equal(gi, want), f"{tag}[l={l}]: kept indices are not the windows of the centres"
            v = grads[l].reshape(-1)
            assert _same_floats(gv, v[want]), f"{tag}[l={l}]: values"
            r_want = v.copy()
            r_want[want] = 0.0
            assert _same_floats(gpu_r[l], r_want), f"{tag}[l={l}]: residual"
        oracle_call(f"after {tag}")
        oracle_call(f"after {tag}, second call")


def test_non_finite_gradients_with_momentum_and_in_the_block_reading():
    """The same for Eq. 12's momentum (u = m u + g carries the NaN on; the kept elements of u and r
    are still cleared) and for the reading with non-overlapping neighbourhoods: k_l centres or
    blocks, ascending, values and arenas bit for bit from the call's own kept set."""
    import torch
    from paper_2312_17530_amd.session import Session, BlockSession
    shapes, ratios, p, m = [(256, 1152), (64, 576), (300, 77)], [0.02, 0.05, 0.03], 3, 0.9
    rng = np.random.default_rng(78)
    grads = [(rng.standard_normal(sh) * 1e-3).astype(np.float32) for sh in shapes]
    u0 = [(rng.standard_normal(sh) * 1e-3).astype(np.float32) for sh in shapes]
    for g in grads:
        flat = g.reshape(-1)
        at = rng.choice(flat.size, size=max(3, flat.size // 3000), replace=False)
        flat[at[0::3]] = np.nan
        flat[at[1::3]] = np.inf
        flat[at[2::3]] = -np.inf
    grads[1][8:24, 100:400] = np.inf
    zero = [np.zeros(sh, np.float32) for sh in shapes]

    sess = Session(shapes, p, 0.5, ratios, momentum=float(m))
    for _ in range(2):
        sess.set_grad(grads)
        sess.set_residual(zero)
        sess.set_momentum(u0)
        sess.compress()
        torch.cuda.synchronize()
        res, gpu_r, gpu_u = sess.results(), sess.unpack(sess.residual), sess.unpack(sess.momentum_buf)
        for l, (R, C) in enumerate(shapes):
            gi, gv, gc, gn = res[l]
            k = int(np.ceil(R * C / (p * p) * ratios[l]))
            assert gn == k and len(gc) == k and np.all(np.diff(gc.astype(np.int64)) > 0) and int(gc[-1]) < R * C
            want = np.flatnonzero(parity.dilate_np(gc, R, C, p)).astype(np.uint32)
            assert np.array_equal(gi, want)
            un, vn = oracle.momentum_accumulate(u0[l], grads[l], zero[l], float(m))   # elementwise: u = m u + g, v = r + u
            u, v = un.reshape(-1).copy(), vn.reshape(-1).copy()
            assert _same_floats(gv, v[want]), f"momentum[l={l}]: values"
            u[want] = 0.0
            v[want] = 0.0
            assert _same_floats(gpu_u[l], u) and _same_floats(gpu_r[l], v), f"momentum[l={l}]: arenas"

    bs = BlockSession(shapes, p, 0.5, ratios)
    bs.set_grad(grads)
    bs.set_residual(zero)
    bs.compress()
    torch.cuda.synchronize()
    res, gpu_r = bs.results(), bs.unpack(bs.residual)
    for l, (R, C) in enumerate(shapes):
        gb, gv = res[l]
        BR, BC = -(-R // p), -(-C // p)
        assert len(gb) == bs.plan.layer_k(l) and np.all(np.diff(gb.astype(np.int64)) > 0) and int(gb[-1]) < BR * BC
        v = grads[l]
        want_r = v.copy()
        want_val = np.zeros(len(gb) * p * p, np.float32)
        for j, b in enumerate(gb):
            bx, by = divmod(int(b), BC)
            x1, y1 = min(R, bx * p + p), min(C, by * p + p)
            blk = np.zeros((p, p), np.float32)
            blk[:x1 - bx * p, :y1 - by * p] = v[bx * p:x1, by * p:y1]
            want_val[j * p * p:(j + 1) * p * p] = blk.ravel()
            want_r[bx * p:x1, by * p:y1] = 0.0
        assert _same_floats(gv, want_val), f"blocks[l={l}]: values"
        assert _same_floats(gpu_r[l], want_r), f"blocks[l={l}]: residual"


def test_set_ratios_and_determinism():
    import torch
    w = synth.scaled_down(synth.config(2), 256, 512)
    grads = synth.gradients(w, 0)
    sess = _session(w.shapes, w.p, w.alpha, w.ratios)
    sess.set_grad(grads)
    sess.compress()
    a = [(i.copy(), v.copy()) for i, v, _, _ in sess.results()]
    ra = sess.residual.clone()
    sess.residual.zero_()
    sess.compress()
    b = sess.results()
    for (ia, va), (ib, vb, _, _) in zip(a, b):
        assert np.array_equal(ia, ib) and np.array_equal(va.view(np.uint32), vb.view(np.uint32))
    assert torch.equal(ra, sess.residual)
    # same plan, new ratios: same result as a fresh plan with those ratios
    from paper_2312_17530_amd import binding
    new = [min(1.0, r * 0.5) for r in w.ratios]
    binding.rsdgc_plan_set_ratios(sess.plan, new)
    fresh = _session(w.shapes, w.p, w.alpha, new)
    assert sess.plan.out_capacity == fresh.plan.out_capacity
    sess.residual.zero_()
    fresh.set_grad(grads)
    sess.compress()
    fresh.compress()
    for l, ((i1, v1, c1, n1), (i2, v2, c2, n2)) in enumerate(zip(sess.results(), fresh.results())):
        assert n1 == n2 == fresh.plan.layer_k(l)
        # out buffers of `sess` were sized for the larger ratios; offsets follow the new plan
        assert np.array_equal(i1, i2) and np.array_equal(v1.view(np.uint32), v2.view(np.uint32))
        assert np.array_equal(c1, c2)


def test_either_centre_output_may_be_given_alone():
    """out_centre_counts without out_centre_idx (and the other way round) gives what the call
    with both gives; with neither, the message is unchanged."""
    import torch
    from paper_2312_17530_amd import binding
    w = synth.scaled_down(synth.config(1), 256, 512)
    grads = synth.gradients(w, 0)
    sess = _session(w.shapes, w.p, w.alpha, w.ratios)
    sess.set_grad(grads)
    sess.compress()
    torch.cuda.synchronize()
    both_idx, both_cnt = sess.out_centre_idx.clone(), sess.out_centre_counts.clone()
    msg = (sess.out_idx.clone(), sess.out_val.clone(), sess.out_counts.clone())
    assert int(both_cnt.sum()) == sum(sess.plan.layer_k(l) for l in range(len(w.shapes)))
    for give_idx, give_cnt in [(False, True), (True, False), (False, False)]:
        ci = torch.full_like(both_idx, -7)
        cc = torch.full_like(both_cnt, -7)
        sess.residual.zero_()
        if sess.residual_next is not None:
            sess.residual_next.zero_()
        binding.rsdgc_compress(sess.plan, sess.grad, sess.residual, sess.residual_next, sess.out_idx,
                               sess.out_val, sess.out_counts, sess.workspace,
                               out_centre_idx=ci if give_idx else None,
                               out_centre_counts=cc if give_cnt else None)
        torch.cuda.synchronize()
        tag = f"idx={give_idx} counts={give_cnt}"
        if give_cnt:
            assert torch.equal(cc, both_cnt), tag
        else:
            assert bool((cc == -7).all()), tag
        if give_idx:
            for l in range(len(w.shapes)):
                o, k = sess.plan.centre_offset(l), sess.plan.layer_k(l)
                assert torch.equal(ci[o:o + k], both_idx[o:o + k]), f"{tag} layer {l}"
        else:
            assert bool((ci == -7).all()), tag
        assert torch.equal(sess.out_idx, msg[0]) and torch.equal(sess.out_val, msg[1]), tag
        assert torch.equal(sess.out_counts, msg[2]), tag


def test_a_recycled_workspace_is_prepared_again_when_the_plan_is_told():
    """The workspace is wiped between two calls (as when its memory was freed and handed out
    again); after rsdgc_plan_forget_workspace the next call uploads the tables afresh and gives
    the same result -- for an element plan and a block plan."""
    import torch
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import BlockSession
    w = synth.scaled_down(synth.config(1), 256, 512)
    grads = synth.gradients(w, 0)
    for make in (lambda: _session(w.shapes, w.p, w.alpha, w.ratios),
                 lambda: BlockSession(w.shapes, w.p, w.alpha, w.ratios)):
        sess = make()
        sess.set_grad(grads)
        sess.compress()
        torch.cuda.synchronize()
        first = [tuple(np.copy(a) if isinstance(a, np.ndarray) else a for a in r) for r in sess.results()]
        sess.workspace.zero_()                       # tables gone
        binding.rsdgc_plan_forget_workspace(sess.plan)
        sess.residual.zero_()
        sess.compress()
        torch.cuda.synchronize()
        for a, b in zip(first, sess.results()):
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


def test_decompress_accumulate_sums_messages():
    import torch
    w = synth.config(0)
    grads = synth.gradients(w, 0)
    sess = _session(w.shapes, w.p, w.alpha, w.ratios)
    sess.set_grad(grads)
    sess.compress()
    idx, val, _, _ = sess.results()[0]
    dense = torch.full_like(sess.grad, 1.0)
    sess.decompress(accumulate=True, dense=dense)
    sess.decompress(accumulate=True, dense=dense)
    torch.cuda.synchronize()
    got = dense.cpu().numpy()
    want = np.ones(got.size, dtype=np.float32)
    want = oracle.decompress(idx, val, want.size, dense=want, accumulate_into=True)
    want = oracle.decompress(idx, val, want.size, dense=want, accumulate_into=True)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_receiving_side_skips_what_a_malformed_message_names():
    """A message that crossed a network is not trusted: indices at or beyond the layer's size are
    skipped, a count beyond the layer's segment is read as the segment's capacity, a negative
    count as zero -- and nothing outside the layers' elements is written (the arena's padding
    keeps its values).  Checked for rsdgc_decompress (overwrite) and rsdgc_apply."""
    import torch
    from paper_2312_17530_amd import binding
    shapes, ratios = [(64, 100), (40, 50), (30, 30)], [0.1, 0.2, 0.1]
    G = [r * c for r, c in shapes]
    sess = _session(shapes, 3, 0.5, ratios)
    sess.set_grad([synth.layer_gradient(sh, 1e-2, 83, 0, l) for l, sh in enumerate(shapes)])
    sess.compress()
    torch.cuda.synchronize()
    plan = sess.plan
    offs = [plan.out_offset(l) for l in range(3)] + [plan.out_capacity]
    caps = [offs[l + 1] - offs[l] for l in range(3)]
    counts = sess.out_counts.cpu().numpy().copy()
    idx = sess.out_idx.cpu().numpy().view(np.uint32).copy()
    val = sess.out_val.cpu().numpy().copy()
    rng = np.random.default_rng(84)
    # layer 0: three pairs name elements that do not exist
    n0 = int(counts[0])
    assert n0 >= 3
    picks = np.array([0, n0 // 2, n0 - 1])
    idx[offs[0] + picks] = np.array([G[0], 0xffffffff, G[0] + 12345], dtype=np.uint32)
    # layer 1: the whole segment holds valid pairs, the count claims far more
    assert caps[1] <= G[1]
    idx[offs[1]:offs[1] + caps[1]] = rng.permutation(G[1])[:caps[1]].astype(np.uint32)
    val[offs[1]:offs[1] + caps[1]] = rng.standard_normal(caps[1]).astype(np.float32)
    counts[1] = caps[1] + 100000
    # layer 2: a negative count
    counts[2] = -5
    dev = sess.grad.device
    idx_t = torch.from_numpy(idx.view(np.int32)).to(dev)
    val_t = torch.from_numpy(val).to(dev)
    cnt_t = torch.from_numpy(counts.astype(np.int32)).to(dev)
    # what a careful reader of the message keeps
    kept = []
    for l in range(3):
        n = min(max(int(counts[l]), 0), caps[l])
        i, v = idx[offs[l]:offs[l] + n], val[offs[l]:offs[l] + n]
        ok = i < G[l]
        kept.append((i[ok], v[ok]))
    assert len(kept[0][0]) == n0 - 3 and len(kept[1][0]) == caps[1] and len(kept[2][0]) == 0

    dense = torch.full_like(sess.grad, 7.0)
    binding.rsdgc_decompress(plan, idx_t, val_t, cnt_t, dense, False, sess.workspace)
    torch.cuda.synchronize()
    want = np.full(dense.numel(), 7.0, dtype=np.float32)          # padding keeps its 7.0
    for l in range(3):
        o = plan.layer_offset(l)
        want[o:o + G[l]] = oracle.decompress(kept[l][0], kept[l][1], G[l])
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), want.view(np.uint32))

    weights = [rng.standard_normal(sh).astype(np.float32) for sh in shapes]
    w_dev = torch.full_like(sess.grad, 3.0)
    sess.pack(weights, w_dev)
    before = w_dev.cpu().numpy().copy()
    binding.rsdgc_apply(plan, [(idx_t, val_t, cnt_t)], w_dev, 0.5, sess.workspace)
    torch.cuda.synchronize()
    want_w = before.copy()
    for l in range(3):
        o = plan.layer_offset(l)
        want_w[o:o + G[l]] = oracle.apply_messages(weights[l], [kept[l]], 0.5).reshape(-1)
    assert np.array_equal(w_dev.cpu().numpy().view(np.uint32), want_w.view(np.uint32))


@pytest.mark.parametrize("work_feed", [FEED_AUTO, FEED_ON], ids=["feed_auto", "feed_on"])
def test_compress_can_be_captured_in_a_hip_graph_and_replayed(in_place, work_feed):
    """rsdgc_compress enqueues kernels only (no allocation, no synchronisation, no memset node),
    so a caller may capture it.  Every replay must reproduce the eager result, with eager work
    and synchronisations between the replays.  With the work feed forced on, every replay also
    has to find the feed's counters cleared by the call's own first kernel."""
    import torch
    w = synth.config(1)
    grads = synth.gradients(w, 0)
    sess = _session(w.shapes, w.p, w.alpha, w.ratios, in_place=in_place, work_feed=work_feed)
    sess.set_grad(grads)
    sess.compress()                                  # first call uploads the plan's tables
    torch.cuda.synchronize()
    sess.residual.zero_()
    sess.compress()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (sess.out_idx, sess.out_val, sess.out_counts, sess.residual,
                               sess.out_centre_idx, sess.out_centre_counts)]
    graph = torch.cuda.CUDAGraph()
    sess.residual.zero_()
    source = sess.residual                           # the arena the captured call reads
    with torch.cuda.graph(graph):
        sess.compress()                              # with two arenas sess.residual is now the other one
    for rep in range(3):
        for t in (sess.out_idx, sess.out_val, sess.out_counts, sess.out_centre_idx,
                  sess.out_centre_counts, sess.residual, source):
            t.zero_()                                # eager work between replays
        scratch = torch.randn(1 << 20, device="cuda").sum().item()
        assert np.isfinite(scratch)
        graph.replay()
        torch.cuda.synchronize()
        got = (sess.out_idx, sess.out_val, sess.out_counts, sess.residual, sess.out_centre_idx,
               sess.out_centre_counts)
        counts = ref[2].cpu().numpy()
        for l in range(w.n_layers):                  # entries past the counts are unspecified
            o, n = sess.plan.out_offset(l), int(counts[l])
            assert torch.equal(got[0][o:o + n], ref[0][o:o + n]), (rep, l)
            assert torch.equal(got[1][o:o + n], ref[1][o:o + n]), (rep, l)
        assert torch.equal(got[2], ref[2]) and torch.equal(got[3], ref[3]), rep
        assert torch.equal(got[4], ref[4]) and torch.equal(got[5], ref[5]), rep
