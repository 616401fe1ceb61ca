"""Do the oracle's pins bite?  Each case plants ONE plausible mistake in a private copy of the
oracle's C source (a dropped term, a wrong sign or index, a wrong divisor, a reversed order),
builds it on the CPU and runs a compact battery of the pins against it.  The unmodified oracle
must pass the whole battery; every mutant must fail at least one pin.  Nothing here touches
the GPU or the GPU library."""
import ctypes
import importlib.util
import math
import os
import subprocess

import numpy as np
import pytest
from scipy import ndimage

from tests.brute import brute_compress

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rsdgc_oracle.c")


def _load_variant(tmp_path, name, source_text):
    """A second, independent instance of the oracle package bound to another C file."""
    c_path = os.path.join(tmp_path, f"{name}.c")
    so_path = os.path.join(tmp_path, f"lib{name}.so")
    with open(c_path, "w") as f:
        f.write(source_text)
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
                           c_path, "-o", so_path, "-lm"])
    spec = importlib.util.spec_from_file_location(f"oracle_variant_{name}",
                                                  os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._SRC, mod._LIB = c_path, so_path
    return mod


def _replace_nth(text, old, new, n=0):
    parts = text.split(old)
    assert len(parts) > n + 1, f"pattern not found {n + 1} times: {old!r}"
    return old.join(parts[:n + 1]) + new + old.join(parts[n + 1:])


def battery(orc):
    """Names of the pins the given oracle instance fails."""
    fails = []

    def check(name, cond):
        if not cond:
            fails.append(name)

    rng = np.random.default_rng(2024)
    # Eq. 11
    check("k_golden", [orc.keep_count(262144, 3, 0.02), orc.keep_count(102760448, 5, 0.001),
                       orc.keep_count(10, 3, 1.0), orc.keep_count(1000, 1, 0.0015)] == [583, 4111, 2, 2])
    # Eq. 12 add
    r = rng.standard_normal(1000).astype(np.float32)
    g = rng.standard_normal(1000).astype(np.float32)
    check("accumulate", np.array_equal(orc.accumulate(r, g), r + g))
    # Eqs. 8-10: closed forms
    c = -3.5
    m = orc.nsi(np.full((7, 9), c, np.float32), 3, 0.25).astype(np.float64)
    a = abs(c)
    check("const_interior", np.allclose(m[1:-1, 1:-1], 0.25 * a, rtol=1e-6))
    check("const_edge", np.allclose(m[0, 1:-1], a * (0.25 * 2 / 3 + 0.75 * math.sqrt(2) / 3), rtol=1e-6))
    check("const_corner", np.isclose(m[0, 0], a * (0.25 * 4 / 9 + 0.75 * math.sqrt(20) / 9), rtol=1e-6))
    v = np.zeros((23, 29), np.float32)
    v[11, 14] = -0.75
    for p in (3, 5):
        mm = orc.nsi(v, p, 0.5).astype(np.float64)
        check(f"impulse_p{p}", np.isclose(mm[11, 14], 0.75 * (0.5 + 0.5 * math.sqrt(p * p - 1)) / (p * p), rtol=1e-6))
    # library box filters, non-square, offset mean
    for p, shape in ((3, (37, 53)), (5, (5, 64)), (1, (9, 4))):
        x = (rng.standard_normal(shape) + 0.7).astype(np.float32)
        x64 = x.astype(np.float64)
        box_abs = ndimage.uniform_filter(np.abs(x64), size=p, mode="constant")
        box = ndimage.uniform_filter(x64, size=p, mode="constant")
        box_sq = ndimage.uniform_filter(x64 * x64, size=p, mode="constant")
        std = np.sqrt(np.maximum(box_sq - box * box, 0))
        check(f"box_a1_p{p}", np.allclose(orc.nsi(x, p, 1.0), box_abs, rtol=1e-6, atol=1e-7))
        check(f"box_a0_p{p}", np.allclose(orc.nsi(x, p, 0.0), std, rtol=1e-5, atol=1e-6))
        check(f"box_mix_p{p}", np.allclose(orc.nsi(x, p, 0.3), 0.3 * box_abs + 0.7 * std, rtol=1e-5, atol=1e-6))
    # ranking
    s = rng.integers(0, 40, size=3000).astype(np.float32)
    centres, tau = orc.select(s, 137)
    order = sorted(range(s.size), key=lambda i: (-float(s[i]), i))
    check("select", centres.tolist() == sorted(order[:137]) and tau == float(s[order[136]]))
    # dilation
    cs = np.sort(rng.choice(33 * 47, size=20, replace=False)).astype(np.uint32)
    seed = np.zeros((33, 47), bool)
    seed.ravel()[cs] = True
    check("dilate", np.array_equal(orc.dilate(cs, 33, 47, 3).astype(bool),
                                   ndimage.binary_dilation(seed, structure=np.ones((3, 3), bool))))
    # one whole iteration: invariants and brute force
    gg = (rng.standard_normal((13, 17)) * 1e-2).astype(np.float32)
    rr = (rng.standard_normal((13, 17)) * 1e-2).astype(np.float32)
    res = orc.compress_layer(gg, rr, 3, 0.5, 0.3)
    vv = rr + gg
    dense = orc.decompress(res.idx, res.val, vv.size).reshape(vv.shape)
    check("sent_plus_residual", np.array_equal(dense + res.r_new, vv))
    check("values", np.array_equal(res.val, vv.ravel()[res.idx]))
    b = brute_compress(gg.tolist(), rr.tolist(), 3, 0.5, 0.3)
    check("brute", res.k == b["k"] and res.centres.tolist() == b["centres"] and res.idx.tolist() == b["idx"]
          and res.r_new.ravel().tolist() == b["r_new"])
    # Eq. 12 in full: momentum, then the same steps; masking of the momentum
    uu = (rng.standard_normal((13, 17)) * 1e-2).astype(np.float32)
    mm = np.float32(0.9)
    un = mm * uu + gg
    mres = orc.compress_layer_momentum(gg, uu, rr, 0.9, 3, 0.5, 0.3)
    check("momentum_v", np.array_equal(mres.layer.v, rr + un))
    sent = np.zeros(gg.size, bool)
    sent[mres.layer.idx] = True
    want_u = un.ravel().copy()
    want_u[sent] = 0.0
    check("momentum_masked", np.array_equal(mres.u_new.ravel(), want_u))
    plain = orc.compress_layer(un, rr, 3, 0.5, 0.3)
    check("momentum_selection", np.array_equal(plain.idx, mres.layer.idx)
          and np.array_equal(plain.r_new, mres.layer.r_new))
    # Eqs. 3-5: dynamic per-layer ratios
    ws = [(rng.standard_normal(sh) * sc).astype(np.float32) for sh, sc in (((9, 11), 1.0), ((40, 3), 0.2), ((5, 5), 4.0))]
    mu = np.concatenate([np.abs(w).ravel() for w in ws])
    lay = np.concatenate([np.full(w.size, l) for l, w in enumerate(ws)])
    K = int(math.ceil(0.2 * mu.size))
    kept = np.bincount(lay[np.argsort(-mu.astype(np.float64), kind="stable")[:K]], minlength=3)
    check("dynamic_ratios", orc.dynamic_ratios(ws, 0.2) == [kept[l] / ws[l].size for l in range(3)])
    ones = [np.ones((2, 5), np.float32), -np.ones((3, 4), np.float32)]
    check("dynamic_ties", orc.dynamic_ratios(ones, 13 / 22) == [1.0, 3 / 12])
    # Eq. 12, third line
    w10 = np.arange(10, dtype=np.float32)
    m1 = (np.array([1, 3], np.uint32), np.array([1.0, 2.0], np.float32))
    m2 = (np.array([3, 9], np.uint32), np.array([0.5, -4.0], np.float32))
    check("apply", orc.apply_messages(w10, [m1, m2], 0.5).tolist() == [0, 0.5, 2, 1.75, 4, 5, 6, 7, 8, 11])
    w45 = np.arange(20, dtype=np.float32).reshape(4, 5)
    b1 = (np.array([0, 3], np.uint32),
          np.array([1, 2, 3, 4, 5, 6, 7, 8, 9] + [10, 20, 99, 99, 99, 99, 99, 99, 99], np.float32))
    b2 = (np.array([0], np.uint32), np.array([0.5, 0, 0, 0, -4, 0, 0, 0, 0], np.float32))
    want45 = w45.copy()
    want45[0:3, 0:3] -= np.float32(0.5) * np.array([[1.5, 2, 3], [4, 1, 6], [7, 8, 9]], np.float32)
    want45[3, 3:5] -= np.float32(0.5) * np.array([10, 20], np.float32)
    check("apply_blocks", orc.apply_block_messages(w45, [b1, b2], 3, 0.5).tolist() == want45.tolist())
    # block reading
    vb = (rng.standard_normal((13, 17)) + 0.3).astype(np.float32)
    pad = np.zeros((15, 18), np.float64)
    pad[:13, :17] = vb
    blk = pad.reshape(5, 3, 6, 3).transpose(0, 2, 1, 3).reshape(5, 6, 9)
    check("block_nsi", np.allclose(orc.block_nsi(vb, 3, 0.3), 0.3 * np.abs(blk).mean(axis=2) + 0.7 * blk.std(axis=2),
                                   rtol=1e-6, atol=1e-7))
    bres = orc.compress_layer_blocks(gg, rr, 3, 0.5, 0.3)
    bs = bres.nsi.ravel()
    border = sorted(range(bs.size), key=lambda i: (-float(bs[i]), i))
    check("block_select", bres.blocks.tolist() == sorted(border[:bres.k]) and bres.k == math.ceil(13 * 17 / 9 * 0.3))
    bdense = orc.decompress_blocks(bres.blocks, bres.val, 13, 17, 3)
    check("block_sent_plus_residual", np.array_equal(bdense + bres.r_new, rr + gg))
    first = int(bres.blocks[0])
    check("block_values", bres.val[:3].tolist() == (rr + gg)[first // 6 * 3, first % 6 * 3:first % 6 * 3 + 3].tolist()
          if first % 6 < 5 else True)
    # block reading with Eq. 12's momentum
    bm = orc.compress_layer_blocks_momentum(gg, uu, rr, 0.9, 3, 0.5, 0.3)
    bplain = orc.compress_layer_blocks(un, rr, 3, 0.5, 0.3)
    check("block_momentum_selection", np.array_equal(bm.layer.blocks, bplain.blocks)
          and np.array_equal(bm.layer.val, bplain.val) and np.array_equal(bm.layer.r_new, bplain.r_new))
    bkept = orc.decompress_blocks(bm.layer.blocks, np.ones(bm.layer.k * 9, np.float32), 13, 17, 3) != 0
    check("block_momentum_masked", np.array_equal(bm.u_new, np.where(bkept, np.float32(0), un)))
    check("block_momentum_v", np.array_equal(bm.layer.v, rr + un))
    d2 = np.ones(10, np.float32)
    orc.decompress(np.array([2, 5], np.uint32), np.array([0.5, -1.0], np.float32), 10, dense=d2, accumulate_into=True)
    check("decompress_acc", d2.tolist() == [1, 1, 1.5, 1, 1, 0, 1, 1, 1, 1])
    return fails


MUTANTS = [
    ("signed_mean", "sum_abs += fabs(w);", "sum_abs += w;", 0),
    ("std_about_abs_mean", "const double mean = sum / n;", "const double mean = sum_abs / n;", 0),
    ("abs_deviation", "sq += d * d;", "sq += fabs(d);", 0),
    ("variance_not_std", "const double std = sqrt(sq / n);", "const double std = sq / n;", 0),
    ("sample_std", "sqrt(sq / n)", "sqrt(sq / (n - 1.0))", 0),
    ("alpha_swapped", "return alpha * mean_abs + (1.0 - alpha) * std;",
     "return (1.0 - alpha) * mean_abs + alpha * std;", 0),
    ("replicate_border", "        return 0.0;\n    return (double)v[x * C + y];",
     "        return (double)v[(x < 0 ? 0 : x >= R ? R - 1 : x) * C + (y < 0 ? 0 : y >= C ? C - 1 : y)];\n"
     "    return (double)v[x * C + y];", 0),
    ("divisor_p", "const double n = (double)p * (double)p;", "const double n = (double)p;", 0),
    ("k_floor", "double kf = ceil(q * rho);", "double kf = floor(q * rho);", 0),
    ("k_divides_by_p", "(double)((int64_t)p * (int64_t)p)", "(double)p", 0),
    ("ties_to_higher_index", "if (p->index < q->index) return -1;\n    if (p->index > q->index) return 1;",
     "if (p->index < q->index) return 1;\n    if (p->index > q->index) return -1;", 0),
    ("rank_ascending", "if (p->score > q->score) return -1;\n    if (p->score < q->score) return 1;",
     "if (p->score > q->score) return 1;\n    if (p->score < q->score) return -1;", 0),
    ("one_sided_window", "for (int dx = -h; dx <= h; ++dx)", "for (int dx = -h; dx < h; ++dx)", 0),
    ("one_sided_dilation", "for (int dx = -h; dx <= h; ++dx)", "for (int dx = -h; dx < h; ++dx)", 2),
    ("residual_keeps_sent", "r_new[i] = mask[i] ? 0.0f : v[i];", "r_new[i] = v[i];", 0),
    ("emit_abs_value", "val[n] = v[i];", "val[n] = fabsf(v[i]);", 0),
    ("accumulate_subtracts", "volatile float s = r[i] + g[i];", "volatile float s = r[i] - g[i];", 0),
    ("decompress_overwrites", "volatile float s = dense[idx[j]] + val[j];", "volatile float s = val[j];", 0),
    ("momentum_scales_gradient", "volatile float mu = m * u[i];", "volatile float mu = m * g[i];", 0),
    ("momentum_not_added_to_v", "volatile float s = r[i] + un;", "volatile float s = r[i] + g[i];", 0),
    ("momentum_fused", "volatile float mu = m * u[i];\n        volatile float un = mu + g[i];",
     "volatile float mu = m * u[i];\n        volatile float un = (float)((double)m * (double)u[i] + (double)g[i]);", 0),
    ("dynamic_signed_weights", "it[i].mu = fabsf(w_all[i]);", "it[i].mu = w_all[i];", 0),
    ("dynamic_keeps_lowest", "if (p->mu > q->mu) return -1;\n    if (p->mu < q->mu) return 1;",
     "if (p->mu > q->mu) return 1;\n    if (p->mu < q->mu) return -1;", 0),
    ("dynamic_floor", "double kf = ceil(rho * (double)N);", "double kf = floor(rho * (double)N);", 0),
    ("dynamic_ties_to_later_layer", "if (p->layer < q->layer) return -1;\n    if (p->layer > q->layer) return 1;",
     "if (p->layer < q->layer) return 1;\n    if (p->layer > q->layer) return -1;", 0),
    ("dynamic_ratio_of_network", "(double)kept[l] / (double)Gl", "(double)kept[l] / (double)N", 0),
    ("apply_adds_the_step", "volatile float wn = w[i] - step;", "volatile float wn = w[i] + step;", 0),
    ("apply_scales_the_weight", "volatile float step = eta * sum[i];", "volatile float step = eta * w[i];", 0),
    ("apply_keeps_last_message_only", "rsdgc_oracle_decompress(idx[k], val[k], n[k], sum, G, 1);",
     "rsdgc_oracle_decompress(idx[k], val[k], n[k], sum, G, 0);", 0),
    ("apply_blocks_adds_the_step", "volatile float wn = w[i] - step;", "volatile float wn = w[i] + step;", 1),
    ("apply_blocks_keeps_last_message_only", "rsdgc_oracle_decompress_blocks(blocks[k], val[k], n[k], R, C, p, sum, 1);",
     "rsdgc_oracle_decompress_blocks(blocks[k], val[k], n[k], R, C, p, sum, 0);", 0),
    ("block_window_centred", "double w = slot(v, R, C, bx * p + dx, by * p + dy);", "double w = slot(v, R, C, bx * p + dx - 1, by * p + dy - 1);", 0),
    ("block_std_around_zero", "double d = slot(v, R, C, bx * p + dx, by * p + dy) - mean;", "double d = slot(v, R, C, bx * p + dx, by * p + dy);", 0),
    ("block_residual_keeps_sent", "if (inside) r[x * C + y] = 0.0f;", "if (inside) r[x * C + y] = v[x * C + y];", 0),
    ("block_values_transposed", "val[j * p * p + dx * p + dy] = inside ? v[x * C + y] : 0.0f;", "val[j * p * p + dy * p + dx] = inside ? v[x * C + y] : 0.0f;", 0),
    ("block_grid_row_stride", "const int64_t bx = blocks[j] / BC, by = blocks[j] % BC;\n        for (int dx = 0; dx < p; ++dx)\n            for (int dy = 0; dy < p; ++dy) {\n                const int64_t x = bx * p + dx, y = by * p + dy;\n                const int inside",
     "const int64_t bx = blocks[j] / BR, by = blocks[j] % BR;\n        for (int dx = 0; dx < p; ++dx)\n            for (int dy = 0; dy < p; ++dy) {\n                const int64_t x = bx * p + dx, y = by * p + dy;\n                const int inside", 0),
    ("block_momentum_not_masked", "                    u[x * C + y] = 0.0f;\n", "", 0),
    ("block_momentum_keeps_old_momentum", "        u[i] = un[i];", "        u[i] = u[i];", 0),
    ("block_momentum_scores_without_residual", "rsdgc_oracle_block_nsi(v, R, C, p, alpha, nsi);            /* step B2 */",
     "rsdgc_oracle_block_nsi(un, R, C, p, alpha, nsi);            /* step B2 */", 1),
    ("block_momentum_sends_momentum_only", "val[j * p * p + dx * p + dy] = within ? v[x * C + y] : 0.0f;",
     "val[j * p * p + dx * p + dy] = within ? un[x * C + y] : 0.0f;", 0),
    ("block_momentum_residual_keeps_sent", "                    r[x * C + y] = 0.0f;\n", "", 0),
    ("momentum_not_masked", "u_out[i] = mask[i] ? 0.0f : u_new[i];", "u_out[i] = u_new[i];", 0),
    ("momentum_masked_where_kept_out", "u_out[i] = mask[i] ? 0.0f : u_new[i];", "u_out[i] = mask[i] ? u_new[i] : 0.0f;", 0),
]


def test_unmodified_oracle_passes_the_battery(tmp_path):
    orc = _load_variant(str(tmp_path), "plain", open(SRC).read())
    assert battery(orc) == []


@pytest.mark.parametrize("name,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_planted_mistake_is_caught(tmp_path, name, old, new, nth):
    text = _replace_nth(open(SRC).read(), old, new, nth)
    orc = _load_variant(str(tmp_path), name, text)
    fails = battery(orc)
    assert fails, f"mutant {name} slipped through every pin"
