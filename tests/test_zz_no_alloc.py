"""rsdgc_compress_static (the entry point that allocates nothing: its workspace is an array inside
the library) against rsdgc_compress with a caller-allocated workspace, through the C ABI.

Both run the same kernels, so every output must be the same bytes: counts, indices, values,
centre lists and the new residual.  The built-in array is shared by all plans and keeps what the
last call left, so the sequence matters: a multi-layer plan, then a smaller one (the array still
holds the first plan's tables and counters), then the first plan again with its residual carried."""
import numpy as np
import pytest

from paper_2312_17530_amd import synth

pytestmark = pytest.mark.gpu

_BIG = dict(shapes=[(300, 1000), (64, 27), (513, 2049), (1, 777), (1024, 1152)], p=3, alpha=0.5,
            ratios=[0.02, 0.5, 0.01, 0.1, 0.03], seed=91)
_SMALL = dict(shapes=[(97, 131), (256, 260)], p=5, alpha=0.25, ratios=[0.05, 0.004], seed=92)


def _gradients(spec, t):
    return [synth.layer_gradient(sh, 1e-3, spec["seed"], t, l) for l, sh in enumerate(spec["shapes"])]


def _same(tag, a, b):
    import torch
    assert torch.equal(a.view(torch.int32), b.view(torch.int32)), tag


def _compare_call(tag, ref, stat_plan, bufs, grads):
    """One iteration on both paths from the same state; returns nothing, asserts equality."""
    import torch
    from paper_2312_17530_amd import binding
    print("no-alloc case", tag, flush=True)
    ref.set_grad(grads)
    bufs["resid_in"].copy_(ref.residual)
    ref.compress()
    binding.rsdgc_compress_static(stat_plan, ref.grad, bufs["resid_in"], bufs["resid_out"], bufs["idx"],
                                  bufs["val"], bufs["counts"], bufs["cidx"], bufs["ccounts"])
    torch.cuda.synchronize()
    _same(f"{tag}: counts", ref.out_counts, bufs["counts"])
    _same(f"{tag}: centre counts", ref.out_centre_counts, bufs["ccounts"])
    for off, sz in zip(ref.offsets, ref.sizes):             # (the padding between layers is never written)
        _same(f"{tag}: residual", ref.residual[off:off + sz], bufs["resid_out"][off:off + sz])
    counts = ref.out_counts.cpu().numpy()
    assert counts.sum() > 0, tag
    for l in range(ref.plan.n_layers):
        o, n = ref.plan.out_offset(l), int(counts[l])
        _same(f"{tag}: idx of layer {l}", ref.out_idx[o:o + n], bufs["idx"][o:o + n])
        _same(f"{tag}: val of layer {l}", ref.out_val[o:o + n], bufs["val"][o:o + n])
        co, k = ref.plan.centre_offset(l), ref.plan.layer_k(l)
        _same(f"{tag}: centres of layer {l}", ref.out_centre_idx[co:co + k], bufs["cidx"][co:co + k])


def _buffers(ref):
    import torch
    return {"resid_in": torch.zeros_like(ref.residual), "resid_out": torch.full_like(ref.residual, 3.0),
            "idx": torch.full_like(ref.out_idx, -1), "val": torch.full_like(ref.out_val, 5.0),
            "counts": torch.full_like(ref.out_counts, -1), "cidx": torch.full_like(ref.out_centre_idx, -1),
            "ccounts": torch.full_like(ref.out_centre_counts, -1)}


def test_static_workspace_call_equals_the_call_with_a_caller_workspace():
    from paper_2312_17530_amd import binding
    from paper_2312_17530_amd.session import Session
    sessions, plans, bufs = {}, {}, {}
    for name, spec in (("big", _BIG), ("small", _SMALL)):
        sessions[name] = Session(spec["shapes"], spec["p"], spec["alpha"], spec["ratios"])
        # a plan of its own for the built-in workspace: the two paths keep separate state
        plans[name] = binding.rsdgc_plan(spec["shapes"], spec["p"], spec["alpha"], spec["ratios"])
        assert plans[name].workspace_bytes <= binding.RSDGC_STATIC_WORKSPACE_BYTES
        bufs[name] = _buffers(sessions[name])
    assert plans["small"].workspace_bytes < plans["big"].workspace_bytes
    _compare_call("big, t=0", sessions["big"], plans["big"], bufs["big"], _gradients(_BIG, 0))
    _compare_call("small after big, t=0", sessions["small"], plans["small"], bufs["small"], _gradients(_SMALL, 0))
    _compare_call("small, t=1 (residual carried)", sessions["small"], plans["small"], bufs["small"],
                  _gradients(_SMALL, 1))
    _compare_call("big after small, t=1 (residual carried)", sessions["big"], plans["big"], bufs["big"],
                  _gradients(_BIG, 1))


def test_static_workspace_refuses_a_plan_beyond_its_size():
    """Refused before anything is enqueued, with both sizes in the message."""
    import torch
    from paper_2312_17530_amd import binding
    plan = binding.rsdgc_plan([(8192, 4096)], 3, 0.5, [0.01])
    assert plan.workspace_bytes > binding.RSDGC_STATIC_WORKSPACE_BYTES
    n = plan.total_elems
    g = torch.zeros(n, dtype=torch.float32, device="cuda")
    r = torch.zeros_like(g)
    ro = torch.full_like(g, 3.0)
    idx = torch.zeros(plan.out_capacity, dtype=torch.int32, device="cuda")
    val = torch.zeros(plan.out_capacity, dtype=torch.float32, device="cuda")
    counts = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.RsdgcError) as e:
        binding.rsdgc_compress_static(plan, g, r, ro, idx, val, counts)
    assert e.value.code == binding.RSDGC_ETOOBIG and str(plan.workspace_bytes) in str(e.value)
    torch.cuda.synchronize()
    assert int(counts[0]) == -1 and float(ro.min()) == 3.0      # nothing was touched
