"""Boundary tests that need no GPU: the C-ABI library loads, exports every symbol the header
declares, validates its arguments, and does the host arithmetic of the plan (Eq. 11 counts,
arena offsets, output capacities) correctly.  No kernel is launched."""
import ctypes
import math
import os
import re
from fractions import Fraction

import pytest

from paper_2312_17530_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    header = open(os.path.join(ROOT, "include", "rsdgc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rsdgc_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(binding.EXPORTS)
    for name in sorted(declared):
        assert hasattr(lib, name), name


def test_plan_counts_match_golden_eq11():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "eq11_keep_counts.txt"))
            if ln.strip() and not ln.startswith("#")]
    for G, p, rho, k in rows:
        G, p, rho, k = int(G), int(p), float(rho), int(k)
        # factor G into a matrix; any factorisation must give the same count
        rows_ = 1
        for cand in (4096, 512, 64, 9, 3, 2):
            if G % cand == 0:
                rows_ = cand
                break
        plan = binding.rsdgc_plan([(rows_, G // rows_)], p, 0.5, [rho])
        assert plan.layer_k(0) == k
        assert plan.centre_capacity == k
        assert plan.out_capacity == min(k * p * p, G)


def test_plan_layout_of_the_five_workloads():
    want_total = [262144, 11189952, 23547072, 139740864, 102760448]
    want_layers = [1, 21, 54, 19, 1]
    for i in range(5):
        w = synth.config(i)
        assert w.total_elems == want_total[i] and w.n_layers == want_layers[i]
        plan = binding.rsdgc_plan(w.shapes, w.p, w.alpha, w.ratios)
        assert plan.n_layers == w.n_layers
        off, out_off, c_off = 0, 0, 0
        for l, (r, c) in enumerate(w.shapes):
            G = r * c
            assert plan.layer_offset(l) == off and off % 64 == 0
            assert plan.layer_elems(l) == G
            exact = Fraction(G, w.p * w.p) * Fraction(w.ratios[l])
            k = plan.layer_k(l)
            assert abs(k - exact) < 1 + 1e-6 and k >= exact - 1e-6          # a ceiling of Eq. 11
            assert plan.out_offset(l) == out_off and plan.centre_offset(l) == c_off
            off += (G + 63) // 64 * 64
            out_off += min(k * w.p * w.p, G)
            c_off += k
        assert plan.total_elems == off
        assert plan.out_capacity == out_off and plan.centre_capacity == c_off
        # workspace holds at least a float32 score map and two bitmasks
        assert plan.workspace_bytes >= 4 * off + 2 * off // 8
        assert plan.workspace_bytes % 256 == 0
    # configuration 0: the survey's worked number
    assert binding.rsdgc_plan([(512, 512)], 3, 0.5, [0.02]).layer_k(0) == 583


@pytest.mark.parametrize("kwargs", [
    dict(shapes=[(0, 5)]), dict(shapes=[(5, -1)]), dict(p=2), dict(p=0), dict(p=9),
    dict(alpha=-0.1), dict(alpha=1.5), dict(alpha=float("nan")), dict(ratios=[1.5]),
    dict(ratios=[-0.01]), dict(ratios=[float("nan")]), dict(shapes=[(70000, 70000)]),
    dict(p_per_layer=[4]), dict(shapes=[]),
])
def test_plan_rejects_bad_arguments(kwargs):
    args = dict(shapes=[(8, 8)], p=3, alpha=0.5, ratios=[0.1], p_per_layer=None)
    args.update(kwargs)
    if "shapes" in kwargs and "ratios" not in kwargs:
        args["ratios"] = [0.1] * len(args["shapes"])
    with pytest.raises(binding.RsdgcError) as ei:
        binding.rsdgc_plan(args["shapes"], args["p"], args["alpha"], args["ratios"], args["p_per_layer"])
    assert ei.value.code == binding.RSDGC_EINVAL


def test_set_ratios_recomputes_counts_and_validates():
    plan = binding.rsdgc_plan([(512, 512), (64, 27)], 3, 0.5, [0.02, 0.02])
    ws = plan.workspace_bytes
    assert [plan.layer_k(0), plan.layer_k(1)] == [583, 4]
    binding.rsdgc_plan_set_ratios(plan, [0.0, 1.0])
    assert [plan.layer_k(0), plan.layer_k(1)] == [0, 192]
    assert plan.out_capacity == min(192 * 9, 1728) and plan.out_offset(1) == 0
    assert plan.workspace_bytes == ws
    with pytest.raises(binding.RsdgcError):
        binding.rsdgc_plan_set_ratios(plan, [0.5, 2.0])
    assert [plan.layer_k(0), plan.layer_k(1)] == [0, 192]      # unchanged after the error


def test_work_feed_mode_is_validated():
    plan = binding.rsdgc_plan([(64, 64)], 3, 0.5, [0.1])
    ws = plan.workspace_bytes
    for mode in (binding.FEED_ON, binding.FEED_OFF, binding.FEED_AUTO):
        binding.rsdgc_plan_set_work_feed(plan, mode)
    assert plan.workspace_bytes == ws
    for bad in (-1, 3):
        with pytest.raises(binding.RsdgcError):
            binding.rsdgc_plan_set_work_feed(plan, bad)
    assert binding.load().rsdgc_plan_set_work_feed(None, 0) == binding.RSDGC_EINVAL
    binding.rsdgc_plan_forget_workspace(plan)
    assert binding.load().rsdgc_plan_forget_workspace(None) == binding.RSDGC_EINVAL


def test_per_layer_neighbourhood_side():
    plan = binding.rsdgc_plan([(90, 90), (90, 90), (90, 90)], 3, 0.5, [0.1, 0.1, 0.1], [1, 3, 5])
    assert [plan.layer_k(l) for l in range(3)] == [810, 90, 33]
    assert plan.out_capacity == 810 + 810 + 825


def test_device_entry_points_validate_before_touching_the_gpu():
    lib = binding.load()
    plan = binding.rsdgc_plan([(8, 8)], 3, 0.5, [0.1])
    null = None
    # null plan / null buffers -> RSDGC_EINVAL, nothing enqueued (this box may have no GPU at all)
    assert lib.rsdgc_compress(null, null, null, null, null, null, null, null, null, null, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_compress(plan.handle, null, null, null, null, null, null, null, null, null, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_nsi(plan.handle, null, null, null, null, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_decompress(plan.handle, null, null, null, null, 0, null, null) == binding.RSDGC_EINVAL
    # misaligned workspace / arenas are refused as well (addresses are never dereferenced here)
    a = 4096
    assert lib.rsdgc_compress(plan.handle, a, a, a, a, a, a, null, null, a + 8, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_compress(plan.handle, a + 4, a, a, a, a, a, null, null, a, null) == binding.RSDGC_EINVAL
    # the new residual goes to the same arena or to one that overlaps neither input: the plan's
    # arena is 64 floats (256 bytes) here, so a second arena 128 bytes further on overlaps
    assert plan.total_elems == 64
    assert lib.rsdgc_compress(plan.handle, a, 2 * a, 2 * a + 128, a, a, a, null, null, a, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_compress(plan.handle, a, 2 * a, a + 128, a, a, a, null, null, a, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_compress(plan.handle, a, 2 * a, a, a, a, a, null, null, a, null) == binding.RSDGC_EINVAL
    assert lib.rsdgc_profile_begin(plan.handle, 0) == binding.RSDGC_EINVAL
    assert lib.rsdgc_profile_end(null, null, null) == binding.RSDGC_EINVAL


def test_queries_on_bad_arguments_and_strerror():
    lib = binding.load()
    plan = binding.rsdgc_plan([(8, 8)], 3, 0.5, [0.1])
    assert lib.rsdgc_layer_k(plan.handle, 1) == -1 and lib.rsdgc_layer_offset(plan.handle, -1) == -1
    assert lib.rsdgc_n_layers(None) == -1 and lib.rsdgc_workspace_bytes(None) == 0
    assert lib.rsdgc_strerror(0) == b"ok"
    assert b"invalid" in lib.rsdgc_strerror(binding.RSDGC_EINVAL)
    assert lib.rsdgc_strerror(-99) == b"unknown error code"
    assert lib.rsdgc_stage_name(2) == b"capture" and lib.rsdgc_stage_name(99) == b""
    lib.rsdgc_plan_destroy(None)     # harmless


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "librsdgc.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load()


def test_block_plan_layout_on_the_host():
    """rsdgc_plan_blocks: k_l from Eq. 11, one index per kept block, p*p values per kept block
    (padding slots of partial blocks included), workspace = the plan's tables + the block grid's
    + the message accumulator."""
    shapes, p_list, ratios = [(90, 90), (10, 10), (64, 27), (7, 1000)], [3, 3, 5, 7], [0.1, 1.0, 0.5, 0.3]
    plan = binding.rsdgc_plan_blocks(shapes, 3, 0.5, ratios, p_list)
    ks = [math.ceil(r * c / (p * p) * rho) for (r, c), p, rho in zip(shapes, p_list, ratios)]
    assert [plan.layer_k(l) for l in range(4)] == ks
    n_blocks = [-(-r // p) * -(-c // p) for (r, c), p in zip(shapes, p_list)]
    assert all(k <= nb for k, nb in zip(ks, n_blocks))           # Eq. 11 never asks for more blocks than exist
    assert plan.centre_capacity == sum(ks)
    assert plan.out_capacity == sum(k * p * p for k, p in zip(ks, p_list))
    assert plan.out_capacity > sum(min(k * p * p, r * c) for k, p, (r, c) in zip(ks, p_list, shapes))  # (10,10): 16 blocks x 9 > 100
    assert [plan.centre_offset(l) for l in range(4)] == [0, ks[0], ks[0] + ks[1], ks[0] + ks[1] + ks[2]]
    assert plan.out_offset(2) == ks[0] * 9 + ks[1] * 9
    element_plan = binding.rsdgc_plan(shapes, 3, 0.5, ratios, p_list)
    assert plan.total_elems == element_plan.total_elems           # the arenas are laid out alike
    assert plan.workspace_bytes % 256 == 0 and 0 < plan.workspace_bytes < element_plan.workspace_bytes
    # ... + the message accumulator of rsdgc_apply_blocks (one float per arena element)
    assert plan.workspace_bytes > 4 * plan.total_elems
    binding.rsdgc_plan_set_ratios(plan, [0.0, 0.5, 0.5, 0.3])
    assert [plan.layer_k(l) for l in range(4)] == [0, 6, ks[2], ks[3]]
    with pytest.raises(binding.RsdgcError):
        binding.rsdgc_plan_blocks([(8, 8)], 4, 0.5, [0.1])


def test_newer_entry_points_validate_before_touching_the_gpu():
    lib = binding.load()
    plan = binding.rsdgc_plan([(8, 8)], 3, 0.5, [0.1])
    bplan = binding.rsdgc_plan_blocks([(8, 8)], 3, 0.5, [0.1])
    E, null, a = binding.RSDGC_EINVAL, None, 4096
    # momentum: null arenas, factor outside [0, 1], overlapping arenas (the arena is 64 floats = 256 bytes)
    assert lib.rsdgc_compress_momentum(plan.handle, a, null, a, 0.9, a, a, a, a, a, null, null, a, null) == E
    assert lib.rsdgc_compress_momentum(plan.handle, a, 2 * a, 3 * a, 1.5, 4 * a, 5 * a, a, a, a, null, null, 6 * a, null) == E
    assert lib.rsdgc_compress_momentum(plan.handle, a, 2 * a, 3 * a, float("nan"), 4 * a, 5 * a, a, a, a, null, null, 6 * a, null) == E
    assert lib.rsdgc_compress_momentum(plan.handle, a, 2 * a, 2 * a + 128, 0.9, 4 * a, 5 * a, a, a, a, null, null, 6 * a, null) == E
    assert lib.rsdgc_compress_momentum(plan.handle, a, 2 * a, 3 * a, 0.9, 4 * a, 3 * a, a, a, a, null, null, 6 * a, null) == E
    # dynamic ratios: bad fraction; nothing / everything kept needs no GPU at all
    out = (ctypes.c_double * 1)()
    assert lib.rsdgc_dynamic_ratios(plan.handle, a, 1.5, out, a, null) == E
    assert lib.rsdgc_dynamic_ratios(plan.handle, null, 0.5, out, a, null) == E
    assert lib.rsdgc_dynamic_ratios(plan.handle, a, 0.0, out, a, null) == binding.RSDGC_OK and out[0] == 0.0
    assert lib.rsdgc_dynamic_ratios(plan.handle, a, 1.0, out, a, null) == binding.RSDGC_OK and out[0] == 1.0
    # apply: message count out of range, null tables
    ptrs = (ctypes.c_void_p * 1)(a)
    assert lib.rsdgc_apply(plan.handle, 0, ptrs, ptrs, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply(plan.handle, 65, ptrs, ptrs, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply(plan.handle, 1, null, ptrs, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply(plan.handle, 1, (ctypes.c_void_p * 1)(None), ptrs, ptrs, a, 0.1, a, null) == E
    # plans of the two readings do not mix
    assert lib.rsdgc_compress(bplan.handle, a, 2 * a, 3 * a, a, a, a, null, null, 4 * a, null) == E
    assert lib.rsdgc_compress_blocks(plan.handle, a, 2 * a, 3 * a, a, a, a, 4 * a, null) == E
    assert lib.rsdgc_decompress_blocks(plan.handle, a, a, a, a, 0, 4 * a, null) == E
    assert lib.rsdgc_decompress(bplan.handle, a, a, a, a, 0, 4 * a, null) == E
    assert lib.rsdgc_nsi(bplan.handle, a, a, a, 4 * a, null) == E
    assert lib.rsdgc_apply(bplan.handle, 1, ptrs, ptrs, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply_blocks(plan.handle, 1, ptrs, ptrs, ptrs, a, 0.1, a, null) == E
    # apply for block messages: the same argument checks
    assert lib.rsdgc_apply_blocks(bplan.handle, 0, ptrs, ptrs, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply_blocks(bplan.handle, 65, ptrs, ptrs, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply_blocks(bplan.handle, 1, ptrs, null, ptrs, a, 0.1, a, null) == E
    assert lib.rsdgc_apply_blocks(bplan.handle, 1, ptrs, ptrs, ptrs, a + 4, 0.1, a, null) == E
    assert lib.rsdgc_apply_blocks(bplan.handle, 1, ptrs, ptrs, ptrs, a, float("nan"), a, null) == E
    assert lib.rsdgc_compress_blocks(bplan.handle, a, 2 * a, 2 * a + 128, a, a, a, 4 * a, null) == E    # overlapping arenas
    assert lib.rsdgc_compress_blocks(bplan.handle, a, a, a, a, a, a, 4 * a, null) == E                    # new residual on the gradient


def test_plans_near_the_32_bit_limits():
    """Per-layer quantities are 32-bit, offsets into the lists and slots 64-bit.  A block plan whose
    value segment k_l p^2 would not fit 32 bits is refused; block grids whose threshold-bucket lists
    add up to more than 2^32 entries are accepted and laid out without wrapping."""
    lib = binding.load()
    G = 65535 * 65537                    # 2^32 - 1 elements in one layer
    assert G == 2 ** 32 - 1
    for rho, ok in ((1.0, False), (0.5, True)):
        try:
            plan = binding.rsdgc_plan_blocks([(65535, 65537)], 3, 0.5, [rho])
            assert ok, "k_l * 9 exceeds 32 bits: must be refused"
            assert plan.layer_k(0) * 9 <= 0xffffffff and plan.out_capacity == plan.layer_k(0) * 9
            with pytest.raises(binding.RsdgcError):
                binding.rsdgc_plan_set_ratios(plan, [1.0])
        except binding.RsdgcError as e:
            assert not ok and e.code == binding.RSDGC_EINVAL
    # five block grids of 2^30 blocks each (p = 1): the lists of the grids hold a layer each
    shapes = [(32768, 32768)] * 5
    plan = binding.rsdgc_plan_blocks(shapes, 1, 0.5, [0.001] * 5)
    total = sum(r * c for r, c in shapes)
    assert total > 2 ** 32
    assert plan.workspace_bytes > 8 * total          # the lists alone: 8 bytes per entry
    del plan, lib


def test_workspace_of_vectors_and_narrow_layers_stays_in_proportion():
    """A tile's candidate slot is no longer than the tile (16 rows x 256 columns of the layer, or
    what the layer has of them), and a single column is laid out as a single row: the workspace of
    a long vector or of a tall layer of a few columns is a few bytes per element, the same for
    N x 1 as for 1 x N, and does not move with the keep ratios."""
    def ws(shapes, ratios=None, p=3):
        return binding.rsdgc_plan(shapes, p, 0.5, ratios or [0.02] * len(shapes)).workspace_bytes
    n = 2_000_000
    col, row = ws([(n, 1)]), ws([(1, n)])
    assert col == row
    assert col < 16 * n + (1 << 20)                      # (it was 260 bytes per element: 512 entries per 16-element tile)
    narrow = ws([(n // 7, 7)])
    assert narrow < 16 * n + (1 << 20)                   # 16 x 7 elements per tile: 112 entries
    # ordinary layers keep their 512 entries per tile: 1 byte per element for the slots
    wide = ws([(1024, 4096)])
    assert ws([(1024, 4096)], [0.0005]) == wide == ws([(1024, 4096)], [0.3])
    plan = binding.rsdgc_plan([(n, 1), (300, 77)], 3, 0.5, [0.02, 0.05])
    before = plan.workspace_bytes
    binding.rsdgc_plan_set_ratios(plan, [0.001, 0.5])
    assert plan.workspace_bytes == before
    # counts, offsets and capacities are those of the shape as given
    assert plan.layer_elems(0) == n and plan.layer_k(0) == math.ceil(n / 9 * 0.001)


def test_static_workspace_entry_point_validates_on_the_host():
    """rsdgc_compress_static refuses a null or block plan and a plan beyond its built-in workspace
    before it touches the GPU (this box may have none)."""
    lib = binding.load()
    null, a = None, 4096
    assert lib.rsdgc_compress_static(null, a, a, a, a, a, a, null, null, null) == binding.RSDGC_EINVAL
    bplan = binding.rsdgc_plan_blocks([(8, 8)], 3, 0.5, [0.1])
    assert lib.rsdgc_compress_static(bplan.handle, a, a, a, a, a, a, null, null, null) == binding.RSDGC_EINVAL
    big = binding.rsdgc_plan([(8192, 4096)], 3, 0.5, [0.01])
    assert big.workspace_bytes > binding.RSDGC_STATIC_WORKSPACE_BYTES
    assert lib.rsdgc_compress_static(big.handle, a, 2 * a, 3 * a, a, a, a, null, null, null) == binding.RSDGC_ETOOBIG
    assert str(big.workspace_bytes).encode() in lib.rsdgc_last_hip_error()
    assert b"built-in" in lib.rsdgc_strerror(binding.RSDGC_ETOOBIG)
