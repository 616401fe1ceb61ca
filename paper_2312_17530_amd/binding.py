"""ctypes binding of librsdgc.so: argument marshalling only.

Function names mirror the C ABI declared in ``include/rsdgc.h``.  Device buffers are
torch tensors (torch is used for device memory and streams only); their addresses are
handed to the library unchanged.  There is no CPU fallback: if the library has not been
built, ``load()`` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librsdgc.so")

RSDGC_OK, RSDGC_EINVAL, RSDGC_ENOMEM, RSDGC_EHIP, RSDGC_ETOOBIG = 0, -1, -2, -3, -4
RSDGC_STATIC_WORKSPACE_BYTES = 64 << 20
RSDGC_MAX_P = 7

EXPORTS = [
    "rsdgc_plan", "rsdgc_plan_set_ratios", "rsdgc_plan_set_path", "rsdgc_plan_set_work_feed", "rsdgc_plan_forget_workspace", "rsdgc_plan_destroy", "rsdgc_n_layers",
    "rsdgc_total_elems", "rsdgc_layer_offset", "rsdgc_layer_elems", "rsdgc_layer_k",
    "rsdgc_out_offset", "rsdgc_out_capacity", "rsdgc_centre_offset", "rsdgc_centre_capacity",
    "rsdgc_workspace_bytes", "rsdgc_compress", "rsdgc_compress_static", "rsdgc_compress_momentum", "rsdgc_dynamic_ratios", "rsdgc_apply", "rsdgc_apply_blocks", "rsdgc_plan_blocks", "rsdgc_compress_blocks", "rsdgc_compress_blocks_momentum",
    "rsdgc_decompress_blocks", "rsdgc_nsi", "rsdgc_decompress",
    "rsdgc_last_paths", "rsdgc_profile_begin", "rsdgc_profile_end", "rsdgc_stage_name",
    "rsdgc_strerror", "rsdgc_last_hip_error",
]
RSDGC_N_STAGES = 9
RSDGC_PATH_AUTO, RSDGC_PATH_FULL_MAP = 0, 1


class Shape(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64)]


class RsdgcError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load()
        msg = lib.rsdgc_strerror(code).decode()
        hip = lib.rsdgc_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({code})" +
                         (f" [{hip}]" if code in (RSDGC_EHIP, RSDGC_ETOOBIG) and hip else ""))
        self.code = code


_lib = None


def load() -> ctypes.CDLL:
    """Load librsdgc.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2312_17530_amd.build` "
            "(or __graft_entry__.build()); there is no fallback implementation")
    # PyTorch ships its own HIP runtime; it has to be in the process before this library
    # is loaded so that both resolve the same runtime (device pointers and streams are
    # only meaningful inside the runtime that created them).
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    lib.rsdgc_plan.argtypes = [ctypes.POINTER(Shape), i32, i32, ctypes.POINTER(i32), f64,
                               ctypes.POINTER(f64), ctypes.POINTER(vp)]
    lib.rsdgc_plan.restype = ctypes.c_int
    lib.rsdgc_plan_set_ratios.argtypes = [vp, ctypes.POINTER(f64)]
    lib.rsdgc_plan_set_ratios.restype = ctypes.c_int
    lib.rsdgc_plan_set_path.argtypes = [vp, i32]
    lib.rsdgc_plan_set_path.restype = ctypes.c_int
    lib.rsdgc_plan_set_work_feed.argtypes = [vp, i32]
    lib.rsdgc_plan_set_work_feed.restype = ctypes.c_int
    lib.rsdgc_plan_forget_workspace.argtypes = [vp]
    lib.rsdgc_plan_forget_workspace.restype = ctypes.c_int
    lib.rsdgc_plan_destroy.argtypes = [vp]
    lib.rsdgc_plan_destroy.restype = None
    lib.rsdgc_n_layers.argtypes = [vp]
    lib.rsdgc_n_layers.restype = i32
    for name in ["rsdgc_total_elems", "rsdgc_out_capacity", "rsdgc_centre_capacity"]:
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = i64
    for name in ["rsdgc_layer_offset", "rsdgc_layer_elems", "rsdgc_layer_k", "rsdgc_out_offset",
                 "rsdgc_centre_offset"]:
        getattr(lib, name).argtypes = [vp, i32]
        getattr(lib, name).restype = i64
    lib.rsdgc_workspace_bytes.argtypes = [vp]
    lib.rsdgc_workspace_bytes.restype = ctypes.c_size_t
    lib.rsdgc_compress.argtypes = [vp] * 11
    lib.rsdgc_compress.restype = ctypes.c_int
    lib.rsdgc_compress_static.argtypes = [vp] * 10
    lib.rsdgc_compress_static.restype = ctypes.c_int
    lib.rsdgc_compress_momentum.argtypes = [vp, vp, vp, vp, ctypes.c_float] + [vp] * 9
    lib.rsdgc_compress_momentum.restype = ctypes.c_int
    lib.rsdgc_dynamic_ratios.argtypes = [vp, vp, f64, ctypes.POINTER(f64), vp, vp]
    lib.rsdgc_dynamic_ratios.restype = ctypes.c_int
    lib.rsdgc_apply.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                ctypes.c_float, vp, vp]
    lib.rsdgc_apply.restype = ctypes.c_int
    lib.rsdgc_apply_blocks.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                ctypes.c_float, vp, vp]
    lib.rsdgc_apply_blocks.restype = ctypes.c_int
    lib.rsdgc_plan_blocks.argtypes = lib.rsdgc_plan.argtypes
    lib.rsdgc_plan_blocks.restype = ctypes.c_int
    lib.rsdgc_compress_blocks.argtypes = [vp] * 9
    lib.rsdgc_compress_blocks.restype = ctypes.c_int
    lib.rsdgc_compress_blocks_momentum.argtypes = [vp, vp, vp, vp, ctypes.c_float] + [vp] * 7
    lib.rsdgc_compress_blocks_momentum.restype = ctypes.c_int
    lib.rsdgc_decompress_blocks.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, vp, vp]
    lib.rsdgc_decompress_blocks.restype = ctypes.c_int
    lib.rsdgc_nsi.argtypes = [vp] * 6
    lib.rsdgc_nsi.restype = ctypes.c_int
    lib.rsdgc_decompress.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, vp, vp]
    lib.rsdgc_decompress.restype = ctypes.c_int
    lib.rsdgc_last_paths.argtypes = [vp, vp, ctypes.POINTER(i32), vp]
    lib.rsdgc_last_paths.restype = ctypes.c_int
    lib.rsdgc_profile_begin.argtypes = [vp, i32]
    lib.rsdgc_profile_begin.restype = ctypes.c_int
    lib.rsdgc_profile_end.argtypes = [vp, ctypes.POINTER(f64), ctypes.POINTER(i32)]
    lib.rsdgc_profile_end.restype = ctypes.c_int
    lib.rsdgc_stage_name.argtypes = [i32]
    lib.rsdgc_stage_name.restype = ctypes.c_char_p
    lib.rsdgc_strerror.argtypes = [ctypes.c_int]
    lib.rsdgc_strerror.restype = ctypes.c_char_p
    lib.rsdgc_last_hip_error.argtypes = []
    lib.rsdgc_last_hip_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(code: int, where: str) -> None:
    if code != RSDGC_OK:
        raise RsdgcError(code, where)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, None for None."""
    if t is None:
        return None
    assert t.is_contiguous()
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = stream if isinstance(stream, int) else stream.cuda_stream
    return h or None


class Plan:
    """Owner of one rsdgc_plan_t (host object)."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:        # at interpreter shutdown the module may already be gone
            _lib.rsdgc_plan_destroy(h)

    @property
    def handle(self):
        return self._h

    @property
    def n_layers(self) -> int:
        return load().rsdgc_n_layers(self._h)

    @property
    def total_elems(self) -> int:
        return load().rsdgc_total_elems(self._h)

    @property
    def out_capacity(self) -> int:
        return load().rsdgc_out_capacity(self._h)

    @property
    def centre_capacity(self) -> int:
        return load().rsdgc_centre_capacity(self._h)

    @property
    def workspace_bytes(self) -> int:
        return load().rsdgc_workspace_bytes(self._h)

    def layer_offset(self, l: int) -> int:
        return load().rsdgc_layer_offset(self._h, l)

    def layer_elems(self, l: int) -> int:
        return load().rsdgc_layer_elems(self._h, l)

    def layer_k(self, l: int) -> int:
        return load().rsdgc_layer_k(self._h, l)

    def out_offset(self, l: int) -> int:
        return load().rsdgc_out_offset(self._h, l)

    def centre_offset(self, l: int) -> int:
        return load().rsdgc_centre_offset(self._h, l)


def rsdgc_plan(shapes: Sequence[Tuple[int, int]], p: int, alpha: float,
               keep_ratio: Sequence[float], p_per_layer: Optional[Sequence[int]] = None,
               blocks: bool = False) -> Plan:
    """blocks=True: rsdgc_plan_blocks (non-overlapping p x p neighbourhoods)."""
    lib = load()
    n = len(shapes)
    if len(keep_ratio) != n or (p_per_layer is not None and len(p_per_layer) != n):
        raise RsdgcError(RSDGC_EINVAL, "rsdgc_plan")
    arr = (Shape * max(n, 1))(*[Shape(int(r), int(c)) for r, c in shapes])
    ratios = (ctypes.c_double * max(len(keep_ratio), 1))(*[float(x) for x in keep_ratio])
    pp = None
    if p_per_layer is not None:
        pp = (ctypes.c_int32 * max(n, 1))(*[int(x) for x in p_per_layer])
    out = ctypes.c_void_p()
    fn = lib.rsdgc_plan_blocks if blocks else lib.rsdgc_plan
    _check(fn(arr, n, int(p), pp, float(alpha), ratios, ctypes.byref(out)),
           "rsdgc_plan_blocks" if blocks else "rsdgc_plan")
    return Plan(out.value)


def rsdgc_plan_blocks(shapes, p: int, alpha: float, keep_ratio, p_per_layer=None) -> Plan:
    return rsdgc_plan(shapes, p, alpha, keep_ratio, p_per_layer, blocks=True)


def rsdgc_compress_blocks(plan: Plan, grad, residual, residual_out, out_block_idx, out_val, out_counts,
                          workspace, stream=None) -> None:
    _check(load().rsdgc_compress_blocks(plan.handle, _ptr(grad), _ptr(residual), _ptr(residual_out),
                                        _ptr(out_block_idx), _ptr(out_val), _ptr(out_counts),
                                        _ptr(workspace), _stream(stream)), "rsdgc_compress_blocks")


def rsdgc_compress_blocks_momentum(plan: Plan, grad, momentum, momentum_out, m: float, residual, residual_out,
                                   out_block_idx, out_val, out_counts, workspace, stream=None) -> None:
    _check(load().rsdgc_compress_blocks_momentum(plan.handle, _ptr(grad), _ptr(momentum), _ptr(momentum_out),
                                                 float(m), _ptr(residual), _ptr(residual_out),
                                                 _ptr(out_block_idx), _ptr(out_val), _ptr(out_counts),
                                                 _ptr(workspace), _stream(stream)),
           "rsdgc_compress_blocks_momentum")


def rsdgc_decompress_blocks(plan: Plan, block_idx, val, counts, dense, accumulate: bool, workspace,
                            stream=None) -> None:
    _check(load().rsdgc_decompress_blocks(plan.handle, _ptr(block_idx), _ptr(val), _ptr(counts), _ptr(dense),
                                          1 if accumulate else 0, _ptr(workspace), _stream(stream)),
           "rsdgc_decompress_blocks")


def rsdgc_plan_set_ratios(plan: Plan, keep_ratio: Sequence[float]) -> None:
    if len(keep_ratio) != plan.n_layers:
        raise RsdgcError(RSDGC_EINVAL, "rsdgc_plan_set_ratios")
    ratios = (ctypes.c_double * len(keep_ratio))(*[float(x) for x in keep_ratio])
    _check(load().rsdgc_plan_set_ratios(plan.handle, ratios), "rsdgc_plan_set_ratios")


FEED_AUTO, FEED_OFF, FEED_ON = 0, 1, 2


def rsdgc_plan_forget_workspace(plan: "Plan") -> None:
    _check(load().rsdgc_plan_forget_workspace(plan.handle), "rsdgc_plan_forget_workspace")


def rsdgc_plan_set_work_feed(plan: "Plan", mode: int) -> None:
    _check(load().rsdgc_plan_set_work_feed(plan.handle, int(mode)), "rsdgc_plan_set_work_feed")


def rsdgc_plan_set_path(plan: Plan, path: int) -> None:
    _check(load().rsdgc_plan_set_path(plan.handle, int(path)), "rsdgc_plan_set_path")


def rsdgc_compress(plan: Plan, grad, residual, residual_out, out_idx, out_val, out_counts, workspace,
                   out_centre_idx=None, out_centre_counts=None, stream=None) -> None:
    """residual_out is a second arena, or the same tensor as residual for an update in place."""
    _check(load().rsdgc_compress(plan.handle, _ptr(grad), _ptr(residual), _ptr(residual_out), _ptr(out_idx),
                                 _ptr(out_val), _ptr(out_counts), _ptr(out_centre_idx),
                                 _ptr(out_centre_counts), _ptr(workspace), _stream(stream)),
           "rsdgc_compress")


def rsdgc_compress_static(plan: Plan, grad, residual, residual_out, out_idx, out_val, out_counts,
                          out_centre_idx=None, out_centre_counts=None, stream=None) -> None:
    """rsdgc_compress with the library's built-in workspace (no device allocation)."""
    _check(load().rsdgc_compress_static(plan.handle, _ptr(grad), _ptr(residual), _ptr(residual_out),
                                        _ptr(out_idx), _ptr(out_val), _ptr(out_counts), _ptr(out_centre_idx),
                                        _ptr(out_centre_counts), _stream(stream)), "rsdgc_compress_static")


def rsdgc_compress_momentum(plan: Plan, grad, momentum, momentum_out, m: float, residual, residual_out,
                            out_idx, out_val, out_counts, workspace, out_centre_idx=None,
                            out_centre_counts=None, stream=None) -> None:
    """Eq. 12 in full; the five arenas must not overlap."""
    _check(load().rsdgc_compress_momentum(plan.handle, _ptr(grad), _ptr(momentum), _ptr(momentum_out),
                                          float(m), _ptr(residual), _ptr(residual_out), _ptr(out_idx),
                                          _ptr(out_val), _ptr(out_counts), _ptr(out_centre_idx),
                                          _ptr(out_centre_counts), _ptr(workspace), _stream(stream)),
           "rsdgc_compress_momentum")


def rsdgc_dynamic_ratios(plan: Plan, weights, global_ratio: float, workspace, stream=None) -> List[float]:
    """Eqs. 3-5: per-layer keep ratios from the weights arena (waits for the GPU)."""
    out = (ctypes.c_double * plan.n_layers)()
    _check(load().rsdgc_dynamic_ratios(plan.handle, _ptr(weights), float(global_ratio), out,
                                       _ptr(workspace), _stream(stream)), "rsdgc_dynamic_ratios")
    return [float(x) for x in out]


def rsdgc_apply(plan: Plan, messages, weights, eta: float, workspace, stream=None) -> None:
    """Eq. 12, third line: weights -= eta * (sum of the messages, in order).
    messages: sequence of (idx, val, counts) device tensors as written by rsdgc_compress."""
    n = len(messages)
    arr = ctypes.c_void_p * max(n, 1)
    idx = arr(*[_ptr(m[0]) for m in messages])
    val = arr(*[_ptr(m[1]) for m in messages])
    cnt = arr(*[_ptr(m[2]) for m in messages])
    _check(load().rsdgc_apply(plan.handle, n, idx, val, cnt, _ptr(weights), float(eta), _ptr(workspace),
                              _stream(stream)), "rsdgc_apply")


def rsdgc_apply_blocks(plan: Plan, messages, weights, eta: float, workspace, stream=None) -> None:
    """rsdgc_apply for a block plan.  messages: sequence of (block_idx, val, counts) device
    tensors as written by rsdgc_compress_blocks."""
    n = len(messages)
    arr = ctypes.c_void_p * max(n, 1)
    idx = arr(*[_ptr(m[0]) for m in messages])
    val = arr(*[_ptr(m[1]) for m in messages])
    cnt = arr(*[_ptr(m[2]) for m in messages])
    _check(load().rsdgc_apply_blocks(plan.handle, n, idx, val, cnt, _ptr(weights), float(eta), _ptr(workspace),
                                     _stream(stream)), "rsdgc_apply_blocks")


def rsdgc_nsi(plan: Plan, grad, residual, nsi_out, workspace, stream=None) -> None:
    _check(load().rsdgc_nsi(plan.handle, _ptr(grad), _ptr(residual), _ptr(nsi_out),
                            _ptr(workspace), _stream(stream)), "rsdgc_nsi")


def rsdgc_decompress(plan: Plan, idx, val, counts, dense, accumulate: bool, workspace,
                     stream=None) -> None:
    _check(load().rsdgc_decompress(plan.handle, _ptr(idx), _ptr(val), _ptr(counts), _ptr(dense),
                                   1 if accumulate else 0, _ptr(workspace), _stream(stream)),
           "rsdgc_decompress")


def rsdgc_profile_begin(plan: Plan, max_calls: int) -> None:
    _check(load().rsdgc_profile_begin(plan.handle, int(max_calls)), "rsdgc_profile_begin")


def rsdgc_profile_end(plan: Plan):
    """Returns ({stage name: mean ms per call}, number of recorded calls)."""
    lib = load()
    ms = (ctypes.c_double * RSDGC_N_STAGES)()
    n = ctypes.c_int32(0)
    _check(lib.rsdgc_profile_end(plan.handle, ms, ctypes.byref(n)), "rsdgc_profile_end")
    return {lib.rsdgc_stage_name(i).decode(): ms[i] for i in range(RSDGC_N_STAGES)}, n.value


def rsdgc_last_paths(plan: Plan, workspace, stream=None):
    """Ranking path per layer of the last compress call (0 candidates, 1 full map, 2 none)."""
    out = (ctypes.c_int32 * plan.n_layers)()
    _check(load().rsdgc_last_paths(plan.handle, _ptr(workspace), out, _stream(stream)),
           "rsdgc_last_paths")
    return list(out)
