"""Device-memory plumbing around the binding: one object that owns the torch buffers a
plan needs (arenas, outputs, workspace) and moves host arrays in and out of them.
No arithmetic of the method happens here."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding


class Session:
    def __init__(self, shapes, p: int, alpha: float, ratios: Sequence[float],
                 p_per_layer: Optional[Sequence[int]] = None, device: str = "cuda:0",
                 want_centres: bool = True, path: int = binding.RSDGC_PATH_AUTO,
                 in_place: bool = False, momentum: Optional[float] = None,
                 work_feed: int = binding.FEED_AUTO):
        self.shapes = [(int(r), int(c)) for r, c in shapes]
        self.plan = binding.rsdgc_plan(self.shapes, p, alpha, ratios, p_per_layer)
        if path != binding.RSDGC_PATH_AUTO:
            binding.rsdgc_plan_set_path(self.plan, path)
        if work_feed != binding.FEED_AUTO:
            binding.rsdgc_plan_set_work_feed(self.plan, work_feed)
        self.device = torch.device(device)
        n = self.plan.total_elems
        L = self.plan.n_layers
        dev = self.device
        self.grad = torch.zeros(n, dtype=torch.float32, device=dev)
        # `residual` is always the newest residual: with two arenas compress() writes the
        # other one and the two names are swapped afterwards
        self.residual = torch.zeros(n, dtype=torch.float32, device=dev)
        self.in_place = in_place
        self.residual_next = None if in_place else torch.zeros(n, dtype=torch.float32, device=dev)
        # Eq. 12's momentum term (optional): `momentum_buf` is the newest u, handled like the residual
        self.m = momentum
        if momentum is not None:
            assert not in_place, "momentum correction needs the two-arena form"
            self.momentum_buf = torch.zeros(n, dtype=torch.float32, device=dev)
            self.momentum_next = torch.zeros(n, dtype=torch.float32, device=dev)
        self.out_idx = torch.zeros(max(1, self.plan.out_capacity), dtype=torch.int32, device=dev)
        self.out_val = torch.zeros(max(1, self.plan.out_capacity), dtype=torch.float32, device=dev)
        self.out_counts = torch.zeros(L, dtype=torch.int32, device=dev)
        self.want_centres = want_centres
        self.out_centre_idx = (torch.zeros(max(1, self.plan.centre_capacity), dtype=torch.int32,
                                           device=dev) if want_centres else None)
        self.out_centre_counts = torch.zeros(L, dtype=torch.int32, device=dev)
        self.workspace = torch.zeros(self.plan.workspace_bytes, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.offsets = [self.plan.layer_offset(l) for l in range(L)]
        self.sizes = [self.plan.layer_elems(l) for l in range(L)]

    # ---- host <-> arena
    def pack(self, arrays: Sequence[np.ndarray], arena: torch.Tensor) -> None:
        host = np.zeros(self.plan.total_elems, dtype=np.float32)
        for a, off, sz in zip(arrays, self.offsets, self.sizes):
            host[off:off + sz] = np.asarray(a, dtype=np.float32).reshape(-1)
        arena.copy_(torch.from_numpy(host))

    def unpack(self, arena: torch.Tensor) -> List[np.ndarray]:
        host = arena.cpu().numpy()
        return [host[off:off + sz].reshape(sh).copy()
                for off, sz, sh in zip(self.offsets, self.sizes, self.shapes)]

    def set_grad(self, arrays):
        self.pack(arrays, self.grad)

    def set_residual(self, arrays):
        self.pack(arrays, self.residual)

    # ---- calls
    def set_ratios(self, ratios: Sequence[float]) -> None:
        """New per-layer keep ratios (the per-epoch refresh); output buffers grow if they have to."""
        binding.rsdgc_plan_set_ratios(self.plan, ratios)
        dev = self.device
        if self.plan.out_capacity > self.out_idx.numel():
            self.out_idx = torch.zeros(self.plan.out_capacity, dtype=torch.int32, device=dev)
            self.out_val = torch.zeros(self.plan.out_capacity, dtype=torch.float32, device=dev)
        if self.want_centres and self.plan.centre_capacity > self.out_centre_idx.numel():
            self.out_centre_idx = torch.zeros(self.plan.centre_capacity, dtype=torch.int32, device=dev)

    def set_momentum(self, arrays):
        self.pack(arrays, self.momentum_buf)

    def compress(self, stream=None) -> None:
        if self.m is not None:
            binding.rsdgc_compress_momentum(self.plan, self.grad, self.momentum_buf, self.momentum_next,
                                            self.m, self.residual, self.residual_next, self.out_idx,
                                            self.out_val, self.out_counts, self.workspace,
                                            self.out_centre_idx,
                                            self.out_centre_counts if self.want_centres else None, stream)
            self.residual, self.residual_next = self.residual_next, self.residual
            self.momentum_buf, self.momentum_next = self.momentum_next, self.momentum_buf
            return
        target = self.residual if self.in_place else self.residual_next
        binding.rsdgc_compress(self.plan, self.grad, self.residual, target, self.out_idx, self.out_val,
                               self.out_counts, self.workspace, self.out_centre_idx,
                               self.out_centre_counts if self.want_centres else None, stream)
        if not self.in_place:
            self.residual, self.residual_next = self.residual_next, self.residual

    def nsi(self, use_residual: bool = True) -> List[np.ndarray]:
        out = torch.zeros_like(self.grad)
        binding.rsdgc_nsi(self.plan, self.grad, self.residual if use_residual else None, out,
                          self.workspace)
        torch.cuda.synchronize()
        return self.unpack(out)

    def decompress(self, accumulate: bool = False, dense: Optional[torch.Tensor] = None) -> torch.Tensor:
        if dense is None:
            dense = torch.full_like(self.grad, 7.0)   # non-zero: overwrite mode must clear it
        binding.rsdgc_decompress(self.plan, self.out_idx, self.out_val, self.out_counts, dense,
                                 accumulate, self.workspace)
        return dense

    # ---- results on the host
    def results(self):
        """Per layer: (idx uint32, val float32, centres uint32, n_centres)."""
        torch.cuda.synchronize()
        counts = self.out_counts.cpu().numpy()
        ccounts = self.out_centre_counts.cpu().numpy()
        idx = self.out_idx.cpu().numpy().view(np.uint32)
        val = self.out_val.cpu().numpy()
        cidx = self.out_centre_idx.cpu().numpy().view(np.uint32) if self.want_centres else None
        out = []
        for l in range(self.plan.n_layers):
            o, n = self.plan.out_offset(l), int(counts[l])
            co, k = self.plan.centre_offset(l), self.plan.layer_k(l)
            out.append((idx[o:o + n].copy(), val[o:o + n].copy(),
                        cidx[co:co + k].copy() if cidx is not None else None, int(ccounts[l])))
        return out


class BlockSession:
    """The same plumbing for the block reading (rsdgc_plan_blocks / rsdgc_compress_blocks)."""

    def __init__(self, shapes, p: int, alpha: float, ratios: Sequence[float],
                 p_per_layer: Optional[Sequence[int]] = None, device: str = "cuda:0", in_place: bool = False,
                 work_feed: int = binding.FEED_AUTO, momentum: Optional[float] = None):
        self.shapes = [(int(r), int(c)) for r, c in shapes]
        self.p_list = [int(x) for x in p_per_layer] if p_per_layer is not None else [int(p)] * len(self.shapes)
        self.plan = binding.rsdgc_plan_blocks(self.shapes, p, alpha, ratios, p_per_layer)
        if work_feed != binding.FEED_AUTO:
            binding.rsdgc_plan_set_work_feed(self.plan, work_feed)
        self.device = torch.device(device)
        dev = self.device
        n, L = self.plan.total_elems, self.plan.n_layers
        self.grad = torch.zeros(n, dtype=torch.float32, device=dev)
        self.residual = torch.zeros(n, dtype=torch.float32, device=dev)
        self.in_place = in_place
        self.residual_next = None if in_place else torch.zeros(n, dtype=torch.float32, device=dev)
        self.m = momentum
        self.momentum_buf = self.momentum_next = None
        if momentum is not None:
            self.momentum_buf = torch.zeros(n, dtype=torch.float32, device=dev)
            self.momentum_next = None if in_place else torch.zeros(n, dtype=torch.float32, device=dev)
        self.out_blocks = torch.zeros(max(1, self.plan.centre_capacity), dtype=torch.int32, device=dev)
        self.out_val = torch.zeros(max(1, self.plan.out_capacity), dtype=torch.float32, device=dev)
        self.out_counts = torch.zeros(L, dtype=torch.int32, device=dev)
        self.workspace = torch.zeros(self.plan.workspace_bytes, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.offsets = [self.plan.layer_offset(l) for l in range(L)]
        self.sizes = [self.plan.layer_elems(l) for l in range(L)]

    pack = Session.pack
    unpack = Session.unpack

    def set_grad(self, arrays):
        self.pack(arrays, self.grad)

    def set_residual(self, arrays):
        self.pack(arrays, self.residual)

    def set_momentum(self, arrays):
        self.pack(arrays, self.momentum_buf)

    def compress(self, stream=None) -> None:
        target = self.residual if self.in_place else self.residual_next
        if self.m is not None:
            u_target = self.momentum_buf if self.in_place else self.momentum_next
            binding.rsdgc_compress_blocks_momentum(self.plan, self.grad, self.momentum_buf, u_target, self.m,
                                                   self.residual, target, self.out_blocks, self.out_val,
                                                   self.out_counts, self.workspace, stream)
            if not self.in_place:
                self.momentum_buf, self.momentum_next = self.momentum_next, self.momentum_buf
        else:
            binding.rsdgc_compress_blocks(self.plan, self.grad, self.residual, target, self.out_blocks,
                                          self.out_val, self.out_counts, self.workspace, stream)
        if not self.in_place:
            self.residual, self.residual_next = self.residual_next, self.residual

    def decompress(self, accumulate: bool = False, dense: Optional[torch.Tensor] = None) -> torch.Tensor:
        if dense is None:
            dense = torch.full_like(self.grad, 7.0)
        binding.rsdgc_decompress_blocks(self.plan, self.out_blocks, self.out_val, self.out_counts, dense,
                                        accumulate, self.workspace)
        return dense

    def results(self):
        """Per layer: (kept block indices uint32, values float32 with p*p per block)."""
        torch.cuda.synchronize()
        counts = self.out_counts.cpu().numpy()
        blocks = self.out_blocks.cpu().numpy().view(np.uint32)
        val = self.out_val.cpu().numpy()
        out = []
        for l in range(self.plan.n_layers):
            n, pp = int(counts[l]), self.p_list[l] ** 2
            bo, vo = self.plan.centre_offset(l), self.plan.out_offset(l)
            out.append((blocks[bo:bo + n].copy(), val[vo:vo + n * pp].copy()))
        return out
