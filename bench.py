#!/usr/bin/env python3
"""Benchmark of the RS-DGC local gradient compressor on one MI355X.

A step is one rsdgc_compress call over all layers of the workload (accumulate, NSI,
per-layer selection, whole-neighbourhood mask, ordered compaction, residual update),
with gradient and residual already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

The default workload is the VGG-19-shaped gradient (19 weight layers, 139,740,864
float32 elements, 3x3 neighbourhoods, per-layer keep ratios averaging 2 %), seeded and
synthetic.  Only one GPU is used; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
METRIC = "gradient elements compressed/sec (full-model, 1 GPU) and % of HBM peak"

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, scaled by a copy
# kernel of known size) are not typed in here: they are read from the summaries under profiles/,
# which carry them on lines of the form
#     bench-traffic: workload=<name> variant=<two_arenas|in_place|momentum> scope=<stage name|path> bytes=<float>
# so that a summary that was not refreshed after a kernel changed can be seen (and replaced) in
# one place.  No matching line = null in the JSON.
PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic(workload: str, variant: str, scope: str):
    import glob
    import re
    pat = re.compile(r"bench-traffic:\s+workload=(\S+)\s+variant=(\S+)\s+scope=(\S+)\s+bytes=(\S+)")
    for path in sorted(glob.glob(os.path.join(PROFILES, "hbm_traffic_*.md"))):
        for line in open(path):
            m = pat.search(line)
            if m and (m.group(1), m.group(2), m.group(3)) == (workload, variant, scope):
                return float(m.group(4)), os.path.relpath(path, ROOT)
    return None, None


def stage_algorithmic_bytes(stage: str, n_elems: int, n_pairs: int, n_cand_elems: int,
                            in_place: bool, momentum: bool = False) -> float:
    """Bytes a stage has to move by its own contract (float32 data).  With two residual
    arenas the NSI passes also store v = r + g (4 more bytes per element) and the emit only
    touches the kept elements; in place the emit streams g and r again and rewrites r."""
    v_store = 0.0 if in_place else 4.0
    if momentum:              # Eq. 12 in full: read u as well, write the new u beside v
        v_store += 8.0
    if stage == "capture":    # read g, read r of the candidate-mode layers (candidates are < 1 %)
        return (8.0 + v_store) * n_cand_elems
    if stage == "first_pass":  # read g, read r, write the score map of the layers ranked on the full map
        return (12.0 + v_store) * (n_elems - n_cand_elems)   # (the sampled tiles of the others not counted)
    if stage == "emit":
        if in_place:          # read g, read r, write r, write (index, value) pairs
            return 12.0 * n_elems + 8.0 * n_pairs
        return n_elems / 8.0 + (20.0 if momentum else 16.0) * n_pairs   # mask bits; per pair: read v, write +0 (also to u), index, value
    return 0.0


def _cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_layer_all_cores(pool, workers, g, r, p, alpha, rho):
    """One layer through the oracle's own step functions, its score map cut into row bands that
    run side by side (a band plus a halo of (p-1)/2 rows gives the same windows, hence the same
    arithmetic, as the whole matrix); ranking, dilation, emit and residual as they stand."""
    import oracle
    R, C = g.shape
    h = (p - 1) // 2
    v = oracle.accumulate(r, g)
    bands = max(1, min(workers, R // 64))
    edges = [R * b // bands for b in range(bands + 1)]

    def band(b):
        a0, a1 = edges[b], edges[b + 1]
        lo, hi = max(0, a0 - h), min(R, a1 + h)
        return oracle.nsi(v[lo:hi], p, alpha)[a0 - lo:a0 - lo + (a1 - a0)]
    nsi_map = np.concatenate(list(pool.map(band, range(bands))), axis=0)
    k = oracle.keep_count(R * C, p, rho)
    centres, _ = oracle.select(nsi_map, k)
    mask = oracle.dilate(centres, R, C, p)
    idx, val = oracle.emit(v, mask)
    return idx, val, oracle.residual(v, mask)


def cpu_baseline(workload, grads, budget_elems: int = 150_000_000):
    """Times the CPU oracle as it stands on a bounded sample of the same workload: once on one
    thread (`value`), once with its step functions spread over the host's cores (`all_cores`)."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    order = sorted(range(workload.n_layers), key=lambda l: grads[l].size)
    chosen, total = [], 0
    for l in order:                      # smallest layers first, until the budget is reached
        if total + grads[l].size > budget_elems and chosen:
            break
        chosen.append(l)
        total += grads[l].size
    oracle.build()
    t0 = time.perf_counter()
    for l in chosen:
        g = grads[l]
        oracle.compress_layer(g, np.zeros_like(g), workload.p, workload.alpha, workload.ratios[l])
    dt = time.perf_counter() - t0
    # all cores: layers side by side (largest first), each layer's score map in row bands; a GPU machine
    # gives one GPU's job 16 cores whatever os.cpu_count() says
    host_cpus = os.cpu_count() or 1
    workers = max(1, min(host_cpus, 16))
    t1 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=workers) as bands, ThreadPoolExecutor(max_workers=workers) as layers:
        futs = [layers.submit(_oracle_layer_all_cores, bands, workers, grads[l], np.zeros_like(grads[l]),
                              workload.p, workload.alpha, workload.ratios[l]) for l in reversed(chosen)]
        for f in futs:
            f.result()
    dt_all = time.perf_counter() - t1
    sample = (f"{len(chosen)} of {workload.n_layers} layers of {workload.name} "
              f"({total} elements, one iteration, zero residual)")
    return {"value": total / dt, "unit": "elements/s", "cores": 1, "kind": "oracle",
            "sample": f"{sample}, {dt:.1f} s single thread",
            "all_cores": {"value": total / dt_all, "unit": "elements/s", "cores": workers,
                          "sample": f"{sample}, {dt_all:.1f} s; layers side by side, score maps in row bands, "
                                    "ranking (full sort) one thread per layer"},
            "host_cpu_count": host_cpus, "cpu_model": _cpu_model()}


def bench_blocks(args, w, grads) -> int:
    """Same contract for the block reading: K timed rsdgc_compress_blocks calls, one JSON line."""
    import torch
    from paper_2312_17530_amd.session import BlockSession
    sess = BlockSession(w.shapes, w.p, w.alpha, w.ratios, in_place=args.in_place, momentum=args.momentum)
    sess.set_grad(grads)
    stream = torch.cuda.current_stream()
    G = w.total_elems
    for _ in range(args.warmup):
        sess.compress(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sess.compress(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    counts = sess.out_counts.cpu().numpy()
    n_blocks = int(counts.sum())
    # the receiving side (Eq. 12, third line): eight nodes' block messages (eight times this node's own)
    from paper_2312_17530_amd import binding
    w_arena = torch.randn(sess.grad.numel(), dtype=torch.float32, device="cuda")
    peers = [(sess.out_blocks, sess.out_val, sess.out_counts)] * 8
    binding.rsdgc_apply_blocks(sess.plan, peers, w_arena, 0.1, sess.workspace, stream)
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    for _ in range(20):
        binding.rsdgc_apply_blocks(sess.plan, peers, w_arena, 0.1, sess.workspace, stream)
    torch.cuda.synchronize()
    apply_ms = (time.perf_counter() - t4) / 20 * 1e3
    del w_arena
    # read g, read r, write v (with momentum also read u, write u); one score per block
    alg = (20.0 if args.momentum is not None else 12.0) * G + 4.0 * G / (w.p * w.p)
    out = {
        "metric": METRIC, "value": G * args.steps / dt, "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "reading": "non-overlapping blocks", "layers": w.n_layers, "elements": G,
                   "p": w.p, "alpha": w.alpha, "blocks_kept_last_step": n_blocks,
                   "residual_update": "in_place" if args.in_place else "two_arenas", "momentum": args.momentum},
        "roofline": {"bound": "hbm", "kernel": "whole call (k_block_nsi dominates)",
                     "achieved": alg / (dt / args.steps) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg / (dt / args.steps) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes": alg},
        "apply_8_messages_ms": round(apply_ms, 5),
        "workspace_bytes": sess.plan.workspace_bytes,
    }
    if not args.no_cpu_baseline:
        import oracle
        l = max(range(w.n_layers), key=lambda i: 0 if grads[i].size > 20_000_000 else grads[i].size)
        oracle.build()
        t0 = time.perf_counter()
        oracle.compress_layer_blocks(grads[l], np.zeros_like(grads[l]), w.p, w.alpha, w.ratios[l])
        dtc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": grads[l].size / dtc, "unit": "elements/s", "cores": 1, "kind": "oracle",
                               "sample": f"layer {l} of {w.name} ({grads[l].size} elements, block reading, one "
                                         f"iteration, zero residual), {dtc:.1f} s single thread",
                               "host_cpu_count": os.cpu_count(), "cpu_model": _cpu_model()}
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="0-based index of the workload (3 = VGG-19)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not record per-stage HIP events")
    ap.add_argument("--centres", action="store_true", help="also emit the selected-centre lists")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times before the timed region "
                         "(reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--in-place", action="store_true",
                    help="update the residual in its own arena (one more streaming pass) instead of "
                         "writing the new residual to a second arena")
    ap.add_argument("--momentum", type=float, default=None,
                    help="momentum correction (Eq. 12 in full) with this factor: rsdgc_compress_momentum, "
                         "20 bytes per element instead of 12")
    ap.add_argument("--blocks", action="store_true",
                    help="the block reading (non-overlapping p x p neighbourhoods, rsdgc_compress_blocks): "
                         "prints its own JSON line and nothing else")
    ap.add_argument("--full-map", action="store_true",
                    help="force the full-score-map ranking path for every layer")
    ap.add_argument("--sequences", type=int, default=2,
                    help="how many times the warm-up + timed sequence is run, each from a fresh state "
                         "(the last one is reported; 1 = only the one of a cold process)")
    ap.add_argument("--grad-cycle", type=int, default=4,
                    help="number of different seeded gradients (iterations 0 .. N-1 of the workload's recipe) "
                         "kept in HBM and fed in turn, one per step; 1 = the same gradient every step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the compressor is per-rank and has no "
              "communication); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2312_17530_amd import binding, synth
    from paper_2312_17530_amd.session import Session

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.load()   # raises if the HIP library is missing: there is no fallback

    w = synth.config(args.config)
    grads = synth.gradients(w, 0)
    if args.blocks:
        return bench_blocks(args, w, grads)
    sess = Session(w.shapes, w.p, w.alpha, w.ratios, want_centres=args.centres,
                   path=binding.RSDGC_PATH_FULL_MAP if args.full_map else binding.RSDGC_PATH_AUTO,
                   in_place=args.in_place, momentum=args.momentum)
    sess.set_grad(grads)
    # the gradients of the following iterations, resident in HBM like the first: a training step
    # brings a new gradient every time, and the residual (Eq. 12) then grows like a random walk
    # instead of in proportion to the step count
    arenas = [sess.grad]
    for t in range(1, max(1, args.grad_cycle)):
        arenas.append(torch.empty_like(sess.grad))
        sess.pack(synth.gradients(w, t), arenas[-1])
    n_calls = 0

    def step():
        nonlocal n_calls
        sess.grad = arenas[n_calls % len(arenas)]
        n_calls += 1
        sess.compress(stream)
    G = w.total_elems
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def reset_state():
        """Back to the state of a fresh session: zero residual (and momentum), a workspace the plan has
        to prepare again (bound history and sampling window of the candidate path start over), and the
        gradient cycle at its first gradient."""
        nonlocal n_calls
        n_calls = 0
        for t in (sess.residual, sess.residual_next, getattr(sess, "momentum_buf", None),
                  getattr(sess, "momentum_next", None)):
            if t is not None:
                t.zero_()
        sess.workspace.zero_()
        binding.rsdgc_plan_forget_workspace(sess.plan)
        torch.cuda.synchronize()

    # The sequence "W untimed warm-up steps, then exactly K timed steps, from a fresh state" is run
    # args.sequences times, each from the same fresh state; the LAST one is reported as the result and
    # all of them are listed.  In a process that has just started, the GPU's power management is still
    # settling during the first few milliseconds of sustained work (the same kernels on the same data
    # run up to 15 % slower there); the first sequence absorbs that, the library's state is the same
    # in each.
    seq_ms = []
    for _ in range(max(1, args.sequences)):
        reset_state()
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        # timed region: exactly K steps, nothing but the compress calls between the two syncs
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        seq_ms.append(dt / args.steps * 1e3)

    # per-stage GPU time: the same K steps again with HIP events recorded on the stream between
    # the stages (each event costs a few microseconds, so this pass is not the one behind `value`)
    stages, n_rec, dt_events = {}, 0, None
    if not args.no_events:
        binding.rsdgc_profile_begin(sess.plan, args.steps)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt_events = time.perf_counter() - t1
        stages, n_rec = binding.rsdgc_profile_end(sess.plan)

    # the inverse (Eq. 12, third line), outside the timed region: dense[idx] = val over a cleared
    # arena, and dense[idx] += val (one call per peer message when several ranks' outputs are summed)
    dense = torch.zeros_like(sess.grad)
    decompress_ms = {}
    for name, acc in (("overwrite", False), ("accumulate", True)):
        sess.decompress(accumulate=acc, dense=dense)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(20):
            sess.decompress(accumulate=acc, dense=dense)
        torch.cuda.synchronize()
        decompress_ms[name] = (time.perf_counter() - t2) / 20 * 1e3
    del dense
    # the receiving side (Eq. 12, third line): eight nodes' messages (eight times this node's own)
    # summed and applied to a weights arena
    w_arena = torch.randn(sess.grad.numel(), dtype=torch.float32, device="cuda")
    peers = [(sess.out_idx, sess.out_val, sess.out_counts)] * 8
    binding.rsdgc_apply(sess.plan, peers, w_arena, 0.1, sess.workspace, stream)
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    for _ in range(20):
        binding.rsdgc_apply(sess.plan, peers, w_arena, 0.1, sess.workspace, stream)
    torch.cuda.synchronize()
    apply_ms = (time.perf_counter() - t4) / 20 * 1e3
    del w_arena
    # the per-epoch step (Eqs. 3-5): keep ratios from a weights arena (synthetic N(0, 0.05^2) weights)
    weights = torch.randn(sess.grad.numel(), dtype=torch.float32, device="cuda") * 0.05
    binding.rsdgc_dynamic_ratios(sess.plan, weights, 0.02, sess.workspace, stream)
    t3 = time.perf_counter()
    for _ in range(5):
        binding.rsdgc_dynamic_ratios(sess.plan, weights, 0.02, sess.workspace, stream)
    dynamic_ratios_ms = (time.perf_counter() - t3) / 5 * 1e3      # includes the wait and the read-back
    del weights

    ms_per_step = dt / args.steps * 1e3
    value = G * args.steps / dt
    counts = sess.out_counts.cpu().numpy()
    ks = [sess.plan.layer_k(l) for l in range(w.n_layers)]
    if args.centres:
        ccounts = sess.out_centre_counts.cpu().numpy()
        assert list(ccounts) == ks, "selected-centre counts differ from Eq. 11"
    assert all(k <= c <= min(k * w.p * w.p, r * cc) for k, c, (r, cc) in zip(ks, counts, w.shapes))
    n_pairs = int(counts.sum())

    roofline = None
    if stages:
        paths = binding.rsdgc_last_paths(sess.plan, sess.workspace)
        n_cand = sum(r * c for (r, c), pth in zip(w.shapes, paths) if pth in (0, 3))   # candidate path
        dom = max(("first_pass", "capture", "emit"), key=lambda s: stages.get(s, 0.0))
        dur_s = stages[dom] * 1e-3
        variant = ("in_place" if args.in_place else "momentum" if args.momentum is not None else
                   "full_map" if args.full_map else "centres" if args.centres else "two_arenas")
        traffic, traffic_src = measured_traffic(w.name, variant, dom)
        alg = stage_algorithmic_bytes(dom, G, n_pairs, n_cand, args.in_place, args.momentum is not None)
        per_elem = 20.0 if args.momentum is not None else 12.0     # whole path: read g, (u,) r; write (u,) r
        achieved = alg / dur_s / 1e9
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": traffic, "traffic_source": traffic_src,
                    "algorithmic_bytes": alg, "avg_ms": stages[dom],
                    "elements_on_candidate_path": n_cand,
                    "path_algorithmic_bytes": per_elem * G + 8.0 * n_pairs,
                    "path_frac": (per_elem * G + 8.0 * n_pairs) / (dt / args.steps) / 1e9 / HBM_PEAK_GBS}
        path_traffic, _ = measured_traffic(w.name, variant, "path")
        roofline["path_traffic"] = path_traffic      # counted bytes of all kernels of one call (None = not measured)
        roofline["path_moved_frac"] = (path_traffic / (dt / args.steps) / 1e9 / HBM_PEAK_GBS) if path_traffic else None

    out = {
        "metric": METRIC, "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "layers": w.n_layers, "elements": G, "p": w.p,
                   "alpha": w.alpha, "mean_keep_ratio": float(np.average(w.ratios, weights=[r * c for r, c in w.shapes])),
                   "pairs_emitted_last_step": n_pairs, "centre_lists": bool(args.centres),
                   "ranking_path": "full_map" if args.full_map else "auto",
                   "residual": "carried across steps, zero before the first warm-up step",
                   "gradients_cycled": len(arenas),
                   "sequences": len(seq_ms), "ms_per_step_each_sequence": [round(x, 5) for x in seq_ms],
                   "bounds_predicted_last_step": sum(1 for pth in paths if pth == 3) if stages else None,
                   "residual_update": "in_place" if args.in_place else "two_arenas",
                   "momentum": args.momentum},
        "roofline": roofline,
        "stages_ms": {k: round(v, 5) for k, v in stages.items()},
        "decompress_ms": {k: round(v, 5) for k, v in decompress_ms.items()},
        "apply_8_messages_ms": round(apply_ms, 5),
        "dynamic_ratios_ms": round(dynamic_ratios_ms, 5),
        "stages_recorded_calls": n_rec,
        "ms_per_step_with_stage_events": (dt_events / args.steps * 1e3) if dt_events else None,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, grads)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
