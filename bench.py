#!/usr/bin/env python3
"""Benchmark of the PacTrain compression path on one MI355X.

One step = pac_build_mask -> pac_compress for each of W workers -> pac_reduce_local ->
pac_decompress over one synthetic gradient set that is resident in HBM before timing starts.
Prints ONE JSON line: whole-step dense-gradient throughput (W*N*e bytes per step time), the
roofline figures of the dominant kernel (the gather of pac_compress, timed with events on the
launch stream inside the timed region), and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "dense-gradient GB/s through mask+compress+sum+decompress; % of HBM peak"
HBM_PEAK_GBPS = 8000.0
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "compress_c4_hbm_traffic.txt")


def measured_traffic(config_id: int):
    """HBM bytes per pac_compress launch from the committed rocprofv3 counter summary (None if absent or
    for another workload)."""
    if config_id != 4 or not os.path.exists(TRAFFIC_SUMMARY):
        return None
    for line in open(TRAFFIC_SUMMARY):
        if line.startswith("traffic_bytes_per_launch"):
            return int(float(line.split("=")[1].split()[0]))
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload id 1..8 (4 = the configuration the metric is quoted on; 6-8 = the paper's own model shapes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=int, default=1 << 28)
    ap.add_argument("--no-around", action="store_true",
                    help="skip the timings of the calls around the hot path (Mask Tracker, fused update)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one whole step in a HIP graph and time its replays (reported as graph_replay_step)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy before the timed loop: a kernel of known traffic "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    return ap.parse_args()


def algorithmic_bytes(n: int, k: int, W: int, e: int) -> dict:
    """Bytes each call must move (mask = n/8, prefix = n/16 bytes)."""
    meta = n // 8 + n // 16
    return {
        "build_mask": 4 * n + meta,
        "compress": e * n + meta + e * k,          # per launch
        "reduce_local": W * e * k + e * k,
        "decompress": e * k + meta + e * n,
    }


def cpu_baseline(wl, sample_elems: int):
    """The oracle, as it stands, on a prefix of the same workload (host cores of this machine)."""
    import numpy as np
    import oracle

    ns = min(wl.n, sample_elems)
    code = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    e = 4 if wl.dtype == "f32" else 2
    w = wl.weights[:ns].cpu().numpy()
    if code == oracle.F32:
        grads = [g[:ns].cpu().numpy() for g in wl.grads]
    else:
        import torch
        grads = [g[:ns].view(torch.int16).cpu().numpy().view(np.uint16) for g in wl.grads]
    s = wl.sparsity_at(0)[0]
    oracle.keep_count(1, 0.5)                      # load the library outside the timed region
    t0 = time.perf_counter()
    mask, prefix, k = oracle.build_mask(w, [0, ns], s)
    t1 = time.perf_counter()
    compact = [oracle.compress(g, mask, k, code) for g in grads]
    t2 = time.perf_counter()
    red = oracle.reduce_local(compact, code)
    t3 = time.perf_counter()
    oracle.decompress(red, mask, ns, code)
    t4 = time.perf_counter()
    total = t4 - t0
    return {
        "value": round(wl.workers * ns * e / total / 1e9, 4),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"first {ns} of {wl.n} flat elements as one global prune scope, s={s}, all W={wl.workers} workers, "
                  f"{total:.2f} s single-threaded",
        "stage_s": {"build_mask": round(t1 - t0, 3), "compress": round(t2 - t1, 3),
                    "reduce_local": round(t3 - t2, 3), "decompress": round(t4 - t3, 3)},
    }


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (W workers are simulated in one GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import paper_2505_18563_amd as pac
    from synth import make_workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    dev = torch.device("cuda", 0)

    wl = make_workload(args.config, device=dev)
    n, W = wl.n, wl.workers
    e = 4 if wl.dtype == "f32" else 2
    tdtype = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    nseg = len(wl.scope_offsets) - 1
    schedule = [wl.sparsity_at(t) for t in range(len(wl.sparsity_schedule))]
    k_by_phase = [sum(pac.pac_keep_count(wl.scope_offsets[i + 1] - wl.scope_offsets[i], sp[i]) for i in range(nseg))
                  for sp in schedule]
    kmax = max(k_by_phase)

    ctx = pac.PacContext(max_elems=n, max_segments=nseg, device=0)
    words = (n + 63) // 64
    mask = torch.empty(words, dtype=torch.int64, device=dev)
    prefix = torch.empty(words, dtype=torch.int32, device=dev)
    compact = [torch.empty(kmax, dtype=tdtype, device=dev) for _ in range(W)]
    red = torch.empty(kmax, dtype=tdtype, device=dev)
    dense_out = torch.empty(n, dtype=tdtype, device=dev)
    h = ctx.handle

    ev_pairs = []

    def step(t: int, timed: bool):
        sp = schedule[t % len(schedule)]
        nnz = pac.pac_build_mask(h, wl.weights, wl.scope_offsets, sp, mask, prefix)
        if timed:
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
        for w in range(W):
            pac.pac_compress(h, wl.grads[w], mask, prefix, compact[w], nnz)
        if timed:
            b.record()
            ev_pairs.append((a, b))
        pac.pac_reduce_local(h, compact, red, nnz)
        pac.pac_decompress(h, red, mask, prefix, dense_out, nnz)
        return nnz

    if args.pmc_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)            # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for t in range(args.warmup):
        step(t, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.steps):
        step(args.warmup + t, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_s = (t1 - t0) / args.steps
    compress_ms = sum(a.elapsed_time(b) for a, b in ev_pairs) / (len(ev_pairs) * W)   # per launch

    # per-call times (outside the timed region), events on the launch stream
    def time_call(fn, reps=5):
        fn()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    sp0 = schedule[0]
    nnz0 = k_by_phase[0]
    stage_ms = {
        "build_mask": time_call(lambda: pac.pac_build_mask(h, wl.weights, wl.scope_offsets, sp0, mask, prefix)),
        "compress_per_worker": time_call(lambda: pac.pac_compress(h, wl.grads[0], mask, prefix, compact[0], nnz0)),
        "reduce_local": time_call(lambda: pac.pac_reduce_local(h, compact, red, nnz0)),
        "decompress": time_call(lambda: pac.pac_decompress(h, red, mask, prefix, dense_out, nnz0)),
    }

    # The step a training loop runs while the Mask Tracker reports a stable mask: the mask of the
    # last build is reused, only compress x W, sum and decompress run.
    def cached_mask_step():
        for w in range(W):
            pac.pac_compress(h, wl.grads[w], mask, prefix, compact[w], nnz0)
        pac.pac_reduce_local(h, compact, red, nnz0)
        pac.pac_decompress(h, red, mask, prefix, dense_out, nnz0)

    pac.pac_build_mask(h, wl.weights, wl.scope_offsets, sp0, mask, prefix)
    cached_ms = time_call(cached_mask_step)

    # The whole step (mask build included) replayed from a HIP graph: what is left of the launch
    # overhead on the small, launch-bound workloads.
    graph_ms = None
    if args.graph:
        def whole_step():
            pac.pac_build_mask(h, wl.weights, wl.scope_offsets, sp0, mask, prefix)
            cached_mask_step()
        whole_step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            whole_step()
        torch.cuda.synchronize()
        graph_ms = time_call(graph.replay, reps=20)
        del graph

    # Calls around the hot path (Mask Tracker, fused weight update): timed on the same workload,
    # outside the timed region, reported with their own algorithmic bytes.
    around = {}
    if not args.no_around:
        meta = n // 8 + n // 16
        nz_out = torch.empty(1, dtype=torch.int64, device=dev)
        mask2 = torch.empty_like(mask)
        prefix2 = torch.empty_like(prefix)
        diff_out = torch.empty(1, dtype=torch.int64, device=dev)
        state_out = torch.empty(2, dtype=torch.int32, device=dev)
        pac.pac_decompress(h, red, mask, prefix, dense_out, nnz0)
        tracker = pac.MaskTracker(ctx, max_elems=n, patience=2)
        w_copy = wl.weights.clone()
        calls = {
            "mask_from_nonzero": (lambda: pac.pac_mask_from_nonzero(h, dense_out, mask2, prefix2, nz_out), e * n + meta),
            "mask_equal": (lambda: pac.pac_mask_equal(h, mask, mask2, n, diff_out), 2 * (n // 8)),
            "tracker_update": (lambda: tracker.update(mask, n, state_out), 3 * (n // 8)),
            "decompress_update": (lambda: pac.pac_decompress_update(h, red, mask, prefix, 1e-3, w_copy, nnz0),
                                  e * nnz0 + meta + 8 * n),
        }
        # ternary payload (Sec. III-D) on the compact buffers of this workload
        t_scale = torch.zeros(1, dtype=torch.float32, device=dev)
        t_packed = [torch.empty((nnz0 + 3) // 4, dtype=torch.uint8, device=dev) for _ in range(W)]
        pac.pac_absmax(h, compact[0], t_scale, count=nnz0)
        for w in range(W):
            pac.pac_ternarize(h, compact[w], t_scale, 1, w, t_packed[w], count=nnz0)
        calls["absmax_per_worker"] = (lambda: pac.pac_absmax(h, compact[0], t_scale, accumulate=True, count=nnz0), e * nnz0)
        calls["ternarize_per_worker"] = (lambda: pac.pac_ternarize(h, compact[0], t_scale, 1, 0, t_packed[0], count=nnz0),
                                         e * nnz0 + nnz0 // 4)
        calls["ternary_reduce_local"] = (lambda: pac.pac_ternary_reduce_local(h, t_packed, t_scale, red, nnz0),
                                         W * (nnz0 // 4) + e * nnz0)
        for name, (fn, nbytes) in calls.items():
            ms = time_call(fn)
            around[name] = {"ms": round(ms, 4), "algorithmic_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
        tracker.close()
        del w_copy, mask2, prefix2, t_packed

    k_avg = sum(k_by_phase[(args.warmup + t) % len(schedule)] for t in range(args.steps)) / args.steps
    alg = algorithmic_bytes(n, int(k_avg), W, e)
    step_alg = alg["build_mask"] + W * alg["compress"] + alg["reduce_local"] + alg["decompress"]
    achieved = alg["compress"] / (compress_ms * 1e-3) / 1e9

    result = {
        "metric": METRIC,
        "value": round(W * n * e / step_s / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(step_s * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"C{args.config} {wl.name}: N={n} flat elements in {len(wl.specs)} tensors, "
                        f"{wl.scope} prune s={'/'.join(str(s) for s in wl.sparsity_schedule)}, W={W} workers, "
                        f"{wl.dtype} payload, mask rebuilt every step",
            "n_elems": n, "workers": W, "nnz": int(k_avg), "prune_scopes": nseg,
        },
        "step_algorithmic_GBps": round(step_alg / step_s / 1e9, 2),
        "step_frac_of_hbm_peak": round(step_alg / step_s / 1e9 / HBM_PEAK_GBPS, 4),
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "cached_mask_step": {"ms": round(cached_ms, 4), "value": round(W * n * e / (cached_ms * 1e-3) / 1e9, 2),
                             "unit": "GB/s", "note": "mask of the last build reused (stable mask): compress x W + sum + decompress"},
        "roofline": {
            "kernel": "compress_tile_kernel<unsigned short, 7> (pac_compress)" if wl.dtype == "bf16" else "compress_tile_kernel<unsigned int, 7> (pac_compress)",
            "bound": "hbm",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": measured_traffic(args.config),
            "bytes_per_launch": alg["compress"],
            "avg_launch_ms": round(compress_ms, 5),
        },
    }
    if graph_ms is not None:
        result["graph_replay_step"] = {"ms": round(graph_ms, 4), "value": round(W * n * e / (graph_ms * 1e-3) / 1e9, 2),
                                       "unit": "GB/s", "note": "one whole step captured in a HIP graph, 20 replays"}
    if around:
        result["around_the_path"] = around
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_elems)
    ctx.close()
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
