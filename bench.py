#!/usr/bin/env python3
"""Benchmark of the beamSearch hot path on one MI355X.

Workload (the one the headline metric is quoted on): N = 1,000,000 base
vectors, d = 128, uint8, 256-component Gaussian mixture; 10,000 queries from the
same mixture; Vamana graph R = 64, L_build = 128, alpha = 1.2 built on the GPU
by batch insertion; search k = 10 with exact int32 L2.  A "step" is one
jx_search call over the whole 10,000-query batch at the smallest beam width L
whose recall@10 against brute force is >= 0.95.

Prints ONE JSON line: queries/s, the roofline record of the beamSearch kernel
(algorithmic bytes / measured duration against the 8 TB/s HBM peak) and the CPU
oracle's rate on a bounded sample of the same queries on the same graph.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

L_SWEEP = [16, 24, 32, 48, 64, 96, 128, 256]
HBM_PEAK_GBS = 8000.0
# HBM-side bytes of one timed launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this same command
# (profiles/beam_search_u8_N1M_L96.md); reported only when the run has the same shape.
MEASURED_TRAFFIC = {(1_000_000, 10_000, 96): 4.485e9 + 1.29e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--n", type=int, default=1_000_000)
    ap.add_argument("--nq", type=int, default=10_000)
    ap.add_argument("--recall", type=float, default=0.95)
    ap.add_argument("--L", type=int, default=0, help="force the beam width (0 = smallest with recall >= target)")
    ap.add_argument("--cpu-queries", type=int, default=2000, help="sample size of the cpu_baseline leg (0 = skip)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, to scale rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; every figure is single-GPU throughput (use --gpus 1)")

    import numpy as np
    import torch

    from paper_2601_07048_amd import datagen, jx

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    R, L_build, alpha, k, d = 64, 128, 1.2, 10, 128
    n, nq = args.n, args.nq

    t0 = time.time()
    x = datagen.base(2, n)
    q = datagen.queries(2, nq)
    log(f"[bench] generated {n}x{d} uint8 base + {nq} queries in {time.time() - t0:.1f}s")
    dx = torch.from_numpy(x).cuda()
    dq = torch.from_numpy(q).cuda()

    g = jx.Index(d, jx.U8, R, L_build, alpha, capacity=n, max_batch=n // 4 + 1)
    torch.cuda.synchronize()
    t0 = time.time()
    g.insert(dx)
    torch.cuda.synchronize()
    t_build = time.time() - t0
    log(f"[bench] built the graph on the GPU in {t_build:.2f}s ({n / t_build:,.0f} inserts/s)")

    t0 = time.time()
    gt, _ = g.bruteforce(dq, k)
    torch.cuda.synchronize()
    log(f"[bench] brute-force ground truth in {time.time() - t0:.2f}s")
    gt_np = gt.cpu().numpy()

    def recall(ids):
        a = ids.cpu().numpy()
        hit = 0
        for f, t in zip(a, gt_np):
            hit += len(set(f.tolist()) & set(t.tolist()))
        return hit / (k * len(a))

    sweep = {}
    L_star = args.L
    for L in L_SWEEP:
        ids, _ = g.search(dq, k, L)
        torch.cuda.synchronize()
        sweep[L] = round(recall(ids), 4)
        if not L_star and sweep[L] >= args.recall:
            L_star = L
            break
    if not L_star:
        L_star = L_SWEEP[-1]
    log(f"[bench] recall@10 sweep {sweep} -> L = {L_star}")

    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
    ids, _, st = g.search(dq, k, L_star, stats=True, out=out)
    rec = recall(ids)
    for _ in range(args.warmup):
        g.search(dq, k, L_star, out=out)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        g.search(dq, k, L_star, out=out)   # exact mode: the call is one beamSearch kernel launch
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    avg_ms = sum(kern_ms) / len(kern_ms)
    ms_per_step = wall * 1e3 / args.steps
    qps = nq * args.steps / wall

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # algorithmic bytes of one launch: adjacency rows + gathered vectors + queries in + results out
    alg_bytes = st["adj_bytes"] + st["vec_bytes"] + nq * d + nq * k * 8
    achieved = alg_bytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "beam_search_kernel<u8,T=8>", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC.get((n, nq, L_star)),
                "bytes_per_launch": int(alg_bytes), "kernel_ms": round(avg_ms, 4),
                "hops_per_query": round(st["hops"] / nq, 1), "dist_evals_per_query": round(st["dist_evals"] / nq, 1)}

    cpu = None
    if args.cpu_queries > 0:
        import oracle

        adj, _ = g.export_graph()
        oix = oracle.Index(d, np.uint8, R, L_build, alpha, n)
        oix.set_graph(x, adj.cpu().numpy().view(np.uint32), g.size()[1])
        m = min(args.cpu_queries, nq)
        oix.search(q[:64], k, L_star)  # touch
        t0 = time.perf_counter()
        res = oix.search(q[:m], k, L_star)
        dt = time.perf_counter() - t0
        same = bool((res["ids"] == ids.cpu().numpy().view(np.uint32)[:m]).all())
        cpu = {"value": round(m / dt, 1), "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {m} of the {nq} queries, same graph, same L={L_star}; ids identical to the GPU's: {same}"}

    line = {
        "metric": "queries/sec at recall@10=0.95 (10k-query batch)", "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"N={n} d=128 uint8 256-component Gaussian mixture, {nq} queries, Vamana R=64 L_build=128 "
                               f"alpha=1.2 built on the GPU, search k=10 exact int32 L2",
                   "L": L_star, "recall_at_10": round(rec, 4), "recall_sweep": sweep,
                   "build_inserts_per_s": round(n / t_build, 1), "build_s": round(t_build, 2)},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
