#!/usr/bin/env python3
"""Benchmark of the beamSearch hot path on one MI355X.

Default workload (the one the headline metric is quoted on): N = 1,000,000 base
vectors, d = 128, uint8, 256-component Gaussian mixture; 10,000 queries from the
same mixture; Vamana graph R = 64, L_build = 128, alpha = 1.2 built on the GPU
by batch insertion; search k = 10 with exact int32 L2.  A "step" is one
jx_search call over the whole 10,000-query batch at the smallest beam width L
whose recall@10 against brute force is >= 0.95.

    python bench.py                      # workload 2 (default)
    python bench.py --workload 3         # N=1M d=960 fp32, 4-bit RaBitQ + exact re-rank of 40
    python bench.py --workload 4         # N=1M d=1536 fp32 unit norm, 1-bit RaBitQ + re-rank of 40
    python bench.py --workload 5 --n 10000000   # streaming inserts of 100,000, a query batch every 1M

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

HBM_PEAK_GBS = 8000.0
# HBM-side bytes of one timed launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this same command
# (profiles/beam_search_u8_N1M_L96.md); reported only when the run has the same shape.
MEASURED_TRAFFIC = {(2, 1_000_000, 10_000, 96): 2.985e9 + 1.92e6,
                    (3, 1_000_000, 10_000, 512): 4.765e10 + 3.85e6,   # profiles/build_search_f32_d960_4bit_N1M.md
                    (4, 1_000_000, 10_000, 512): 2.087e10 + 3.85e6}   # profiles/build_search_f32_d1536_1bit_N1M.md

SPEC = {
    2: dict(d=128, u8=True, bits=0, sweep=[16, 24, 32, 48, 64, 96, 128, 256], kernel="beam_search_kernel<u8>",
            text="d=128 uint8 256-component Gaussian mixture, search k=10 exact int32 L2"),
    3: dict(d=960, u8=False, bits=4, sweep=[64, 96, 128, 192, 256, 384, 512], kernel="beam_search_kernel<4-bit RaBitQ>",
            text="d=960 float32 128-component anisotropic mixture, 4-bit RaBitQ codes (B_q=8), exact fp32 re-rank of 40, k=10"),
    4: dict(d=1536, u8=False, bits=1, sweep=[64, 96, 128, 192, 256, 384, 512], kernel="beam_search_kernel<1-bit RaBitQ>",
            text="d=1536 float32 unit-norm 512-component mixture, 1-bit RaBitQ codes (B_q=4), exact fp32 re-rank of 40, k=10"),
}
SPEC[6] = dict(d=96, u8=False, bits=0, sweep=[16, 24, 32, 48, 64, 96, 128, 256], kernel="beam_search_kernel<f32>",
               text="d=96 float32 unit-norm 256-component anisotropic mixture (Deep-like), search k=10 exact fp32 L2")
SPEC[7] = dict(d=200, u8=False, bits=0, sweep=[16, 24, 32, 48, 64, 96, 128, 256], kernel="beam_search_kernel<f32>", mips=True,
               text="d=200 float32 embeddings of varying norm (Text2Image-like), inner-product search through one extra "
                    "dimension (204 stored), k=10 exact fp32 L2 on the augmented vectors")
SPEC[8] = dict(d=128, u8=True, bits=4, sweep=[48, 64, 96, 128, 192, 256], kernel="beam_search_kernel<4-bit RaBitQ>",
               text="workload 2's uint8 data searched on 4-bit RaBitQ codes (B_q=8) with exact re-rank of 40, k=10")
SPEC[5] = dict(SPEC[2], sweep=[128], text="streaming: batches of 100,000 inserts, a 10,000-query batch at L=128 every 1M; " + SPEC[2]["text"])


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=2, choices=[2, 3, 4, 5, 6, 7, 8])
    ap.add_argument("--n", type=int, default=0, help="base vectors (0 = the workload's own: 1,000,000; 10,000,000 for the streaming workload 5)")
    ap.add_argument("--nq", type=int, default=10_000)
    ap.add_argument("--recall", type=float, default=0.95)
    ap.add_argument("--L", type=int, default=0, help="force the beam width (0 = smallest with recall >= target)")
    ap.add_argument("--query-bits", type=int, default=0, help="B_q of the integer query (0 = 8 for 4-bit codes, 4 for 1-bit codes)")
    ap.add_argument("--cpu-queries", type=int, default=10000, help="sample size of the cpu_baseline leg (0 = skip)")
    ap.add_argument("--bits", type=int, default=0, choices=[0, 1, 2, 4, 8],
                    help="RaBitQ code width for the quantised workloads (0 = the workload's own: 4, 4, 1 for 3, 8, 4)")
    ap.add_argument("--f16", action="store_true", help="store the float workloads (3, 4) as binary16 (App. D of the paper)")
    ap.add_argument("--delete-frac", type=float, default=0.0,
                    help="after everything else: mark this fraction of the vertices deleted, consolidate, and report "
                         "rates, queries/s and recall before / after (Sec. 4.6, Table 2 of the paper)")
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
    wl = args.workload
    sp = SPEC[wl]
    R, L_build, alpha, k, d = 64, 128, 1.2, 10, sp["d"]
    n, nq = args.n or (10_000_000 if args.workload == 5 else 1_000_000), args.nq
    if args.bits and sp["bits"]:
        sp = dict(sp, bits=args.bits, kernel=f"beam_search_kernel<{args.bits}-bit RaBitQ>",
                  text=sp["text"].replace("4-bit", f"{args.bits}-bit").replace("1-bit", f"{args.bits}-bit"))
    rabitq = sp["bits"] > 0
    if not args.query_bits:
        args.query_bits = 4 if sp["bits"] in (1, 2) else 8
    mode = jx.RABITQ if rabitq else jx.EXACT
    rerank = 4 * k if rabitq else 0
    gen_wl = 2 if wl in (5, 8) else wl

    t0 = time.time()
    q = datagen.queries(gen_wl, nq)
    dq = torch.from_numpy(q).cuda()
    # the base set goes to the GPU chunk by chunk (the float workloads are several GB)
    f16 = args.f16 and not sp["u8"]
    tdt = torch.uint8 if sp["u8"] else (torch.float16 if f16 else torch.float32)
    dx = torch.empty((n, d), dtype=tdt, device="cuda")
    step = 16 * datagen.CHUNK
    for s0 in range(0, n, step):
        m = min(step, n - s0)
        dx[s0:s0 + m] = torch.from_numpy(datagen.base(gen_wl, m, start=s0)).cuda().to(tdt)
    if sp.get("mips"):
        # inner-product data: one extra coordinate (padded to a multiple of 4) makes it an L2 problem
        assert not f16, "--f16 is not offered for the inner-product workload"
        norms = jx.mips_augment(dx, want_norms=True)
        big_m = float(norms.max()) * (1 + 1e-6)
        d = (d + 1 + 3) // 4 * 4
        dx = jx.mips_augment(dx, big_m, dim_out=d)
        dq = jx.mips_augment(dq, big_m, is_query=True, dim_out=d)
        q = dq.cpu().numpy()
    if f16:
        dq = dq.half()
        q = q.astype(np.float16)
    log(f"[bench] workload {wl}: generated {n}x{d} base + {nq} queries in {time.time() - t0:.1f}s")

    batch = 100_000 if wl == 5 else n
    g = jx.Index(d, jx.U8 if sp["u8"] else (jx.F16 if f16 else jx.F32), R, L_build, alpha, capacity=n,
                 max_batch=max(n // 4 + 1, min(batch, n), nq), quant_bits=sp["bits"])

    def recall_of(ids, gt_np):
        a = ids.cpu().numpy()
        hit = 0
        for f, t in zip(a, gt_np):
            hit += len(set(f.tolist()) & set(t.tolist()))
        return hit / (k * len(a))

    stream_log = []
    torch.cuda.synchronize()
    t0 = time.time()
    if wl == 5:
        # streaming: batches of 100,000; every 1M points a query batch with recall against brute force
        t_ins = 0.0
        for s0 in range(0, n, batch):
            m = min(batch, n - s0)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            g.insert(dx[s0:s0 + m])
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            t_ins += dt
            done = s0 + m
            if done % 1_000_000 == 0 or done == n:
                gt_c, _ = g.bruteforce(dq, k)
                ids, _ = g.search(dq, k, 128)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(5):
                    g.search(dq, k, 128)
                torch.cuda.synchronize()
                qps_c = 5 * nq / (time.perf_counter() - t1)
                stream_log.append({"N": done, "batch_inserts_per_s": round(m / dt, 1), "qps_L128": round(qps_c, 1),
                                   "recall_at_10": round(recall_of(ids, gt_c.cpu().numpy()), 4)})
                log(f"[bench] stream {stream_log[-1]}")
        t_build = t_ins
    else:
        g.insert(dx)
        torch.cuda.synchronize()
        t_build = time.time() - t0
    log(f"[bench] built the graph on the GPU in {t_build:.2f}s ({n / t_build:,.0f} inserts/s)")

    t_quant = None
    if rabitq:
        P = torch.from_numpy(datagen.rotation(gen_wl)).cuda()
        torch.cuda.synchronize()
        t0 = time.time()
        g.quantize(sp["bits"], P, None, query_bits=args.query_bits)
        torch.cuda.synchronize()
        t_quant = time.time() - t0
        log(f"[bench] quantised ({sp['bits']} bit) in {t_quant:.2f}s")

    t0 = time.time()
    gt, _ = g.bruteforce(dq, k)
    torch.cuda.synchronize()
    log(f"[bench] brute-force ground truth in {time.time() - t0:.2f}s")
    gt_np = gt.cpu().numpy()

    sweep = {}
    L_star = args.L
    for L in sp["sweep"]:
        ids, _ = g.search(dq, k, L, mode=mode, rerank=rerank)
        torch.cuda.synchronize()
        sweep[L] = round(recall_of(ids, gt_np), 4)
        if not L_star and sweep[L] >= args.recall:
            L_star = L
            break
    if not L_star:
        L_star = sp["sweep"][-1]
    log(f"[bench] recall@10 sweep {sweep} -> L = {L_star}")

    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
    ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank, out=out)
    rec = recall_of(ids, gt_np)
    for _ in range(args.warmup):
        g.search(dq, k, L_star, mode=mode, rerank=rerank, out=out)
    torch.cuda.synchronize()
    # timed region 1: K whole jx_search calls back to back -> value
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.search(dq, k, L_star, mode=mode, rerank=rerank, out=out)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    qps = nq * args.steps / wall
    # timed region 2: the same K calls with the library's HIP events around each stage
    # (recorded on the launch stream) -> duration of the beamSearch kernel
    stage = {"rotate_ms": 0.0, "prep_ms": 0.0, "beam_ms": 0.0, "rerank_ms": 0.0}
    for _ in range(args.steps):
        _, _, st = g.search(dq, k, L_star, mode=mode, rerank=rerank, out=out, stats=True)
        for key in stage:
            stage[key] += st[key] / args.steps
    beam_ms = stage["beam_ms"]

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # What this GPU delivers for dependency-free gathers of records of the kernel's size class from a table of the
    # index's footprint: the practical ceiling for the gather part of beamSearch (context for the 8 TB/s peak).
    esize = 1 if sp["u8"] else (2 if f16 else 4)
    fam, ncp = (1 if sp["bits"] <= 2 else 4), (2 if sp["bits"] in (2, 8) else 1)
    code_chunks = ncp * ((d * fam // 8 + 15) // 16)      # 2- and 8-bit codes are two planes, each in whole chunks
    rec_bytes = d * esize if not rabitq else (code_chunks + 1) * 16
    rec_class = min((64, 128, 256, 512), key=lambda c: abs(c - rec_bytes))
    tab = torch.randint(0, 255, (n * rec_class,), dtype=torch.uint8, device="cuda")
    gid = torch.randint(0, n, ((2 << 30) // rec_class,), dtype=torch.int32, device="cuda")
    jx.probe_gather(tab, rec_class, gid)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(5):
        jx.probe_gather(tab, rec_class, gid)
    ev[1].record()
    torch.cuda.synchronize()
    gather_gbs = gid.numel() * rec_class / (ev[0].elapsed_time(ev[1]) / 5 * 1e-3) / 1e9
    del tab, gid

    # algorithmic bytes of one beamSearch launch: adjacency rows + gathered records + query records in + results out
    qrec = d * esize if not rabitq else (16 + (2 if fam == 4 else args.query_bits) * (code_chunks // ncp) * 16)
    out_k = rerank if rerank else k
    alg_bytes = st["adj_bytes"] + st["vec_bytes"] + nq * qrec + nq * out_k * 8
    achieved = alg_bytes / (beam_ms * 1e-3) / 1e9
    kernel_name = sp["kernel"]
    if sp["u8"] and 64 <= L_star <= 128 and nq <= 32768 and R <= 64 and os.environ.get("JX_BEAM_PAIR") is None:
        kernel_name = kernel_name.replace("beam_search_kernel", "beam_search_pair_kernel")  # two expansions per round
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get((wl, n, nq, L_star)) if not args.bits else None,
                "bytes_per_launch": int(alg_bytes), "kernel_ms": round(beam_ms, 4),
                "hops_per_query": round(st["hops"] / nq, 1), "dist_evals_per_query": round(st["dist_evals"] / nq, 1),
                "stage_ms": {k2: round(v, 4) for k2, v in stage.items()},
                "gather_ceiling": {"GB/s": round(gather_gbs, 1), "rec_bytes": rec_class, "table_bytes": n * rec_class,
                                   "what": "jx_probe_gather: independent random gathers, measured in this run"}}

    cpu = None
    if args.cpu_queries > 0:
        import oracle

        adj, _ = g.export_graph()
        oix = oracle.Index(d, np.uint8 if sp["u8"] else (np.float16 if f16 else np.float32), R, L_build, alpha, n)
        oix.set_graph(dx.cpu().numpy(), adj.cpu().numpy().view(np.uint32), g.size()[1])
        if rabitq:
            codes, meta, cen = [t.cpu().numpy() for t in g.export_codes()]
            oix.set_codes(sp["bits"], datagen.rotation(gen_wl), cen, codes, meta, qbits=args.query_bits)
        m = min(args.cpu_queries, nq)
        oix.search(q[:32], k, L_star, mode=1 if rabitq else 0, rerank=rerank)  # touch
        t0 = time.perf_counter()
        res = oix.search(q[:m], k, L_star, mode=1 if rabitq else 0, rerank=rerank)
        dt = time.perf_counter() - t0
        agree = float((res["ids"] == ids.cpu().numpy().view(np.uint32)[:m]).mean())
        # the oracle's batch insertion on a bounded prefix of the same base set (uint8 workloads)
        ins = None
        if sp["u8"]:
            pre = min(n, 200_000)
            oins = oracle.Index(d, np.uint8, R, L_build, alpha, pre)
            t0 = time.perf_counter()
            oins.insert(dx[:pre].cpu().numpy())
            ins = round(pre / (time.perf_counter() - t0), 1)
            del oins
        cpu = {"value": round(m / dt, 1), "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "inserts_per_s": ins, "insert_sample": f"first {min(n, 200_000):,} base vectors inserted into an empty index" if ins else None,
               "sample": f"first {m} of the {nq} queries, same graph" + (" and codes" if rabitq else "") +
                         f", same L={L_star}; fraction of result ids identical to the GPU's: {agree:.4f}"}

    cfg = {"workload": f"workload {wl}: N={n} {sp['text']}{' (stored as binary16)' if f16 else ''}; {nq} queries; Vamana R=64 L_build=128 alpha=1.2 built on the GPU",
           "L": L_star, "recall_at_10": round(rec, 4), "recall_sweep": sweep,
           "build_inserts_per_s": round(n / t_build, 1), "build_s": round(t_build, 2)}
    if t_quant is not None:
        cfg["quantize_s"] = round(t_quant, 2)
    if stream_log:
        cfg["stream"] = stream_log
    if args.delete_frac > 0:
        # batch deletion: random victims; ground truth on the live set from a wider brute force with the victims removed
        def timed_qps(reps=5):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(reps):
                g.search(dq, k, L_star, mode=mode, rerank=rerank)
            torch.cuda.synchronize()
            return reps * nq / (time.perf_counter() - t1)

        rng = np.random.Generator(np.random.PCG64(4242))
        victims = rng.choice(n, int(args.delete_frac * n), replace=False).astype(np.int64)
        dead = np.zeros(n, bool)
        dead[victims] = True
        wide, _ = g.bruteforce(dq, 64)
        wide = wide.cpu().numpy().view(np.uint32)
        gt_live = np.stack([row[~dead[row]][:k] for row in wide])
        qps_before = timed_qps()
        dv = torch.from_numpy(victims.astype(np.int32)).cuda()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        g.delete(dv)
        torch.cuda.synchronize()
        t_mark = time.perf_counter() - t1
        ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank)
        rec_marked = recall_of(ids, gt_live)
        qps_marked = timed_qps()
        t1 = time.perf_counter()
        g.consolidate()
        torch.cuda.synchronize()
        t_cons = time.perf_counter() - t1
        ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank)
        rec_after = recall_of(ids, gt_live)
        qps_after = timed_qps()
        t1 = time.perf_counter()
        ren = g.compact()
        torch.cuda.synchronize()
        t_comp = time.perf_counter() - t1
        ren = ren.cpu().numpy().view(np.uint32)
        ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank)
        rec_comp = recall_of(ids, ren[gt_live])
        qps_comp = timed_qps()
        cfg["delete"] = {"fraction": args.delete_frac, "deleted": int(victims.size), "mark_ms": round(t_mark * 1e3, 3),
                         "consolidate_s": round(t_cons, 3), "consolidate_vertices_per_s": round(n / t_cons, 1),
                         "compact_s": round(t_comp, 4),
                         "recall_at_10": {"before": round(rec, 4), "marked": round(rec_marked, 4), "consolidated": round(rec_after, 4),
                                          "compacted": round(rec_comp, 4)},
                         "queries_per_s": {"before": round(qps_before, 1), "marked": round(qps_marked, 1),
                                           "consolidated": round(qps_after, 1), "compacted": round(qps_comp, 1)}}
        log(f"[bench] delete {cfg['delete']}")
    line = {
        "metric": "queries/sec at recall@10=0.95 (10k-query batch)", "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("u4+u8" if rabitq else "u8") if sp["u8"] else ({0: "f16" if f16 else "f32"}.get(sp["bits"], f"u{sp['bits']}+f32")), "data": "synthetic",
        "config": cfg, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
