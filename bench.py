#!/usr/bin/env python3
"""Benchmark of the beamSearch hot path on one MI355X.

Headline workload (the one the metric is quoted on): N = 1,000,000 base
vectors, d = 128, uint8, 256-component Gaussian mixture; 10,000 queries from the
same mixture; Vamana graph R = 64, L_build = 128, alpha = 1.2 built on the GPU
by batch insertion; search k = 10 with exact int32 L2.  A "step" is one
jx_search call over the whole 10,000-query batch at the smallest beam width L
whose recall@10 against brute force is >= 0.95.

    python bench.py                      # workload 2 timed as the headline; the other four configurations of the
                                         # workload list (1, 3, 4, 5) measured more briefly into config.others
    python bench.py --no-others          # the headline only
    python bench.py --workload 3         # N=1M d=960 fp32, 4-bit RaBitQ + exact re-rank of 40
    python bench.py --workload 4         # N=1M d=1536 fp32 unit norm, 1-bit RaBitQ + re-rank of 40
    python bench.py --workload 5 --n 10000000   # streaming inserts of 100,000, a query batch every 1M
    python bench.py --ablate             # kernel-variant ablation table (see ablate())

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
# rocprofv3 FETCH_SIZE / WRITE_SIZE summaries of these same commands (HBM-side bytes per launch are in the files;
# they are figures of those runs, not of this one, so the line only points to them)
TRAFFIC_SOURCE = {2: "profiles/beam_search_u8_N1M_L96.md", 3: "profiles/build_search_f32_d960_4bit_N1M.md",
                  4: "profiles/build_search_f32_d1536_1bit_N1M.md", 5: "profiles/streaming_insert_u8_N5M.md"}

SWEEP_SMALL = [10, 12, 16, 20, 24, 32, 48, 64, 96, 128, 256]
SWEEP_WIDE = [64, 96, 128, 192, 256, 384, 512]
SPEC = {
    1: dict(u8=False, bits=0, sweep=[16, 24, 32, 48, 64], R=32, L_build=64, n=10_000, nq=1_000,
            text="search k=10 exact fp32 L2, inserted in seeded random order"),
    2: dict(u8=True, bits=0, sweep=SWEEP_SMALL, text="search k=10 exact int32 L2"),
    3: dict(u8=False, bits=4, sweep=SWEEP_WIDE, text="4-bit RaBitQ codes (max-cosine rule, B_q=8), exact fp32 re-rank of 40, k=10"),
    4: dict(u8=False, bits=1, sweep=SWEEP_WIDE, text="1-bit RaBitQ codes (B_q=4), exact fp32 re-rank of 40, k=10"),
    6: dict(u8=False, bits=0, sweep=SWEEP_SMALL, text="(Deep-like) search k=10 exact fp32 L2"),
    7: dict(u8=False, bits=0, sweep=SWEEP_SMALL, mips=True,
            text="(Text2Image-like) inner-product search through one extra dimension (204 stored), k=10 exact fp32 L2 on the augmented vectors"),
    8: dict(u8=True, bits=4, sweep=[48, 64, 96, 128, 192, 256], gen=2,
            text="workload 2's uint8 data searched on 4-bit RaBitQ codes (B_q=8) with exact re-rank of 40, k=10"),
}
SPEC[5] = dict(SPEC[2], sweep=[128], gen=2, n=10_000_000,
               text="streaming: batches of 100,000 inserts, a 10,000-query batch at L=128 every 1M; " + SPEC[2]["text"])


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def generator_text(datagen, gen_wl):
    """The generator's parameters as the workload string carries them (free parameters included)."""
    s = datagen.spec(gen_wl)
    kind = s["kind"]
    if kind == "iso":
        return f"d={s['d']} float32, {s['comps']} isotropic Gaussians, centres N(0,{s['centre_std']}^2), sigma={s['sigma']}"
    if kind == "u8":
        return (f"d={s['d']} uint8, {s['comps']}-component Gaussian mixture, centres N({s['centre_mean']},{s['centre_std']}^2), "
                f"in-component covariance eigenvalues ~ i^-{s['decay']} (mean {s['sigma']}^2) in a seeded orthogonal basis, "
                f"rounded and clipped to [0,255]")
    return (f"d={s['d']} float32, {s['comps']}-component Gaussian mixture, centres N(0,{s['centre_std']}^2), covariance "
            f"eigenvalues ~ i^-{s['decay']} (mean {s['sigma']}^2) through a seeded orthogonal matrix"
            f"{', L2-normalised' if s.get('normalise') else ''}")


def recall_of(ids, gt_np, k):
    a = ids.cpu().numpy()
    hit = 0
    for f, t in zip(a, gt_np):
        hit += len(set(f.tolist()) & set(t.tolist()))
    return hit / (k * len(a))


_TWO_STREAMS = None


def measure(wl, args, headline, cand=None, extras=False):
    """Build workload `wl` on the GPU, pick L, time K search steps; returns (config, roofline, cpu_baseline, timing).
    extras: also time the listed beam widths and two batches in flight (the default run; left out of single-workload
    runs so that a profile of those holds the timed launches only)."""
    cand = cand or args.cand_mode
    import numpy as np
    import torch

    from paper_2601_07048_amd import datagen, jx

    sp = SPEC[wl]
    if headline and args.bits and sp["bits"]:
        sp = dict(sp, bits=args.bits, text=sp["text"].replace("4-bit", f"{args.bits}-bit").replace("1-bit", f"{args.bits}-bit"))
    gen_wl = sp.get("gen", wl)
    R, L_build, alpha, k = sp.get("R", 64), sp.get("L_build", 128), 1.2, 10
    d = datagen.spec(gen_wl)["d"]
    own = headline or wl == args.workload     # --n / --nq size the workload named on the command line
    n = (args.n if own and args.n else 0) or sp.get("n", 1_000_000)
    if not own and args.others_scale != 1.0:
        n = max(2000, int(n * args.others_scale))   # rehearsal of the default run at reduced sizes
    nq = (args.nq if own and args.nq else 0) or sp.get("nq", 10_000)
    steps, warmup = (args.steps, args.warmup) if headline else (min(args.steps, 10), min(args.warmup, 2))
    rabitq = sp["bits"] > 0
    query_bits = (args.query_bits if headline else 0) or (4 if sp["bits"] in (1, 2) else 8)
    mode = jx.RABITQ if rabitq else jx.EXACT
    rerank = 4 * k if rabitq else 0
    f16 = headline and args.f16 and not sp["u8"]

    t0 = time.time()
    q = datagen.queries(gen_wl, nq)
    dq = torch.from_numpy(q).cuda()
    # the base set goes to the GPU chunk by chunk (the float workloads are several GB)
    tdt = torch.uint8 if sp["u8"] else (torch.float16 if f16 else torch.float32)
    dx = torch.empty((n, d), dtype=tdt, device="cuda")
    step = 16 * datagen.CHUNK
    order = datagen.insertion_order(1, n) if wl == 1 else None
    if order is not None:
        dx.copy_(torch.from_numpy(datagen.base(gen_wl, n)[order]))
    else:
        for s0 in range(0, n, step):
            m = min(step, n - s0)
            dx[s0:s0 + m] = torch.from_numpy(datagen.base(gen_wl, m, start=s0)).cuda().to(tdt)
            if n >= 20_000_000 and (s0 // step) % 40 == 39:
                log(f"[bench] generated {s0 + m:,} of {n:,} base vectors")
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
    # one jx_insert call takes the whole base set (internal batches grow to a quarter of the index) -- or, streaming,
    # 100,000 points per call
    max_batch = max(min(batch, n), nq) if wl == 5 else max(n // 4 + 1, nq)
    cand_mode = jx.CAND_VISITED if cand == "visited" else jx.CAND_FRONTIER
    try:
        g = jx.Index(d, jx.U8 if sp["u8"] else (jx.F16 if f16 else jx.F32), R, L_build, alpha, capacity=n,
                     max_batch=max_batch, quant_bits=sp["bits"], cand_mode=cand_mode, flags=args.flags)
    except jx.JxError:
        if cand_mode != jx.CAND_VISITED:
            raise
        cand_mode = jx.CAND_FRONTIER   # the expansion-list mode is not offered for this record shape
        g = jx.Index(d, jx.U8 if sp["u8"] else (jx.F16 if f16 else jx.F32), R, L_build, alpha, capacity=n,
                     max_batch=max_batch, quant_bits=sp["bits"], cand_mode=cand_mode, flags=args.flags)

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
            if done % args.stream_every == 0 or done == n:
                gt_c, _ = g.bruteforce(dq, k)
                ids, _ = g.search(dq, k, 128)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(5):
                    g.search(dq, k, 128)
                torch.cuda.synchronize()
                qps_c = 5 * nq / (time.perf_counter() - t1)
                stream_log.append({"N": done, "batch_inserts_per_s": round(m / dt, 1), "qps_L128": round(qps_c, 1),
                                   "recall_at_10": round(recall_of(ids, gt_c.cpu().numpy(), k), 4)})
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
        g.quantize(sp["bits"], P, None, query_bits=query_bits)
        torch.cuda.synchronize()
        t_quant = time.time() - t0
        log(f"[bench] quantised ({sp['bits']} bit) in {t_quant:.2f}s")

    t0 = time.time()
    gt, _ = g.bruteforce(dq, k)
    torch.cuda.synchronize()
    log(f"[bench] brute-force ground truth in {time.time() - t0:.2f}s")
    gt_np = gt.cpu().numpy()

    def sweep_for(rr_of_L):
        sw, star = {}, 0
        for L in sp["sweep"]:
            ids, _ = g.search(dq, k, L, mode=mode, rerank=rr_of_L(L))
            torch.cuda.synchronize()
            sw[L] = round(recall_of(ids, gt_np, k), 4)
            if sw[L] >= args.recall:
                star = L
                break
        return sw, star

    forced_L = args.L if headline else 0
    sweep, L_star = sweep_for(lambda L: rerank)
    target_met = bool(L_star)
    if forced_L:
        L_star = forced_L
    elif not L_star:
        # the sweep ends below the target: time the smallest beam width within half a point of the best recall
        # (the ceiling) and say so
        best = max(sweep.values())
        L_star = min(L for L in sweep if sweep[L] >= best - 0.005)
    log(f"[bench] recall@10 sweep {sweep} -> L = {L_star}{'' if target_met or forced_L else ' (target not reached)'}")

    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))

    def timed(L, rr):
        ids, _ = g.search(dq, k, L, mode=mode, rerank=rr, out=out)
        rec = recall_of(ids, gt_np, k)
        for _ in range(warmup):
            g.search(dq, k, L, mode=mode, rerank=rr, out=out)
        torch.cuda.synchronize()
        # timed region 1: K whole jx_search calls back to back -> value; two HIP events on the launch stream (torch's
        # current stream is the one the binding hands to the library) bracket the same region
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        t1 = time.perf_counter()
        ev[0].record()
        for _ in range(steps):
            g.search(dq, k, L, mode=mode, rerank=rr, out=out)
        ev[1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t1
        region_ms = ev[0].elapsed_time(ev[1]) / steps
        # timed region 2: the same K calls, each with the library's HIP events around every stage (recorded on the
        # launch stream; the call then synchronises) -> duration of the beamSearch kernel alone
        stage = {"rotate_ms": 0.0, "prep_ms": 0.0, "beam_ms": 0.0, "rerank_ms": 0.0}
        for _ in range(steps):
            _, _, st = g.search(dq, k, L, mode=mode, rerank=rr, out=out, stats=True)
            for key in stage:
                stage[key] += st[key] / steps
        return rec, wall * 1e3 / steps, nq * steps / wall, stage, dict(st, region_ms=region_ms)

    rec, ms_per_step, qps, stage, st = timed(L_star, rerank)
    # duration of one beamSearch launch.  Exact search: a step is that one kernel, so the HIP events around the K
    # back-to-back steps of the timed region give its average launch duration (start to start, launch gap included).
    # Code search: a step is four kernels; the beamSearch share comes from the library's own events around each stage
    # in the second loop.  The isolated figure (an event pair and a synchronisation per launch) is reported beside it:
    # for sub-millisecond kernels it is longer, the GPU idles between launches and the counters' atomics are on.
    beam_ms = stage["beam_ms"] if rabitq else st["region_ms"]

    if headline and args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    esize = 1 if sp["u8"] else (2 if f16 else 4)
    fam, ncp = (1 if sp["bits"] <= 2 else 4), (2 if sp["bits"] in (2, 8) else 1)
    code_chunks = ncp * ((d * fam // 8 + 15) // 16)      # 2- and 8-bit codes are two planes, each in whole chunks
    rec_bytes = d * esize if not rabitq else (code_chunks + 1) * 16
    gather = None
    if headline:
        # What this GPU delivers for dependency-free gathers of records of the kernel's size class from a table of
        # the index's footprint: the practical ceiling for the gather part of beamSearch (context for the 8 TB/s peak)
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
        gather = {"GB/s": round(gather_gbs, 1), "rec_bytes": rec_class, "table_bytes": n * rec_class,
                  "what": "jx_probe_gather: independent random gathers, measured in this run"}

    # algorithmic bytes of one beamSearch launch: adjacency rows + gathered records + query records in + results out
    qrec = d * esize if not rabitq else (16 + (2 if fam == 4 else query_bits) * (code_chunks // ncp) * 16)
    out_k = rerank if rerank else k
    alg_bytes = st["adj_bytes"] + st["vec_bytes"] + nq * qrec + nq * out_k * 8
    achieved = alg_bytes / (beam_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": st["beam_kernel"], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "traffic_source": ("profiles/beam_search_u8_N1M_L16.md" if wl == 2 and cand_mode == jx.CAND_VISITED else TRAFFIC_SOURCE.get(wl)),
                "bytes_per_launch": int(alg_bytes), "kernel_ms": round(beam_ms, 4),
                "kernel_ms_source": ("HIP events around each stage inside the library, second loop of the same K calls" if rabitq else
                                     "HIP events on the launch stream around the K back-to-back launches of the timed region, divided by K"),
                "kernel_ms_isolated": round(stage["beam_ms"], 4),
                "hops_per_query": round(st["hops"] / nq, 1), "dist_evals_per_query": round(st["dist_evals"] / nq, 1),
                "stage_ms": {k2: round(v, 4) for k2, v in stage.items()}}
    if gather:
        roofline["gather_ceiling"] = gather

    cfg = {"workload": f"workload {wl}: N={n} {generator_text(datagen, gen_wl)}; {sp['text']}{' (stored as binary16)' if f16 else ''}; "
                       f"{nq} queries; Vamana R={R} L_build={L_build} alpha=1.2 built on the GPU, robustPrune candidates = "
                       f"{'expansion list V (Alg. 4 as printed)' if cand_mode == jx.CAND_VISITED else 'final frontier F (Alg. 2 output)'}, batch_growth=0.25",
           "L": L_star, "recall_at_10": round(rec, 4), "recall_target": args.recall, "recall_target_met": bool(rec >= args.recall),
           "recall_sweep": sweep, "build_inserts_per_s": round(n / t_build, 1), "build_s": round(t_build, 2)}
    if t_quant is not None:
        cfg["quantize_s"] = round(t_quant, 2)
    if extras and headline and wl == 2 and not forced_L:
        # the beam widths the workload text lists, each timed like the headline (K back-to-back steps)
        listed = []
        for Lb in (32, 64, 128, 256):
            rec_b, ms_b, qps_b, _, st_b = timed(Lb, rerank)
            by = st_b["adj_bytes"] + st_b["vec_bytes"] + nq * qrec + nq * k * 8
            listed.append({"L": Lb, "recall_at_10": round(rec_b, 4), "queries_per_s": round(qps_b, 1), "ms_per_step": round(ms_b, 4),
                           "kernel": st_b["beam_kernel"], "kernel_ms": round(st_b["region_ms"], 4),
                           "frac": round(by / st_b["region_ms"] / 1e6 / HBM_PEAK_GBS, 4)})
        cfg["listed_beam_widths"] = listed
    if extras and not rabitq:
        # Not the headline figure: the same K steps issued alternately on two streams (separate result buffers), as a
        # server with two batches in flight would.  A single launch ends with a few long searches on an emptying
        # machine; the next batch's launch fills that drain.  Exact-mode searches touch only their inputs and outputs,
        # so they may overlap; code searches share the index workspace and may not.
        global _TWO_STREAMS
        if _TWO_STREAMS is None:   # one pair for the whole run: streams share a few hardware queues
            _TWO_STREAMS = [torch.cuda.Stream(), torch.cuda.Stream()]
        streams = _TWO_STREAMS
        outs = [out, (torch.empty_like(out[0]), torch.empty_like(out[1]))]
        best = None
        reps = max(steps, 20)
        for _ in range(3):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for i in range(reps):
                with torch.cuda.stream(streams[i & 1]):
                    g.search(dq, k, L_star, mode=mode, rerank=rerank, out=outs[i & 1])
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            best = dt if best is None else min(best, dt)
        same = bool(torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]))
        cfg["two_batches_in_flight"] = {"queries_per_s": round(nq * reps / best, 1), "ms_per_step": round(best * 1e3 / reps, 4),
                                        "steps": reps, "streams": 2, "results_equal": same,
                                        "what": "max(K, 20) steps issued alternately on two HIP streams; best of 3 repetitions; "
                                                "context for the drain of a single launch, never the headline value"}
    if stream_log:
        cfg["stream"] = stream_log
    if rabitq and not target_met and not forced_L:
        # the same search with every frontier entry re-ranked: shows whether the 40-candidate re-rank is what caps recall
        sweep_all, L_all = sweep_for(lambda L: L)
        if L_all:
            rec_a, ms_a, qps_a, stage_a, st_a = timed(L_all, L_all)
            bytes_a = st_a["adj_bytes"] + st_a["vec_bytes"] + nq * qrec + nq * L_all * 8
            cfg["rerank_whole_frontier"] = {"L": L_all, "rerank": L_all, "recall_at_10": round(rec_a, 4), "recall_sweep": sweep_all,
                                            "queries_per_s": round(qps_a, 1), "ms_per_step": round(ms_a, 4),
                                            "stage_ms": {k2: round(v, 4) for k2, v in stage_a.items()},
                                            "roofline": {"kernel": st_a["beam_kernel"], "bytes_per_launch": int(bytes_a),
                                                         "kernel_ms": round(stage_a["beam_ms"], 4),
                                                         "achieved": round(bytes_a / stage_a["beam_ms"] / 1e6, 1),
                                                         "frac": round(bytes_a / stage_a["beam_ms"] / 1e6 / HBM_PEAK_GBS, 4)}}
        else:
            cfg["rerank_whole_frontier"] = {"recall_sweep": sweep_all, "recall_target_met": False}
        log(f"[bench] re-rank of the whole frontier: {cfg['rerank_whole_frontier']}")

    cpu = None
    if headline and args.cpu_queries > 0:
        import oracle

        adj, _ = g.export_graph()
        oix = oracle.Index(d, np.uint8 if sp["u8"] else (np.float16 if f16 else np.float32), R, L_build, alpha, n)
        oix.set_graph(dx.cpu().numpy(), adj.cpu().numpy().view(np.uint32), g.size()[1])
        if rabitq:
            codes, meta, cen = [t.cpu().numpy() for t in g.export_codes()]
            oix.set_codes(sp["bits"], datagen.rotation(gen_wl), cen, codes, meta, qbits=query_bits)
        m = min(args.cpu_queries, nq)
        oix.search(q[:32], k, L_star, mode=1 if rabitq else 0, rerank=rerank)  # touch
        t1 = time.perf_counter()
        res = oix.search(q[:m], k, L_star, mode=1 if rabitq else 0, rerank=rerank)
        dt = time.perf_counter() - t1
        ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank, out=out)
        agree = float((res["ids"] == ids.cpu().numpy().view(np.uint32)[:m]).mean())
        # the oracle's batch insertion on a bounded prefix of the same base set (uint8 workloads)
        ins = None
        if sp["u8"]:
            pre = min(n, 200_000)
            oins = oracle.Index(d, np.uint8, R, L_build, alpha, pre)
            t1 = time.perf_counter()
            oins.insert(dx[:pre].cpu().numpy())
            ins = round(pre / (time.perf_counter() - t1), 1)
            del oins
        cpu = {"value": round(m / dt, 1), "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "inserts_per_s": ins, "insert_sample": f"first {min(n, 200_000):,} base vectors inserted into an empty index" if ins else None,
               "sample": f"first {m} of the {nq} queries, same graph" + (" and codes" if rabitq else "") +
                         f", same L={L_star}; fraction of result ids identical to the GPU's: {agree:.4f}"}
        del oix

    if headline and args.delete_frac > 0:
        cfg["delete"] = delete_leg(g, dq, gt_np, n, nq, k, L_star, mode, rerank, rec, args.delete_frac)
    dtype = ("u4+u8" if rabitq else "u8") if sp["u8"] else ({0: "f16" if f16 else "f32"}.get(sp["bits"], f"u{sp['bits']}+f32"))
    timing = {"value": round(qps, 1), "ms_per_step": round(ms_per_step, 4), "dtype": dtype, "steps": steps, "warmup": warmup}
    del g, dx, dq
    torch.cuda.empty_cache()
    return cfg, roofline, cpu, timing


def delete_leg(g, dq, gt_np, n, nq, k, L_star, mode, rerank, rec, frac):
    """Batch deletion: random victims; ground truth on the live set from a wider brute force with the victims removed."""
    import numpy as np
    import torch

    def timed_qps(reps=5):
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(reps):
            g.search(dq, k, L_star, mode=mode, rerank=rerank)
        torch.cuda.synchronize()
        return reps * nq / (time.perf_counter() - t1)

    rng = np.random.Generator(np.random.PCG64(4242))
    victims = rng.choice(n, int(frac * n), replace=False).astype(np.int64)
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
    rec_marked = recall_of(ids, gt_live, k)
    qps_marked = timed_qps()
    t1 = time.perf_counter()
    g.consolidate()
    torch.cuda.synchronize()
    t_cons = time.perf_counter() - t1
    ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank)
    rec_after = recall_of(ids, gt_live, k)
    qps_after = timed_qps()
    t1 = time.perf_counter()
    ren = g.compact()
    torch.cuda.synchronize()
    t_comp = time.perf_counter() - t1
    ren = ren.cpu().numpy().view(np.uint32)
    ids, _ = g.search(dq, k, L_star, mode=mode, rerank=rerank)
    rec_comp = recall_of(ids, ren[gt_live], k)
    qps_comp = timed_qps()
    out = {"fraction": frac, "deleted": int(victims.size), "mark_ms": round(t_mark * 1e3, 3),
           "consolidate_s": round(t_cons, 3), "consolidate_vertices_per_s": round(n / t_cons, 1),
           "compact_s": round(t_comp, 4),
           "recall_at_10": {"before": round(rec, 4), "marked": round(rec_marked, 4), "consolidated": round(rec_after, 4),
                            "compacted": round(rec_comp, 4)},
           "queries_per_s": {"before": round(qps_before, 1), "marked": round(qps_marked, 1),
                             "consolidated": round(qps_after, 1), "compacted": round(qps_comp, 1)}}
    log(f"[bench] delete {out}")
    return out


def ablate(args):
    """Kernel-variant ablation (the paper's Sec. 6.5 "Ablation study" and its Block-Size, Tile Size and Load
    microbenchmarks, on this kernel's own axes): every variant is a JX_FLAG_* switch of the library, returns the same
    results as the default (the parity tests check that), and is timed here on the same index, one 10,000-query
    beamSearch launch per cell, median of `--steps` launches (HIP events around the kernel)."""
    import numpy as np
    import torch

    from paper_2601_07048_amd import datagen, jx

    k, nq, reps = 10, 10_000, max(3, min(args.steps, 7))
    scale = args.others_scale

    def build(wl, bits=0):
        d = datagen.spec(wl)["d"]
        u8 = datagen.spec(wl)["dtype"] == np.uint8
        n = max(2000, int(1_000_000 * scale))
        dx = torch.empty((n, d), dtype=torch.uint8 if u8 else torch.float32, device="cuda")
        step = 16 * datagen.CHUNK
        for s0 in range(0, n, step):
            m = min(step, n - s0)
            dx[s0:s0 + m] = torch.from_numpy(datagen.base(wl, m, start=s0)).cuda()
        dq = torch.from_numpy(datagen.queries(wl, nq)).cuda()
        g = jx.Index(d, jx.U8 if u8 else jx.F32, 64, 128, 1.2, capacity=n, max_batch=max(n // 4 + 1, nq), quant_bits=bits,
                     cand_mode=jx.CAND_VISITED if args.cand_mode == "visited" else jx.CAND_FRONTIER)
        g.insert(dx)
        if bits:
            g.quantize(bits, torch.from_numpy(datagen.rotation(wl)).cuda(), None, query_bits=8 if bits == 4 else 4)
        gt = g.bruteforce(dq, k)[0].cpu().numpy()
        torch.cuda.synchronize()
        log(f"[ablate] workload {wl}: N={n} built")
        return g, dq, gt, n

    def cell(g, dq, gt, L, flags, mode=0, rerank=0):
        g.set_flags(flags)
        try:
            ids, _ = g.search(dq, k, L, mode=mode, rerank=rerank)
            ms = []
            for _ in range(reps):
                _, _, st = g.search(dq, k, L, mode=mode, rerank=rerank, stats=True)
                ms.append(st["beam_ms"])
        finally:
            g.set_flags(0)
        m = float(np.median(ms))
        return {"L": L, "kernel": st["beam_kernel"], "beam_ms": round(m, 4), "queries_per_s_kernel": round(nq / m * 1e3, 1),
                "dist_evals_per_query": round(st["dist_evals"] / nq, 1), "hops_per_query": round(st["hops"] / nq, 1),
                "recall_at_10": round(recall_of(ids, gt, k), 4)}

    table = []

    def rows(tag, g, dq, gt, Ls, variants, mode=0, rerank=0):
        for name, fl in variants:
            for L in Ls:
                table.append(dict({"workload": tag, "variant": name}, **cell(g, dq, gt, L, fl, mode, min(rerank, L))))
            log(f"[ablate] {tag}: {name}: " + ", ".join(f"L={r['L']} {r['beam_ms']} ms" for r in table[-len(Ls):]))

    F = jx
    # --- 128-byte uint8 vectors (the paper's BigANN axis)
    g, dq, gt, n = build(2)
    rows(f"workload 2 (N={n}, d=128 uint8, exact)", g, dq, gt, (16, 32, 96), [
        ("default: tag table, 4 lanes x 2 chunks, chunked loads, 1 query per workgroup, two expansions per round where it applies", 0),
        ("one expansion per round", F.FLAG_NO_PAIR),
        ("visited: direct-mapped table of full ids", F.FLAG_VISITED_IDS | F.FLAG_NO_PAIR),
        ("visited: none (Alg. 2 as printed)", F.FLAG_VISITED_NONE),
        ("lanes per vector: 8 x 1 chunk", F.FLAG_LANES_WIDE | F.FLAG_NO_PAIR),
        ("lanes per vector: 2 x 4 chunks", F.FLAG_LANES_NARROW),
        ("tiled (4-byte strided) loads", F.FLAG_TILED_LOADS),
        ("2 queries per workgroup", F.FLAG_QPW_2),
        ("4 queries per workgroup", F.FLAG_QPW_4)])
    del g
    torch.cuda.empty_cache()
    # --- 3,840-byte float32 vectors (the paper's GIST axis), exact and on 4-bit codes
    g, dq, gt, n = build(3, bits=4)
    rows(f"workload 3 (N={n}, d=960 float32, exact)", g, dq, gt, (32, 128), [
        ("default: 64 lanes x 4 chunks, chunked loads, 1 wavefront per query", 0),
        ("visited: none (Alg. 2 as printed)", F.FLAG_VISITED_NONE),
        ("tiled (4-byte strided) loads", F.FLAG_TILED_LOADS),
        ("2 wavefronts per query", F.FLAG_WAVES_2),
        ("4 wavefronts per query", F.FLAG_WAVES_4)])
    rows(f"workload 3 (N={n}, d=960 float32, 4-bit RaBitQ codes + re-rank 40)", g, dq, gt, (32, 128), [
        ("default: 16 lanes x 2 chunks", 0), ("32 lanes x 1 chunk", F.FLAG_LANES_WIDE), ("visited: none (Alg. 2 as printed)", F.FLAG_VISITED_NONE)],
        mode=jx.RABITQ, rerank=40)
    del g
    torch.cuda.empty_cache()
    # --- 6,144-byte float32 vectors: wavefronts per query
    g, dq, gt, n = build(4, bits=1)
    rows(f"workload 4 (N={n}, d=1536 float32, exact)", g, dq, gt, (32, 128), [
        ("default: 64 lanes x 6 chunks, 1 wavefront per query", 0),
        ("2 wavefronts per query", F.FLAG_WAVES_2),
        ("4 wavefronts per query", F.FLAG_WAVES_4)])
    rows(f"workload 4 (N={n}, d=1536 float32, 1-bit RaBitQ codes + re-rank 40)", g, dq, gt, (32, 128), [
        ("default: 4 lanes x 3 code chunks, meta chunk apart", 0), ("16 lanes x 1 chunk", F.FLAG_LANES_WIDE),
        ("visited: none (Alg. 2 as printed)", F.FLAG_VISITED_NONE)], mode=jx.RABITQ, rerank=40)
    del g
    return {"metric": "beamSearch kernel-variant ablation: kernel time per 10,000-query launch", "unit": "ms", "n_gpus": 1,
            "launches_per_cell": reps, "data": "synthetic", "graphs_built_from": args.cand_mode, "table": table}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=2, choices=sorted(SPEC))
    ap.add_argument("--n", type=int, default=0, help="base vectors (0 = the workload's own: 1,000,000; 10,000 for workload 1; 10,000,000 for the streaming workload 5)")
    ap.add_argument("--nq", type=int, default=0, help="queries (0 = the workload's own: 10,000; 1,000 for workload 1)")
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
    ap.add_argument("--cand-mode", choices=["frontier", "visited"], default="visited",
                    help="what beamSearch hands to robustPrune during the build: the final frontier F (Alg. 2's output) or the "
                         "expansion list V (Alg. 4 as printed)")
    ap.add_argument("--flags", type=int, default=0, help="JX_FLAG_* switches of the library (include/jx.h), e.g. 1 = one expansion per round")
    ap.add_argument("--stream-every", type=int, default=1_000_000, help="streaming workload: points between two query batches")
    ap.add_argument("--no-others", action="store_true", help="skip the brief measurements of the other configurations")
    ap.add_argument("--extras", action="store_true", help="also time the listed beam widths and two batches in flight (always on in the default run)")
    ap.add_argument("--others", type=str, default="1,3,4,5", help="configurations measured briefly after the headline (default run only)")
    ap.add_argument("--others-scale", type=float, default=1.0, help="scale the sizes of the other configurations (rehearsals and tests)")
    ap.add_argument("--ablate", action="store_true", help="kernel-variant ablation instead of the benchmark (one JSON line with a table)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; every figure is single-GPU throughput (use --gpus 1)")

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.ablate:
        print(json.dumps(ablate(args)), flush=True)
        return
    with_others = args.workload == 2 and not (args.no_others or args.L or args.bits or args.f16 or args.delete_frac or args.flags)
    cfg, roofline, cpu, tm = measure(args.workload, args, headline=True, extras=with_others or args.extras)
    if with_others and args.cand_mode == "visited":
        # the same headline workload on the graph built from final frontiers (the library's default candidate
        # set): shows what the choice of robustPrune's candidate set is worth
        c, r, _, t = measure(args.workload, args, headline=False, cand="frontier", extras=True)
        cfg["graph_from_final_frontier"] = {"workload": c["workload"], "L": c["L"], "recall_at_10": c["recall_at_10"],
                                            "recall_sweep": c["recall_sweep"], "queries_per_s": t["value"], "ms_per_step": t["ms_per_step"],
                                            "steps": t["steps"], "build_inserts_per_s": c["build_inserts_per_s"],
                                            "roofline": {key: r[key] for key in ("kernel", "bytes_per_launch", "kernel_ms", "achieved", "frac")}}
        if "two_batches_in_flight" in c:
            cfg["graph_from_final_frontier"]["two_batches_in_flight"] = c["two_batches_in_flight"]
    if with_others:
        others = []
        for wl in [int(t) for t in args.others.split(",") if t]:
            t0 = time.time()
            c, r, _, t = measure(wl, args, headline=False, extras=True)
            entry = {"workload": c["workload"], "L": c["L"], "recall_at_10": c["recall_at_10"], "recall_target_met": c["recall_target_met"],
                     "queries_per_s": t["value"], "ms_per_step": t["ms_per_step"], "steps": t["steps"], "dtype": t["dtype"],
                     "recall_sweep": c["recall_sweep"], "build_inserts_per_s": c["build_inserts_per_s"],
                     "roofline": {key: r[key] for key in ("kernel", "bytes_per_launch", "kernel_ms", "achieved", "frac", "stage_ms", "traffic_source")}}
            for key in ("stream", "rerank_whole_frontier", "quantize_s", "two_batches_in_flight"):
                if key in c:
                    entry[key] = c[key]
            others.append(entry)
            log(f"[bench] workload {wl} done in {time.time() - t0:.1f}s")
        cfg["others"] = others
    met = cfg["recall_target_met"] or bool(args.L)
    line = {
        "metric": "queries/sec at recall@10=0.95 (10k-query batch)" if met else
                  f"queries/sec at the sweep's best recall@10={cfg['recall_at_10']} (10k-query batch; the 0.95 target is not reached: see config.recall_sweep)",
        "value": tm["value"], "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": tm["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": tm["dtype"], "data": "synthetic",
        "config": cfg, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
