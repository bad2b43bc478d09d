#!/usr/bin/env python3
"""Benchmark of the PQT online query path on one MI355X.

One "step" = one pqt_query_batch over all queries of the workload (traversal, bin ranking,
gather, re-rank, top-k), queries resident in HBM.  Prints ONE JSON line: queries/s, recall
against exact brute force, per-stage times from HIP events recorded by the library on the
launch stream, the roofline of the dominant kernel, and the CPU oracle timed on a bounded
sample of the same queries.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload tiny|sift|gist|large|billion] [--w 8]
                    [--batch B]
"""
import argparse
import json
import os
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix
# integer/compare work of the bin-ranking kernel runs on the vector ALU: 256 CUs x 4 SIMD16
# x 16 lanes x 2.4 GHz = 39.3 T lane-ops/s (one 32-bit op per lane per clock)
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
VALU_ISSUE_PEAK_G = 256 * 4 * 2.4e9 / 4 / 1e9     # wave-level vector instructions per second, in G


def make_data(cfg, device):
    """Database (or None when it never exists as raw vectors), queries, and a chunk generator."""
    import numpy as np
    import torch
    from workloads import synth
    if cfg.kind == "tiny":
        X = torch.from_numpy(synth.tiny_mixture(cfg.N, d=cfg.D, seed=cfg.data_seed)).to(device)
        Y = torch.from_numpy(synth.tiny_mixture(cfg.nq, d=cfg.D, seed=cfg.query_seed)).to(device)
        return X, Y, (lambda s, n: X[s:s + n])
    if cfg.kind == "sift":
        tables = synth.sift_like_tables(cfg.D)
        Y = synth.sift_like_torch(0, cfg.nq, d=cfg.D, seed=cfg.query_seed, tables=tables, device=device)

        def chunks(s, n):
            return synth.sift_like_torch(s, n, d=cfg.D, seed=cfg.data_seed, tables=tables, device=device,
                                         chunk=1 << 19)
        X = chunks(0, cfg.N) if cfg.N <= 4_000_000 else None
        return X, Y, (chunks if X is None else (lambda s, n: X[s:s + n]))
    if cfg.kind == "gist":
        X = synth.gist_like_torch(0, cfg.N, d=cfg.D, seed=cfg.data_seed, device=device)
        Y = synth.gist_like_torch(0, cfg.nq, d=cfg.D, seed=cfg.query_seed + 100, device=device)
        return X, Y, (lambda s, n: X[s:s + n])
    raise ValueError(cfg.kind)


class ExactNN:
    """Exact nearest neighbour (Eq. 1) of every query by brute force on the GPU: a running minimum
    over database chunks (fed one by one while the index is built), ties to the smaller id.
    Measurement infrastructure, untimed."""

    def __init__(self, Y):
        import torch
        self.Y = Y
        self.yn = (Y * Y).sum(1)
        self.best_d = torch.full((Y.shape[0],), float("inf"), device=Y.device)
        self.best_i = torch.full((Y.shape[0],), -1, dtype=torch.int64, device=Y.device)

    def update(self, start, Xc):
        import torch
        xn = (Xc * Xc).sum(1)
        step = max(1, (1 << 31) // max(Xc.shape[0], 1))           # at most 8 GiB of distances at a time
        for q0 in range(0, self.Y.shape[0], step):
            sl = slice(q0, q0 + step)
            d = self.yn[sl, None] - 2.0 * (self.Y[sl] @ Xc.t()) + xn[None, :]
            dmin, imin = d.min(1)
            better = dmin < self.best_d[sl]
            self.best_d[sl] = torch.where(better, dmin, self.best_d[sl])
            self.best_i[sl] = torch.where(better, imin + start, self.best_i[sl])


def recall_at(ids, gt, xs=(1, 10, 100)):
    out = {}
    for x in xs:
        if x <= ids.shape[1]:
            out[f"R@{x}"] = float((ids[:, :x] == gt[:, None]).any(1).float().mean())
    return out


def measured_traffic(kernel, workload, w, field="bytes_per_launch"):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a copy kernel of known size), or None when there is no summary for
    this kernel and workload.  Counters cannot be read from inside this process.
    field="valu_insts_per_launch": the wave-level vector instructions per launch (SQ_INSTS_VALU)."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except OSError:
        return None
    entry = table.get(f"{workload}:w{w}:{kernel}")
    return None if entry is None else entry.get(field)


def _oracle_worker(args):
    path, Y, k, w, lo, hi, order, gpu_ids = args
    import numpy as np
    from oracle import pqt_index_io, pqt_query
    ix = pqt_index_io.read_index(path)
    t0 = time.perf_counter()
    res = []
    for q in range(lo, hi):
        tr = pqt_query.query(ix, Y[q], k, w, with_margins=False, order_method=order)
        res.append(tr.out_ids)
    work = time.perf_counter() - t0
    # untimed: a query whose ids differ from the GPU's is run again with the oracle's decision margins; it
    # counts as a decided mismatch if every set-changing decision had a relative margin above 1e-5 (then
    # fp32 rounding cannot explain the difference)
    differing = decided = 0
    if gpu_ids is not None and order != "static":
        for q in range(lo, hi):
            if not np.array_equal(res[q - lo], gpu_ids[q]):
                differing += 1
                tr = pqt_query.query(ix, Y[q], k, w, with_margins=True, order_method=order)
                decided += int(tr.margins["min"] > 1e-5)
    return work, res, differing, decided


def under_profiler():
    """rocprofv3 preloads a library that initialises the GPU in every process it starts; sixteen oracle
    workers on top of the benchmark exceed what a GPU machine allows, so the CPU baseline is skipped then."""
    env = os.environ
    return any(k.startswith(("ROCPROF", "ROCP_", "ROCPROFILER")) for k in env) or "rocprof" in env.get("LD_PRELOAD", "")


def cpu_baseline(path, Y_host, k, w, gpu_ids, budget_s=20.0, max_procs=16, order="fullsort"):
    """The CPU oracle, as it stands, on a bounded sample of the same queries and the same index
    file, one process per host core.  Also cross-checks the GPU ids on that sample."""
    import multiprocessing as mp
    import numpy as np
    cores = min(len(os.sched_getaffinity(0)), max_procs)
    # size the sample from one timed query
    t0 = time.perf_counter()
    _oracle_worker((path, Y_host, k, w, 0, 1, order, None))
    per_q = max(time.perf_counter() - t0, 1e-3)
    n = int(max(cores, min(Y_host.shape[0], budget_s / per_q * cores)))
    n -= n % cores
    n = max(n, cores) if Y_host.shape[0] >= cores else Y_host.shape[0]
    bounds = [(i * n) // cores for i in range(cores + 1)]
    jobs = [(path, Y_host, k, w, bounds[i], bounds[i + 1], order, gpu_ids) for i in range(cores) if bounds[i + 1] > bounds[i]]
    t0 = time.perf_counter()
    with mp.get_context("spawn").Pool(len(jobs)) as pool:
        outs = pool.map(_oracle_worker, jobs)
    wall = time.perf_counter() - t0
    work = max(o[0] for o in outs)            # slowest worker, excludes process start-up and index load
    ids = np.concatenate([np.stack(o[1]) for o in outs if o[1]])
    agree = float(np.mean(np.all(ids == gpu_ids[:n], axis=1)))
    return {"value": n / work, "unit": "queries/s", "cores": len(jobs), "kind": "oracle",
            "sample": f"first {n} of {Y_host.shape[0]} queries, float64 NumPy oracle, {len(jobs)} processes "
                      f"(wall {wall:.1f}s incl. start-up)",
            "single_core_queries_per_s": 1.0 / per_q,
            "gpu_ids_identical_on_sample": agree,
            "queries_differing": int(sum(o[2] for o in outs)),
            # of those, the ones whose oracle decision margins all exceed 1e-5 relative (must be 0: every
            # difference is then a near-tie that fp32 and float64 settle differently)
            "decided_mismatches": int(sum(o[3] for o in outs))}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 2000, or 20 with --batch: a step then makes many calls)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default steps // 10)")
    ap.add_argument("--workload", default="sift")
    ap.add_argument("--also", default=None, metavar="W1,W2,..",
                    help="further workloads measured after the headline one and reported as sub-records under "
                         "\"hbm_resident\" (default: large,billion -- 100M and 1B vectors, 0.8 and 8 GB of codes: indexes "
                         "that do not fit the caches; the 1B one takes a minute to build -- when the headline workload "
                         "is sift; none otherwise; pass an empty string for none)")
    ap.add_argument("--w", type=int, default=None)
    ap.add_argument("--nq", type=int, default=None, help="queries per step (default: the workload's)")
    ap.add_argument("--T", type=int, default=None, help="bin tuples examined per query (default: the workload's)")
    ap.add_argument("--C", type=int, default=None, help="candidate budget per query (default: the workload's)")
    ap.add_argument("--k", type=int, default=None, help="results per query (default: the workload's)")
    ap.add_argument("--exact", type=int, default=0, metavar="K_SHORT",
                    help="also time pqt_query_batch_exact: exact re-ranking of the first K_SHORT results (the raw "
                         "vectors stay in HBM, one byte per element for the integer-valued workloads)")
    ap.add_argument("--brute-force", action="store_true",
                    help="also time pqt_brute_force (exact k nearest neighbours on the matrix cores, the paper's strong "
                         "baseline) on the same queries")
    ap.add_argument("--batch", type=int, default=None,
                    help="queries per library call (default: all of them in one call); 1 gives a latency figure")
    ap.add_argument("--sweep-w", default="", metavar="W1,W2,..",
                    help="after the main measurement, queries/s and recall for each listed w")
    ap.add_argument("--M", type=int, default=None, help="code bytes per vector (default: the workload's)")
    ap.add_argument("--also-batches", default="", metavar="B1,B2,..",
                    help="after the main measurement, answer the same queries B per call for each listed B "
                         "(queued back to back, and one call at a time for the latency)")
    ap.add_argument("--codes", choices=("table", "pair"), default="table",
                    help="re-rank code format: one byte per sub-part naming a table entry (default), or two bytes "
                         "holding (centroid pair, lambda level) as in Sec. 3.3; with --M or --sweep-w also prints the "
                         "codes' distortion")
    ap.add_argument("--order", choices=("summed", "static"), default="summed",
                    help="bin proposal order: by summed level-2 distance (default) or the paper's fixed anisotropic "
                         "orders for ten slopes (two tree parts, unhashed bins)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline", action="store_true",
                    help="also for the 100M / 1B workloads (writes the index to a file for the oracle's processes)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 256 MiB out-of-place elementwise square roots (a streaming kernel of known traffic, "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (a batch of queries needs no second one); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    # A step takes 0.15-2 ms, and the GPU's clocks need some milliseconds of work to settle: twenty steps
    # right after the idle set-up read 8-10 % low, so the default is 2000 steps (under a second to a few
    # seconds of timed work) after 200 untimed ones.
    if args.steps is None:
        args.steps = 20 if args.batch else 2000
    if args.warmup is None:
        args.warmup = max(3, args.steps // 10)
    return args


def run_workload(args, workload, primary, peaks):
    """One workload end to end: data, index (trained and built by the library), timed steps, stage times,
    recall, rooflines.  primary: the headline workload (gets the CPU baseline and every optional extra);
    otherwise a sub-record with the timing, recall and rooflines only.  peaks: (HBM GB/s, MFMA TFLOP/s)
    measured on this machine before any timed loop."""
    import numpy as np
    import torch
    from workloads import CONFIGS
    from paper_1702_05911_amd import builder
    import paper_1702_05911_amd.binding as pqt

    cfg = CONFIGS[workload]
    if args.nq:
        cfg = cfg.with_(nq=args.nq)
    if args.T:
        cfg = cfg.with_(T=args.T)
    if args.C:
        cfg = cfg.with_(C=args.C)
    if args.k:
        cfg = cfg.with_(k=args.k)
    if args.M:
        cfg = cfg.with_(M=args.M)
    w = args.w or cfg.w
    code_format = 1 if args.codes == "pair" else 0
    code_bytes = cfg.M * (2 if code_format else 1)
    dev = torch.device("cuda", 0)
    t_setup = time.perf_counter()
    X, Y, chunks = make_data(cfg, dev)
    in_hbm_only = cfg.N > 4_000_000            # the database never exists as raw vectors: built chunk by chunk
    n_gt = min(cfg.nq, 1000) if in_hbm_only else cfg.nq     # queries with exact ground truth
    gt = ExactNN(Y[:n_gt])

    raw_dtype = torch.uint8 if cfg.kind == "sift" else torch.float32
    raw = torch.empty((cfg.N, cfg.D), dtype=raw_dtype, device=dev) if (primary and (args.exact or args.brute_force)) else None

    def observe(start, Xc):
        gt.update(start, Xc)
        if raw is not None:
            raw[start:start + Xc.shape[0]] = Xc.to(raw_dtype)
        if in_hbm_only and (start >> 20) % 16 == 0:
            print(f"[bench] built {start + Xc.shape[0]:,} of {cfg.N:,} vectors "
                  f"({time.perf_counter() - t_setup:.0f} s)", file=sys.stderr, flush=True)

    # the library's own streaming builder (pqt_builder_*): codebooks trained here on a sample, every
    # vector binned and encoded by HIP kernels, lists assembled on the GPU
    result_tables = {}
    index = builder.build_index_native(trained_out=result_tables, chunks=chunks, N=cfg.N, D=cfg.D, P=cfg.P, k1=cfg.k1, k2=cfg.k2, M=cfg.M,
                                       H=cfg.H, T=cfg.T, C=cfg.C, train_n=cfg.train_n, device=0,
                                       chunk_rows=(1 << 20) if in_hbm_only else (1 << 18), observer=observe,
                                       code_format=code_format)
    if args.order == "static":
        pqt.pqt_set_bin_order(index, pqt.PQT_ORDER_STATIC_SLOPES)
    runs = torch.diff(pqt.pqt_index_export(index, ("offsets",))["offsets"])
    occupancy = {"nonempty_slots": int((runs > 0).sum()), "max_run": int(runs.max()),
                 "mean_run_nonempty": float(runs[runs > 0].float().mean())}
    del runs
    tmp = path = None
    if primary and not (in_hbm_only and not args.cpu_baseline) and not args.no_cpu_baseline and not under_profiler():
        tmp = tempfile.mkdtemp(prefix="pqt_bench_")
        path = os.path.join(tmp, f"{cfg.name}.pqt")
        pqt.pqt_index_save(index, path)        # the oracle's processes read the same index from this file
    del X
    torch.cuda.empty_cache()
    gt = gt.best_i
    setup_s = time.perf_counter() - t_setup

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)      # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.sqrt(src, out=dst)          # the only sqrt kernel of the run: easy to find in the counter output
        torch.cuda.synchronize()
        del src, dst

    out_ids = torch.empty((cfg.nq, cfg.k), dtype=torch.int64, device=dev)
    out_d = torch.empty((cfg.nq, cfg.k), dtype=torch.float32, device=dev)
    B = args.batch or cfg.nq                   # queries per library call; one step still answers all nq

    def step():
        for o in range(0, cfg.nq, B):
            pqt.pqt_query_batch(index, Y[o:o + B], cfg.k, w, out_ids[o:o + B], out_d[o:o + B])

    # Untimed, before the W warm-up steps: the same step repeated for a third of a second.  The index build
    # that precedes leaves the GPU's clocks low, a step lasts 0.15-2 ms, and a short run (--steps 20
    # --warmup 5 is 4 ms of work) would otherwise be timed while the clocks are still rising -- 10 % below
    # what the same kernels do in a loop that has run for a moment, which is the rate a serving loop sees.
    if not args.batch:
        t_settle = time.perf_counter()
        while time.perf_counter() - t_settle < 0.3:
            for _ in range(10):
                step()
            torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps, nothing else on the stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # the same steps once more with the library's HIP events around every launch, for the stage
    # durations (the events themselves cost a few microseconds per step, so they stay out of `value`)
    pqt.pqt_set_profiling(index, True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if B == cfg.nq:
            step()
        else:
            pqt.pqt_query_batch(index, Y, cfg.k, w, out_ids, out_d)
    torch.cuda.synchronize()
    elapsed_profiled = time.perf_counter() - t0
    stage_ms, calls = pqt.pqt_stage_times(index)
    pqt.pqt_set_profiling(index, False)
    if B != cfg.nq:
        step()
        torch.cuda.synchronize()
    stage_ms = [m / max(calls, 1) for m in stage_ms][:3]

    # candidates actually gathered (for the byte accounting) via the debug taps, untimed
    _, _, taps = pqt.pqt_query_batch_debug(index, Y, cfg.k, w, taps=("n_cand", "n_slots"))
    torch.cuda.synchronize()
    mean_cand = float(taps["n_cand"].float().mean())
    mean_runs = float(taps["n_slots"].float().mean())
    rec = recall_at(out_ids[:n_gt], gt)
    rec["queries_with_ground_truth"] = n_gt
    # two tree parts, unhashed: how many tuples of the order a query needs before its runs fill C
    # (the ranking head pass stops at 32, 64 or 128; beyond that the query gets the full ranking)
    tuples_needed = None
    if cfg.P == 2 and cfg.H == (cfg.k1 * cfg.k2) ** 2:
        nsub = min(cfg.nq, 2000)
        _, _, t2 = pqt.pqt_query_batch_debug(index, Y[:nsub], cfg.k, w, taps=("slots", "n_tuples"))
        off = pqt.pqt_index_export(index, ("offsets",))["offsets"].to(torch.int64)
        sl = t2["slots"].clamp_(0, cfg.H - 1)
        lens = off[sl + 1] - off[sl]
        valid = torch.arange(cfg.T, device=dev)[None, :] < t2["n_tuples"][:, None]
        csum = torch.cumsum(lens * valid, dim=1)
        need = (csum < cfg.C).sum(dim=1) + 1            # tuples until the budget is reached (T + 1: never)
        tuples_needed = {"queries": nsub}
        for t in (32, 64, 128):
            tuples_needed[f"<={t}"] = float((need <= min(t, cfg.T)).float().mean())
        del t2, off, sl, lens, valid, csum

    # ---- algorithmic work per launch (one launch = all nq queries) -----------------------------------
    nq, R = cfg.nq, w * cfg.k2
    trav_flops = 2.0 * cfg.D * (cfg.k1 + R) * nq                       # level-1 + level-2 distance evaluations
    trav_bytes = 4.0 * cfg.D * nq                                      # queries streamed once
    # bin ranking, head pass (two tree parts): the pairs with (r1+1)(r2+1) <= 32 are sorted in blocks of 64
    # keys (21 compare-exchange steps of 32 each) and folded into the first block (a 64-wide minimum
    # plus 6 steps of 32); a second level with the 64-tuple region runs only for queries that need it and
    # is not counted.  Four parts have no head pass: the stage is the full ranking, counted as the sort
    # of T keys.
    if cfg.P == 2:
        T1 = min(cfg.T, R * R, 32)
        npairs = sum(T1 // (a + 1) for a in range(T1))
        nblk = -(-npairs // 64)
        rank_ops = nq * (nblk * 21 * 32 + (nblk - 1) * (64 + 6 * 32))
    else:
        Tn = min(cfg.T, R ** cfg.P)
        lg = max(1, (Tn - 1).bit_length())
        rank_ops = nq * (Tn // 2) * lg * (lg + 1) // 2
    rerank_bytes = nq * (mean_cand * code_bytes + cfg.k * (8 + 4 + 4) + cfg.M * cfg.k1 * 4 + mean_runs * 8)
    stages = [
        {"kernel": "traverse_kernel", "ms": stage_ms[0], "bound": "mfma", "achieved": trav_flops / (stage_ms[0] * 1e-3) / 1e12,
         "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "hbm_GBs": trav_bytes / (stage_ms[0] * 1e-3) / 1e9,
         # the two levels against their own bounds, both over the whole stage duration (they are phases of one
         # kernel): level 1 is a dense contraction on the matrix cores; level 2 is a gather of the selected
         # clusters' children, R * D floats per query, delivered from L2 through the compute units' vector L1s
         # (256 CUs x 64 B/clock x 2.4 GHz)
         "level1": {"bound": "mfma", "flops_per_launch": 2.0 * cfg.D * cfg.k1 * nq,
                    "achieved": 2.0 * cfg.D * cfg.k1 * nq / (stage_ms[0] * 1e-3) / 1e12, "peak": MFMA_FP32_PEAK_TFLOPS,
                    "unit": "TFLOP/s"},
         "level2": {"bound": "l1", "bytes_per_launch": 4.0 * cfg.D * R * nq,
                    "achieved": 4.0 * cfg.D * R * nq / (stage_ms[0] * 1e-3) / 1e9, "peak": 256 * 64 * 2.4,
                    "unit": "GB/s (cached centroid reads)",
                    "frac": 4.0 * cfg.D * R * nq / (stage_ms[0] * 1e-3) / 1e9 / (256 * 64 * 2.4)}},
        {"kernel": "rank_static_kernel" if args.order == "static" else "rank_head_kernel" if cfg.P == 2 else "rank_kernel",
         "ms": stage_ms[1], "bound": "alu",
         "achieved": rank_ops / (stage_ms[1] * 1e-3) / 1e12, "peak": VALU_PEAK_TOPS, "unit": "T compare-exchange/s",
         "note": "compare-exchanges of the first ranking level only; register/ALU work, no HBM or MFMA roofline applies"},
        {"kernel": "rerank_kernel", "ms": stage_ms[2], "bound": "hbm", "achieved": rerank_bytes / (stage_ms[2] * 1e-3) / 1e9,
         "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "note": "includes the full bin ranking of the queries the head pass leaves over (two tree parts)"},
    ]
    hbm_meas, mfma_meas = peaks                          # streaming read of 4 GiB; loop of independent MFMAs
    for s in stages:
        s["frac"] = s["achieved"] / s["peak"]
        meas = {"hbm": hbm_meas, "mfma": mfma_meas}.get(s["bound"])
        if meas:
            s["frac_of_measured_peak"] = s["achieved"] / meas
    # LDS look-ups of the re-rank scoring (M per candidate) against the LDS rate of the chip:
    # 256 CUs x 32 banks x 4 bytes x 2.4 GHz = 78.6 TB/s, i.e. 19.7 T look-ups/s without bank conflicts
    stages[2]["lds_lookups_per_s"] = nq * mean_cand * cfg.M / (stage_ms[2] * 1e-3)
    stages[2]["lds_lookup_frac"] = stages[2]["lds_lookups_per_s"] / (256 * 32 * 2.4e9)
    # Vector instruction issue: a 64-lane instruction occupies its 16-lane SIMD for 4 cycles, so the chip
    # issues at most 256 CUs x 4 SIMDs x 2.4 GHz / 4 = 614 G wave-instructions/s.  Instruction counts come
    # from the committed counter run (same workload and launch shape), durations from this run.
    if not (code_format or args.M or args.order == "static" or args.batch):
        for s in stages:
            n = measured_traffic(s["kernel"], cfg.name, w, "valu_insts_per_launch")
            if n:
                s["valu_issue"] = {"insts_per_launch": n, "achieved": n / (s["ms"] * 1e-3) / 1e9, "peak": VALU_ISSUE_PEAK_G,
                                   "unit": "G wave-instructions/s", "frac": n / (s["ms"] * 1e-3) / 1e9 / VALU_ISSUE_PEAK_G,
                                   "source": "insts_per_launch: profiles/pmc_traffic.json (rocprofv3 --pmc SQ_INSTS_VALU, "
                                             "a separate run); duration: this run"}
    dom = max(stages, key=lambda s: s["ms"])
    traffic = None if (code_format or args.M or args.order == "static") else measured_traffic(dom["kernel"], cfg.name, w)
    roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic,
                "traffic_source": None if traffic is None else
                "profiles/pmc_traffic.json (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, separate runs of the same command)",
                "launch_us": dom["ms"] * 1e3, "algorithmic_bytes_per_launch": rerank_bytes if dom["bound"] == "hbm" else None}

    ms_per_step = elapsed / args.steps * 1e3
    result = {
        "metric": "queries/sec at fixed Recall@1/@100 (1M x 128 and 1B x 128-shaped); per-stage % roofline",
        "value": cfg.nq * args.steps / elapsed, "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_with_stage_events": elapsed_profiled / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={cfg.N} D={cfg.D} nq={cfg.nq} P={cfg.P} k1={cfg.k1} k2={cfg.k2} "
                               f"M={cfg.M} H={cfg.H} w={w} T={cfg.T} C={cfg.C} k={cfg.k}" + (" codes=(pair,lambda)" if code_format else "")
                               + (" order=static-slopes" if args.order == "static" else ""),
                   "queries_per_call": B, "mean_candidates": mean_cand, "mean_runs": mean_runs, **occupancy},
        "recall": rec, "tuples_needed": tuples_needed, "stage_ms": stage_ms, "stages": stages, "roofline": roofline, "setup_s": setup_s,
        "measured_peaks": {"hbm_read_GBs": hbm_meas, "mfma_f32_TFLOPs": mfma_meas,
                           "how": "pqt_measure_peaks: 4 GiB streaming read; loop of independent v_mfma_f32_16x16x4_f32"},
    }
    if B != cfg.nq:
        result["us_per_call"] = elapsed / args.steps / (-(-cfg.nq // B)) * 1e6     # calls queued back to back
        # latency of one call: submit, then wait for its results, one call at a time
        ncalls = min(-(-cfg.nq // B), 200)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in range(ncalls):
            o = c * B
            pqt.pqt_query_batch(index, Y[o:o + B], cfg.k, w, out_ids[o:o + B], out_d[o:o + B])
            torch.cuda.synchronize()
        result["latency_us_per_call"] = (time.perf_counter() - t0) / ncalls * 1e6
    if not primary:
        result["cpu_baseline"] = None
    elif under_profiler():
        result["cpu_baseline"] = None
        print("[bench] a profiler is attached: the CPU baseline (sixteen worker processes) is skipped", file=sys.stderr)
    elif path is not None and not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(path, Y.cpu().numpy(), cfg.k, w, out_ids.cpu().numpy(),
                                              max_procs=4 if cfg.N > 200_000_000 else 16,
                                              order="static" if args.order == "static" else "fullsort")
    else:
        result["cpu_baseline"] = None
    sweep = []
    for wx in [int(v) for v in args.sweep_w.split(",") if v and primary]:
        pqt.pqt_query_batch(index, Y, cfg.k, wx, out_ids, out_d)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pqt.pqt_query_batch(index, Y, cfg.k, wx, out_ids, out_d)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        sweep.append({"w": wx, "queries_per_s": cfg.nq * args.steps / el, "ms_per_step": el / args.steps * 1e3,
                      "recall": recall_at(out_ids[:n_gt], gt)})
    if sweep:
        result["w_sweep"] = sweep
        pqt.pqt_query_batch(index, Y, cfg.k, w, out_ids, out_d)
        torch.cuda.synchronize()
    if primary and (args.M or args.sweep_w):
        # mean squared error of the stored codes against the vectors they stand for (Table 3's distortion):
        # reconstruction per Sec. 3.3 from the exported codes, on the first 100,000 database ids
        ex = pqt.pqt_index_export(index, ("ids", "codes"))
        ids_e = ex["ids"].to(torch.int64) & 0xFFFFFFFF
        pick = torch.nonzero(ids_e < 100_000).flatten()
        codes_e = ex["codes"][pick].to(torch.int64)
        Xs = chunks(0, min(100_000, cfg.N))[ids_e[pick]]
        tr = result_tables
        ds_ = cfg.D // cfg.M
        err = torch.zeros(pick.numel(), device=dev, dtype=torch.float64)
        pair_ij = torch.tensor([(i, j) for i in range(cfg.k1) for j in range(i + 1, cfg.k1)], device=dev).reshape(-1, 2)
        for m in range(cfg.M):
            p_, lo_ = (m * ds_) // (cfg.D // cfg.P), (m * ds_) % (cfg.D // cfg.P)
            cen = torch.from_numpy(tr["C1"][p_][:, lo_:lo_ + ds_]).to(dev)
            if code_format:
                ij = pair_ij[codes_e[:, 2 * m]]
                lam_ = ((codes_e[:, 2 * m + 1].float() - 96.0) / 16.0)[:, None]
                rec = (1.0 - lam_) * cen[ij[:, 0]] + lam_ * cen[ij[:, 1]]
            else:
                ti_ = torch.from_numpy(tr["tbl_i"][m].astype(np.int64)).to(dev)
                tj_ = torch.from_numpy(tr["tbl_j"][m].astype(np.int64)).to(dev)
                lam_ = torch.from_numpy(tr["tbl_lam"][m]).to(dev)[:, None]
                rec = ((1.0 - lam_) * cen[ti_] + lam_ * cen[tj_])[codes_e[:, m]]
            diff = Xs[:, m * ds_:(m + 1) * ds_] - rec
            err += (diff.double() ** 2).sum(dim=1)
        # the columns of Table 3: smallest, largest and average squared error over the vectors
        result["distortion"] = {"min": float(err.min()), "max": float(err.max()), "mean_squared_error": float(err.mean()),
                                "vectors": int(pick.numel()), "M": cfg.M, "code_bytes": code_bytes}
        del ex
    extra = []
    for Bx in [int(v) for v in args.also_batches.split(",") if v and primary]:
        ncall = -(-cfg.nq // Bx)
        reps = max(1, min(args.steps, 20000 // ncall))

        def run_all():
            for o in range(0, cfg.nq, Bx):
                pqt.pqt_query_batch(index, Y[o:o + Bx], cfg.k, w, out_ids[o:o + Bx], out_d[o:o + Bx])
        run_all()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            run_all()
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        nlat = min(ncall, 200)
        t1 = time.perf_counter()
        for c in range(nlat):
            o = c * Bx
            pqt.pqt_query_batch(index, Y[o:o + Bx], cfg.k, w, out_ids[o:o + Bx], out_d[o:o + Bx])
            torch.cuda.synchronize()
        lat = (time.perf_counter() - t1) / nlat
        extra.append({"queries_per_call": Bx, "queries_per_s": cfg.nq * reps / el,
                      "us_per_call_queued": el / reps / ncall * 1e6, "latency_us_per_call": lat * 1e6})
    if extra:
        result["batches"] = extra
    if args.exact and primary:
        # exact re-ranking of the first K_SHORT results (the paper's PQT_2): HBM-bound gather of raw rows
        ks = args.exact
        pqt.pqt_index_set_vectors(index, raw)
        for _ in range(args.warmup):
            pqt.pqt_query_batch_exact(index, Y, ks, cfg.k, w, out_ids, out_d)
        torch.cuda.synchronize()
        pqt.pqt_set_profiling(index, True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pqt.pqt_query_batch_exact(index, Y, ks, cfg.k, w, out_ids, out_d)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        ems, ecalls = pqt.pqt_stage_times(index)
        pqt.pqt_set_profiling(index, False)
        ems = [m / max(ecalls, 1) for m in ems]
        row_bytes = cfg.D * raw.element_size()
        ebytes = nq * (min(ks, mean_cand) * (row_bytes + 8) + cfg.D * 4 + cfg.k * 12)
        result["exact"] = {"k_short": ks, "value": cfg.nq * args.steps / el, "unit": "queries/s",
                           "ms_per_step": el / args.steps * 1e3, "stage_ms": ems,
                           "recall": recall_at(out_ids[:n_gt], gt), "vector_bytes": row_bytes,
                           "roofline": {"kernel": "exact_rerank_kernel", "bound": "hbm",
                                        "achieved": ebytes / (ems[3] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                                        "unit": "GB/s", "frac": ebytes / (ems[3] * 1e-3) / 1e9 / HBM_PEAK_GBS}}
    if args.brute_force and primary:
        pqt.pqt_index_set_vectors(index, raw)
        bf_ids, bf_d = pqt.pqt_brute_force(index, Y, cfg.k)          # warm-up: workspace and database norms
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(1, min(args.steps, 3))
        e0.record()
        for _ in range(reps):
            pqt.pqt_brute_force(index, Y, cfg.k, bf_ids, bf_d)
        e1.record()
        torch.cuda.synchronize()
        bf_ms = e0.elapsed_time(e1) / reps
        flops = 2.0 * cfg.nq * cfg.N * cfg.D
        result["brute_force"] = {"k": cfg.k, "value": cfg.nq / (bf_ms * 1e-3), "unit": "queries/s", "ms_per_step": bf_ms,
                                 "agrees_with_ground_truth": float((bf_ids[:n_gt, 0] == gt).float().mean()),
                                 "roofline": {"kernel": "bf_distance_kernel", "bound": "mfma",
                                              "achieved": flops / (bf_ms * 1e-3) / 1e12, "peak": MFMA_FP32_PEAK_TFLOPS,
                                              "unit": "TFLOP/s", "frac": flops / (bf_ms * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS,
                                              "note": "whole call (distance and selection kernels)"}}
    pqt.pqt_index_free(index)
    del index, Y, out_ids, out_d
    torch.cuda.empty_cache()
    if tmp is not None:
        import shutil
        shutil.rmtree(tmp, ignore_errors=True)
    return result


def main():
    args = parse_args()
    import paper_1702_05911_amd.binding as pqt
    # Measured ceilings first: about a second of streaming reads and matrix-core work, which also brings the
    # clocks up from idle before anything is timed (twenty steps straight after an idle set-up read 8-10 % low).
    peaks = pqt.pqt_measure_peaks(0)
    result = run_workload(args, args.workload, True, peaks)
    also = args.also if args.also is not None else ("large,billion" if args.workload == "sift" and not args.batch else "")
    extra = {}
    for name in [v for v in also.split(",") if v]:
        print(f"[bench] sub-record: {name}", file=sys.stderr, flush=True)
        sub = run_workload(args, name, False, peaks)
        extra[name] = {key: sub[key] for key in ("value", "unit", "ms_per_step", "steps", "warmup", "dtype", "config", "recall",
                                                 "stage_ms", "stages", "roofline", "tuples_needed", "setup_s")}
    if extra:
        # the index of the headline workload (8 MB of codes) lives in the caches; these do not
        result["hbm_resident"] = extra
    print(json.dumps(result))


if __name__ == "__main__":
    main()
