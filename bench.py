"""Benchmark of the query path on the Glove-shaped configuration (one GPU).

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path -- table build, ADC scan with top-100
selection, merge, exact fp32 re-ranking to top-10 -- over one batch of 10,000
synthetic queries against n = 1,183,514 points (d = 100, 50 subspaces x 16
codewords, 25 B/point), with every input already resident in HBM. The index is
built by the library itself (avq_train on the first 262,144 points, avq_encode
under the anisotropic loss, T = 0.2) before the timed region.

Prints one JSON line. `value` is queries/s over the timed steps at batch
10,000 with fp32 tables; `roofline` describes the kernel that dominates those
steps (the fp32 scan). The same line carries the 8-bit-table rate (matrix-core
scan), the batch-1 numbers with their own roofline object (the HBM-bound
regime, warm and cold cache), Recall@10 against exact search, and the CPU
oracle timed on this host on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
# fp32 vector peak is 157.3 TFLOP/s counting an FMA as two flops: 78.6e12 single
# operations per second (256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz). The scan's arithmetic
# is plain adds of table entries.
VALU_PEAK_TOPS = 157.3 / 2
# LDS: 256 CUs x 256 B/clk x 2.4 GHz (a conflict-free 16-byte gather reaches 224 B/clk/CU)
LDS_PEAK_GBS = 256 * 256 * 2.4
MFMA_I8_PEAK_TOPS = 5000.0       # dense int8, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def unpack4(packed, M):
    out = np.empty((packed.shape[0], M), np.uint8)
    out[:, 0::2] = packed[:, : (M + 1) // 2] & 15
    out[:, 1::2] = (packed[:, : M // 2] >> 4) & 15
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="glove", choices=["tiny", "glove", "glove100", "glove_ivf", "large4", "large8"],
                    help="workload (default: the Glove-shaped one the headline metric is quoted on)")
    ap.add_argument("--batch", type=int, default=0, help="queries per step (default: the configuration's)")
    ap.add_argument("--n", type=int, default=0, help="override the number of points (debugging)")
    ap.add_argument("--b1-steps", type=int, default=2000)
    ap.add_argument("--recall-queries", type=int, default=1000)
    ap.add_argument("--oracle-queries", type=int, default=0,
                    help="queries of the CPU baseline sample (default: about 15 s of oracle work on 16 threads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of the datapoint array (known size) so that "
                         "hardware byte counters can be scaled against them")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); sharding over several GPUs "
                 "is a design note, not an implementation")

    import torch

    import paper_1908_10396_amd as avq
    import synth_inputs as si

    cfg = dict(si.CONFIGS[args.config])
    if args.n:
        cfg["n"] = args.n
    n, d, M, bits, k, R = cfg["n"], cfg["d"], cfg["M"], cfg["bits"], cfg["k"], cfg["reorder_k"]
    B = args.batch or cfg["nq"]
    nb = (M * bits + 7) // 8
    n_leaves = cfg.get("n_leaves", 0)
    Lp = cfg.get("leaves_to_search", 0)
    glove_default = args.config == "glove" and not args.n

    t0 = time.time()
    q = si.make_queries(cfg, B)
    qd = torch.from_numpy(q).cuda()
    if n * d * 4 <= 8 << 30:
        x = si.make_data(cfg)
        xd = torch.from_numpy(x).cuda()
    else:
        # too large to hold twice on the host: generate chunk by chunk straight into HBM
        x = None
        xd = torch.empty((n, d), dtype=torch.float32, device="cuda")
        centers = si.mixture_centers(cfg["n_comp"], d, cfg["seed"])
        for c, lo, hi in si._chunks(n):
            xd[lo:hi] = torch.from_numpy(si.mixture_chunk(c, hi - lo, d, centers, cfg["sigma"], cfg["seed"],
                                                          si.STREAM_DATA, cfg.get("lognormal_sigma"))).cuda()
            if c % 16 == 0:
                log("[bench] generated %d of %d rows" % (hi, n))
    log("[bench] generated %d x %d points and %d queries in %.1fs" % (n, d, B, time.time() - t0))
    idx = avq.Index(d, M, bits, T=cfg["T"], kmeans_iters=20, encode_passes=10, seed=cfg["seed"],
                    n_leaves=n_leaves, leaf_kmeans_iters=10)
    t0 = time.time()
    idx.train(xd[: min(n, si.CHUNK)])
    t_train = time.time() - t0
    t0 = time.time()
    idx.encode(xd)
    torch.cuda.synchronize()
    t_encode = time.time() - t0
    log("[bench] train %.2fs, encode %.2fs" % (t_train, t_encode))

    ids = torch.empty((B, k), dtype=torch.int32, device="cuda")
    sc = torch.empty((B, k), dtype=torch.float32, device="cuda")

    if args.copy_calibration:
        y = torch.empty_like(xd)
        for _ in range(3):
            y.copy_(xd)
        torch.cuda.synchronize()
        log("[bench] copy calibration: 3 device copies of %d bytes (read) + %d bytes (write) each"
            % (xd.numel() * 4, xd.numel() * 4))
        del y

    def timed_batch(lut_mode, steps):
        """K steps at batch B, bracketed by synchronize; per-stage kernel time from HIP events."""
        for _ in range(args.warmup):
            idx.search(qd, k, R, lut_mode, Lp, out=(ids, sc))
        torch.cuda.synchronize()
        idx.profile_enable(True)
        idx.profile_read(reset=True)
        t0 = time.perf_counter()
        for _ in range(steps):
            idx.search(qd, k, R, lut_mode, Lp, out=(ids, sc))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = idx.profile_read(reset=True)
        idx.profile_enable(False)
        stage_ms = {s: (v[0] / v[1] if v[1] else 0.0) for s, v in prof.items()}
        return dt, stage_ms

    def timed_single(lut_mode, steps):
        """Single-query calls: end-to-end time without instrumentation, then per-stage kernel
        time from HIP events in a second, instrumented loop (the event records are extra
        packets on the stream and would otherwise be part of the latency)."""
        ids1 = torch.empty((1, k), dtype=torch.int32, device="cuda")
        sc1 = torch.empty((1, k), dtype=torch.float32, device="cuda")
        q1 = [qd[i:i + 1] for i in range(min(B, 64))]
        for i in range(50):
            idx.search(q1[i % len(q1)], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            idx.search(q1[i % len(q1)], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        idx.profile_enable(True)
        idx.profile_read(reset=True)
        for i in range(max(50, steps // 4)):
            idx.search(q1[i % len(q1)], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        prof = idx.profile_read(reset=True)
        idx.profile_enable(False)
        stage_us = {s: (v[0] / v[1] * 1e3 if v[1] else 0.0) for s, v in prof.items()}
        return dt, stage_us

    def cold_single_scan_us(lut_mode, reps=20):
        """Scan-stage time of single-query calls when the codes are not in the Infinity Cache:
        a 1 GiB buffer is read through before every call (outside the stage's event pair;
        reading leaves no dirty lines whose write-back would compete with the scan)."""
        ids1 = torch.empty((1, k), dtype=torch.int32, device="cuda")
        sc1 = torch.empty((1, k), dtype=torch.float32, device="cuda")
        evict = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        sink = torch.zeros((), dtype=torch.float32, device="cuda")
        idx.profile_enable(True)
        idx.profile_read(reset=True)
        for i in range(reps):
            sink += evict.sum()
            idx.search(qd[i % min(B, 64):i % min(B, 64) + 1], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        prof = idx.profile_read(reset=True)
        idx.profile_enable(False)
        del evict
        return prof["scan"][0] / prof["scan"][1] * 1e3 if prof["scan"][1] else 0.0

    # ---- timed region 1: batches of B queries, fp32 tables (the headline) ------------------
    dt, stage_ms = timed_batch(avq.LUT_F32, args.steps)
    ms_per_step = dt / args.steps * 1e3
    qps = B * args.steps / dt
    scan_ms = stage_ms["scan"]
    scanned = float(n) * (Lp / n_leaves if n_leaves else 1.0)   # points a query scans (expected, with leaves)
    # Arithmetic of the fp32 scan per (query, point): 4-bit codes on a flat index use the
    # 16-entry tables (two entries of a byte are added, then accumulated: 2*NB adds, 8*NB bytes
    # of LDS); byte tables take NB adds and 4*NB bytes.
    nib_tile = bits == 4 and not n_leaves and B >= 8
    # batches with fp32 tables on a flat index of 4-bit codes take their candidates from the
    # matrix-core scan over the 8-bit tables and re-score them in fp32 (exact, see include/avq.h)
    prefiltered = bits == 4 and not n_leaves and B >= 16 and nb in (8, 13, 25, 32) and M <= 64
    n_pad = float((n + 255) // 256 * 256)
    b_pad = float((B + 31) // 32 * 32)
    # the sparse matrix instruction multiplies 32 points x 32 queries over 32 stored positions (64 logical ones: two
    # code bytes, four subspaces); ceil(NB / 2) instructions per (32, 32). Counted: the multiply-adds it executes,
    # which is what the dense int8 peak prices; the dense contraction it stands for has twice as many.
    steps_per_pair = (nb + 1) // 2
    mfma_ops = 2.0 * n_pad * b_pad * steps_per_pair * 32

    def direct_roofline(ms):
        adds = (2.0 if nib_tile else 1.0) * nb * scanned * B
        lds_bytes = (8.0 if nib_tile else 4.0) * nb * scanned * B
        if n_leaves:
            kern = "adc_scan_kernel<1,false,%d,1>" % (nb if nb in (8, 13, 25, 32) else 0)
        else:
            kern = "adc_scan_kernel<%d,false,%d,0>" % (8 if nib_tile else 4, nb if nb in (8, 13, 25, 32) else 0)
        r = {"bound": "alu", "achieved": adds / (ms * 1e-3) / 1e12, "peak": VALU_PEAK_TOPS,
             "unit": "TFLOP/s", "traffic": None, "kernel": kern, "avg_launch_ms": ms,
             "note": "fp32 adds of table entries (no multiplies); the other binding unit is the LDS gather",
             "lds_gather": {"achieved_GBs": lds_bytes / (ms * 1e-3) / 1e9, "peak_GBs": LDS_PEAK_GBS,
                            "frac": lds_bytes / (ms * 1e-3) / 1e9 / LDS_PEAK_GBS}}
        r["frac"] = r["achieved"] / r["peak"]
        return r

    fp32_direct = None
    # the matrix-core scan takes two launches per step unless the chunks are very short (the library's rule:
    # at least 4 blocks): about one block in 32 of every chunk first (2 to 16 per chunk), then everything
    n_blocks = (n + 255) // 256
    n_tiles32 = (B + 31) // 32
    # waves of a launch = tiles x chunks, in whole rounds of 2048 resident waves (the library's rule: the fewest
    # rounds, up to 4, that leave under 3 % of the last one empty, else the fullest)
    target, best = 2048, 0.0
    for rounds in range(1, 5):
        c = rounds * 2048 // n_tiles32
        if c < 1:
            continue
        fill = c * n_tiles32 / (rounds * 2048.0)
        if fill > best + 1e-9:
            best, target = fill, rounds * 2048
        if fill >= 0.97:
            break
    chunks = max(1, min(target // n_tiles32, 256, n_blocks // 4))
    bpc = -(-n_blocks // chunks)
    sampled = bpc >= 4
    per_chunk = max(2, min(16, (bpc + 31) // 32))
    visited = -(-bpc // max(1, bpc // per_chunk))
    grouped = (bool(n_leaves) and bits == 4 and B >= 64 and B * Lp >= 131072 and nb in (8, 13, 25, 32) and M <= 64
               and 16 <= Lp <= 512)   # the library's rule
    if grouped:
        # partitioned index: the (query, leaf) pairs regrouped by leaf, leaves scanned on the matrix cores;
        # the scan stage also holds the bounds pass over every query's best leaves and the regrouping
        unverified = idx.debug_unverified_queries(reasons=True)
        ops = 2.0 * scanned * B * steps_per_pair * 32
        batch_roof = {"bound": "mfma", "achieved": ops / (scan_ms * 1e-3) / 1e12, "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s",
                      "traffic": None, "kernel": "adc_mfma_scan_kernel<%d,false,true,true>" % nb, "avg_launch_ms": scan_ms,
                      "sample_stage_ms": stage_ms.get("sample", 0.0),
                      "note": "int8 multiply-adds executed by the scan over leaves (sparse instruction, 32 queries per leaf "
                              "and work item); before it, timed apart (sample_stage_ms): the bounds pass (leaf_bound_kernel "
                              "over each query's best leaves) and the regrouping of the (query, leaf) pairs",
                      "queries_scanned_again": unverified[0]}
        batch_roof["frac"] = batch_roof["achieved"] / batch_roof["peak"]
    elif prefiltered:
        unverified = idx.debug_unverified_queries(reasons=True)
        # HBM-side bytes of the launch over all blocks from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a
        # plain copy of known size (profiles/scan_glove_pmc_traffic.md); only valid for the default workload
        batch_roof = {"bound": "mfma", "achieved": mfma_ops / (scan_ms * 1e-3) / 1e12, "peak": MFMA_I8_PEAK_TOPS,
                      "unit": "TOP/s", "traffic": (0.38e9 + 0.05e9) if (glove_default and B == 10000) else None,
                      "kernel": "adc_mfma_scan_kernel<%d,false,false,%s>" % (nb, "true" if sampled else "false"),
                      "launches_per_step": 1, "avg_launch_ms": scan_ms,
                      "sample_stage_ms": stage_ms.get("sample", 0.0),
                      "note": "int8 multiply-adds executed by the launch over all blocks of the candidate scan over the "
                              "8-bit tables (v_smfmac_i32_32x32x64_i8: the one-hot operand is 2:4 sparse, so an instruction "
                              "covers 64 positions with 32 multiply-adds per output; 8 executed per useful table add). "
                              "Before it, timed apart (sample_stage_ms): margins, a launch of the store variant over a "
                              "sample of the blocks (%.1f %% of these operations) and the bounds guessed from it; the fp32 "
                              "scores are formed for the kept points only" % (100.0 * visited / bpc if sampled else 0.0),
                      "queries_scanned_again_with_fp32_tables": unverified[0],
                      "of_which_too_many_kept_or_bound_too_high_or_other": unverified[1:]}
        batch_roof["frac"] = batch_roof["achieved"] / batch_roof["peak"]
        # for orientation: the dense one-hot contraction the sparse instruction stands for (twice the executed
        # operations), and the table adds the method itself asks for (M per query and point)
        batch_roof["dense_equivalent_frac"] = 2.0 * batch_roof["frac"] * (nb / (2.0 * steps_per_pair))
        batch_roof["table_adds_per_s"] = float(M) * scanned * B / (scan_ms * 1e-3)
        # the same step with every point scored in fp32 (the kernel the candidate scan replaces)
        idx.set_tuning("scan_prefilter", 1)
        dt_d, stage_d = timed_batch(avq.LUT_F32, max(2, args.steps // 5))
        idx.set_tuning("scan_prefilter", 0)
        fp32_direct = {"queries_per_s": B * max(2, args.steps // 5) / dt_d, "stage_ms": stage_d,
                       "roofline": direct_roofline(stage_d["scan"])}
        log("[bench] fp32 batch %d, every point scored in fp32: %.0f q/s, stages(ms) %s"
            % (B, fp32_direct["queries_per_s"], stage_d))
    else:
        batch_roof = direct_roofline(scan_ms)
    log("[bench] fp32 batch %d: %.2f ms/step, %.0f q/s, stages(ms) %s" % (B, ms_per_step, qps, stage_ms))

    # ---- same with 8-bit tables ---------------------------------------------------------------
    dt8, stage8_ms = timed_batch(avq.LUT_U8, max(2, args.steps // 2))
    qps8 = B * max(2, args.steps // 2) / dt8
    log("[bench] u8   batch %d: %.0f q/s, stages(ms) %s" % (B, qps8, stage8_ms))
    u8_roof = None
    if bits == 4 and not n_leaves and B >= 16 and nb in (8, 13, 25, 32):
        # one-hot contraction on the sparse int8 matrix instruction: 32 points x 32 queries, four subspaces (64
        # positions, 32 of them stored) per instruction, ceil(NB / 2) instructions per (32 points, 32 queries)
        u8_roof = {"bound": "mfma", "achieved": mfma_ops / (stage8_ms["scan"] * 1e-3) / 1e12, "peak": MFMA_I8_PEAK_TOPS,
                   "unit": "TOP/s", "kernel": "adc_mfma_scan_kernel<%d,false,false,%s>" % (nb, "true" if sampled else "false"),
                   "launches_per_step": 1, "avg_launch_ms": stage8_ms["scan"], "sample_stage_ms": stage8_ms.get("sample", 0.0),
                   "traffic": None,
                   "note": "int8 multiply-adds executed (sparse instruction); 8 of them per useful table add (one-hot operand)"}
        u8_roof["frac"] = u8_roof["achieved"] / u8_roof["peak"]

    # ---- timed region 2: single queries (the HBM-bound regime) ---------------------------------
    dt1, stage1_us = timed_single(avq.LUT_F32, args.b1_steps)
    scan1_ms = stage1_us["scan"] / 1e3
    code_bytes = float(nb) * scanned             # algorithmic bytes of one single-query scan
    # HBM-side bytes per launch of this kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by
    # a plain copy of known size (profiles/scan_glove_pmc_traffic.md); only valid for the default n
    traffic = 29.72e6 + 0.037e6 if glove_default else None
    b1_roof = {"bound": "hbm", "achieved": code_bytes / (scan1_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
               "unit": "GB/s", "traffic": traffic, "kernel": ("adc_scan_kernel<1,false,%d,1>" % nb) if n_leaves else ("block_max_nibble_kernel<false,%d>" % nb if bits == 4 else "block_max_kernel<false,%d>" % nb),
               "avg_launch_ms": scan1_ms,
               "note": "repeated scans of a code array below 256 MB are served from the Infinity Cache (see cold)"}
    b1_roof["frac"] = b1_roof["achieved"] / b1_roof["peak"]
    log("[bench] fp32 batch 1: %.1f us/query end to end, stages(us) %s" % (dt1 / args.b1_steps * 1e6, stage1_us))
    # what a HIP event pair reports around nothing: part of every per-stage figure above
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    torch.cuda.synchronize()
    for a_, b_ in evs:
        a_.record()
        b_.record()
    torch.cuda.synchronize()
    ev_over_us = float(np.median([a_.elapsed_time(b_) for a_, b_ in evs])) * 1e3
    b1_roof["event_pair_overhead_us"] = ev_over_us
    # the floor for this array on this machine: the scan's loads in the scan's launch shape, no lookups
    words = idx.debug_stream_codes()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    torch.cuda.synchronize()
    for a_, b_ in evs:
        a_.record()
        idx.debug_stream_codes(out=words)
        b_.record()
    torch.cuda.synchronize()
    floor_us = float(np.median([a_.elapsed_time(b_) for a_, b_ in evs])) * 1e3
    b1_roof["stream_floor"] = {"kernel": "stream_codes_kernel<%d>" % (nb if nb in (8, 13, 25, 32) else 0),
                               "avg_launch_ms": floor_us / 1e3,
                               "achieved": float(nb) * float(n) / (floor_us * 1e-6) / 1e9,
                               "scan_over_floor": stage1_us["scan"] / floor_us if floor_us else None,
                               "note": "the same loads and launch shape without table lookups, same event timing"}
    log("[bench] code stream alone (no lookups): %.1f us" % floor_us)
    cold_us = cold_single_scan_us(avq.LUT_F32)
    b1_roof["cold"] = {"avg_launch_ms": cold_us / 1e3, "achieved": code_bytes / (cold_us * 1e-6) / 1e9 if cold_us else None,
                       "note": "1 GiB read through the Infinity Cache before every call"}
    log("[bench] fp32 batch 1, cold cache: scan %.1f us" % cold_us)
    dt1u, stage1u_us = timed_single(avq.LUT_U8, max(100, args.b1_steps // 2))
    log("[bench] u8   batch 1: %.1f us/query end to end, stages(us) %s"
        % (dt1u / max(100, args.b1_steps // 2) * 1e6, stage1u_us))

    # ---- recall against exact search (untimed) ---------------------------------------------------
    nr = min(args.recall_queries, B)
    gt_ids, _ = idx.brute_force(qd[:nr], k)
    recall = {}
    for name, mode in (("f32", avq.LUT_F32), ("u8", avq.LUT_U8)):
        got_ids, _ = idx.search(qd[:nr], k, R, mode, Lp)
        torch.cuda.synchronize()
        g, t = got_ids.cpu().numpy(), gt_ids.cpu().numpy()
        recall[name] = float(np.mean([len(set(g[i]) & set(t[i])) / k for i in range(nr)]))
    log("[bench] recall@%d over %d queries: %s" % (k, nr, recall))

    # ---- CPU oracle on this host, bounded sample of the same workload ------------------------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline and x is not None:
        import oracle
        # the oracle does about 1e2 queries/s at the Glove shape on 16 threads; its time goes with points x subspaces
        auto = int(1536 * (1183514.0 * 50.0) / max(1.0, scanned * M))
        no = min(args.oracle_queries if args.oracle_queries > 0 else max(16, auto), B)
        cb = idx.get_codebooks()
        codes = unpack4(idx.get_codes(), M) if bits == 4 else idx.get_codes()
        okw = {}
        if n_leaves:
            okw = dict(centers=idx.get_leaf_centers(), assign=idx.get_leaf_assign(), leaves_to_search=Lp)
        t0 = time.perf_counter()
        oi, os_ = oracle.search(x, cb, codes, bits, q[:no], k, R, avq.LUT_F32, **okw)
        dto = time.perf_counter() - t0
        gi, gs = idx.search(qd[:no], k, R, avq.LUT_F32, Lp)
        torch.cuda.synchronize()
        parity = bool(np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gs.cpu().numpy(), os_))
        o8, s8 = oracle.search(x, cb, codes, bits, q[:16], k, R, avq.LUT_U8, **okw)
        g8, gs8 = idx.search(qd[:16], k, R, avq.LUT_U8, Lp)
        torch.cuda.synchronize()
        parity = parity and bool(np.array_equal(g8.cpu().numpy(), o8) and np.array_equal(gs8.cpu().numpy(), s8))
        cpu = {"value": no / dto, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d of the %d queries against all %d points (table build, ADC, full sort to "
                         "top-%d, exact re-rank), OpenMP over queries" % (no, B, n, R),
               "host_cpus": os.cpu_count(), "seconds": dto}
        log("[bench] oracle: %d queries in %.1fs on %d threads; GPU results identical: %s"
            % (no, dto, cpu["cores"], parity))

    out = {
        "metric": "queries/sec at Recall@10 vs brute force; ADC codes/sec and % HBM BW",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: n=%d d=%d PQ %dx%d (%d-bit, %d B/point) T=0.2%s, batch %d, "
                               "ADC top-%d re-ranked to top-%d"
                               % (args.config, n, d, M, 1 << bits, bits, nb,
                                  (", %d leaves, %d searched" % (n_leaves, Lp)) if n_leaves else "", B, R, k),
                   "lut": "f32", "train_s": t_train, "encode_s": t_encode,
                   "scan": ("int8 matrix-core candidate scan + fp32 re-scoring of the kept points (results equal "
                            "a full fp32 scan)") if prefiltered else "fp32 table sums of every point"},
        "recall_at_10": recall["f32"], "recall_at_10_u8": recall["u8"], "recall_queries": nr,
        "adc_points_per_s": scanned * B / (scan_ms * 1e-3),
        "adc_codes_per_s": scanned * B * M / (scan_ms * 1e-3),
        "stage_ms": stage_ms,
        "fp32_every_point": fp32_direct,
        "u8": {"queries_per_s": qps8, "stage_ms": stage8_ms,
               "adc_codes_per_s": scanned * B * M / (stage8_ms["scan"] * 1e-3), "roofline": u8_roof},
        "roofline": batch_roof,
        "roofline_batch1": b1_roof,
        "batch1": {"queries_per_s": args.b1_steps / dt1, "us_per_query": dt1 / args.b1_steps * 1e6,
                   "steps": args.b1_steps, "stage_us": stage1_us,
                   "adc_points_per_s": scanned / (scan1_ms * 1e-3),
                   "adc_codes_per_s": scanned * M / (scan1_ms * 1e-3),
                   "hbm_frac": b1_roof["frac"],
                   "u8_us_per_query": dt1u / max(100, args.b1_steps // 2) * 1e6, "u8_stage_us": stage1u_us},
        "cpu_baseline": cpu, "matches_oracle": parity,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
