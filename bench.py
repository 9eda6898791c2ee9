"""Benchmark of the query path (one GPU).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config glove|glove_ivf|large4|large8|...]

A step is one pass of the whole hot path -- table build, ADC scan with top-R
selection, exact fp32 re-ranking to top-k -- over one batch of synthetic
queries, with every input already resident in HBM. The default workload is the
Glove-shaped one the headline metric is quoted on: 10,000 queries against
n = 1,183,514 points (d = 100, 50 subspaces x 16 codewords, 25 B/point), ADC
top-100 re-ranked to top-10. The index is built by the library itself
(avq_train on the first 262,144 points, avq_encode under the anisotropic loss,
T = 0.2) before the timed region.

Prints one JSON line. `value` is queries/s over the timed steps at the
configuration's batch size with fp32 tables. `roofline` describes the kernel
that dominates those steps; its `frac` prices the method's own work (M table
lookups + M additions per query and point) against the peak of the unit the
kernel runs on, and the operations the kernel executes to get there are
reported beside it (`mfma_pipe_util`). `roofline_batch1` is the HBM-bound
regime: the single-query scan, timed as back-to-back launches inside one event
pair, next to the code stream alone and the table lookups alone. The line
also carries the 8-bit-table rate, Recall@k against exact search, and the CPU
oracle timed on this host (all threads and one thread) on a bounded sample of
the same workload.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
# fp32 vector peak is 157.3 TFLOP/s counting an FMA as two flops: 78.6e12 single
# operations per second (256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz). A scan over fp32
# tables only adds table entries.
VALU_PEAK_TOPS = 157.3 / 2
LDS_PEAK_GBS = 256 * 256 * 2.4   # 256 CUs x 256 B/clk x 2.4 GHz
MFMA_I8_PEAK_TOPS = 5000.0       # dense int8, published
SPECIAL_NB = (8, 13, 25, 32)     # code sizes with specialised kernels


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def unpack4(packed, M):
    out = np.empty((packed.shape[0], M), np.uint8)
    out[:, 0::2] = packed[:, : (M + 1) // 2] & 15
    out[:, 1::2] = (packed[:, : M // 2] >> 4) & 15
    return out


def traffic_from_profiles(kernel, workload):
    """HBM-side bytes per launch of `kernel` on `workload`, as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE in an earlier run whose summary under profiles/ carries a line
        traffic_bytes_per_launch: kernel=<name> workload=<name> fetch=<bytes> write=<bytes>
    (scaled by a plain copy of known size, as that file explains). None if no such record exists."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None, None
    for fn in sorted(os.listdir(pdir)):
        try:
            with open(os.path.join(pdir, fn)) as f:
                for line in f:
                    m = re.match(r"\s*traffic_bytes_per_launch: kernel=(\S+) workload=(\S+) fetch=([0-9.e+]+) write=([0-9.e+]+)", line)
                    if m and m.group(1) == kernel and m.group(2) == workload:
                        return float(m.group(3)) + float(m.group(4)), "profiles/" + fn
        except OSError:
            pass
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="glove", choices=["tiny", "glove", "glove100", "glove8", "glove_ivf", "large4", "large8"],
                    help="workload (default: the Glove-shaped one the headline metric is quoted on)")
    ap.add_argument("--batch", type=int, default=0, help="queries per step (default: the configuration's)")
    ap.add_argument("--n", type=int, default=0, help="override the number of points (debugging)")
    ap.add_argument("--b1-steps", type=int, default=2000)
    ap.add_argument("--recall-queries", type=int, default=1000)
    ap.add_argument("--oracle-queries", type=int, default=0,
                    help="queries of the CPU baseline sample (default: about 15 s of oracle work on all threads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extra-batches", default="", help="comma-separated batch sizes to time as well (e.g. 64)")
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
    workload = args.config if not args.n else "%s_n%d" % (args.config, n)

    t0 = time.time()
    q = si.make_queries(cfg, max(B, 64))
    qd_all = torch.from_numpy(q).cuda()
    qd = qd_all[:B].contiguous()
    if cfg["kind"] == "gaussian":
        x = si.make_data(cfg)
        xd = torch.from_numpy(x).cuda()
    else:
        # chunk by chunk straight into HBM; a host copy is kept for the CPU baseline while it fits comfortably
        x = np.empty((n, d), np.float32) if n * d * 4 <= 64 << 30 and not args.no_cpu_baseline else None
        xd = torch.empty((n, d), dtype=torch.float32, device="cuda")
        centers = si.mixture_centers(cfg["n_comp"], d, cfg["seed"])
        for c, lo, hi in si._chunks(n):
            rows = si.mixture_chunk(c, hi - lo, d, centers, cfg["sigma"], cfg["seed"], si.STREAM_DATA,
                                    cfg.get("lognormal_sigma"))
            if x is not None:
                x[lo:hi] = rows
            xd[lo:hi] = torch.from_numpy(rows).cuda()
            if c % 16 == 15:
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

    if args.copy_calibration:
        y = torch.empty_like(xd)
        for _ in range(3):
            y.copy_(xd)
        torch.cuda.synchronize()
        log("[bench] copy calibration: 3 device copies of %d bytes (read) + %d bytes (write) each"
            % (xd.numel() * 4, xd.numel() * 4))
        del y

    def timed_batch(lut_mode, steps, queries=None):
        """K steps, bracketed by synchronize; per-stage kernel time per step from HIP events on the stream."""
        qq = qd if queries is None else queries
        ids = torch.empty((qq.shape[0], k), dtype=torch.int32, device="cuda")
        sc = torch.empty((qq.shape[0], k), dtype=torch.float32, device="cuda")
        for _ in range(args.warmup):
            idx.search(qq, k, R, lut_mode, Lp, out=(ids, sc))
        torch.cuda.synchronize()
        idx.profile_enable(True)
        idx.profile_read(reset=True)
        t0 = time.perf_counter()
        for _ in range(steps):
            idx.search(qq, k, R, lut_mode, Lp, out=(ids, sc))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = idx.profile_read(reset=True)
        idx.profile_enable(False)
        return dt, {s: v[0] / steps for s, v in prof.items()}

    def timed_single(lut_mode, steps):
        """Single-query calls: end-to-end time without instrumentation, then per-stage kernel time per call from
        HIP events in a second, instrumented loop (the event records are extra packets on the stream; every
        stage figure includes the few microseconds an event pair costs)."""
        ids1 = torch.empty((1, k), dtype=torch.int32, device="cuda")
        sc1 = torch.empty((1, k), dtype=torch.float32, device="cuda")
        q1 = [qd_all[i:i + 1] for i in range(64)]
        for i in range(50):
            idx.search(q1[i % 64], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            idx.search(q1[i % 64], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        calls = max(50, steps // 4)
        idx.profile_enable(True)
        idx.profile_read(reset=True)
        for i in range(calls):
            idx.search(q1[i % 64], k, R, lut_mode, Lp, out=(ids1, sc1))
        torch.cuda.synchronize()
        prof = idx.profile_read(reset=True)
        idx.profile_enable(False)
        return dt, {s: v[0] / calls * 1e3 for s, v in prof.items()}

    def launches_us(part, lut_mode, reps=200, evict=None):
        """Mean duration of one launch of a part of the single-query scan: `reps` launches back to back on the
        stream inside one HIP event pair (avq_debug_scan_parts), the pair's own cost spread over all of them.
        evict: a buffer read through before every launch (then one launch per pair, its cost included)."""
        s = torch.cuda.current_stream()
        idx.debug_scan_parts(qd_all[:1], lut_mode, part, 20)
        torch.cuda.synchronize()
        if evict is None:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(s)
            idx.debug_scan_parts(qd_all[:1], lut_mode, part, reps)
            b.record(s)
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e3 / reps
        sink = torch.zeros((), dtype=torch.float32, device="cuda")
        ts = []
        for _ in range(20):
            sink += evict.sum()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(s)
            idx.debug_scan_parts(qd_all[:1], lut_mode, part, 1)
            b.record(s)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3)
        return float(np.median(ts))

    # ---- timed region 1: batches of B queries, fp32 tables (the headline) ------------------
    dt, stage_ms = timed_batch(avq.LUT_F32, args.steps)
    ms_per_step = dt / args.steps * 1e3
    qps = B * args.steps / dt
    scan_ms = stage_ms["scan"]
    scanned = float(n) * (Lp / n_leaves if n_leaves else 1.0)   # points a query scans (expected, with leaves)
    # The method's work (Section 4.1, Section 2.2.2's O(mn) term): one table lookup and one addition per
    # subspace, per scanned point, per query.
    method_ops = 2.0 * M * scanned * B
    nib_tile = bits == 4 and not n_leaves and B >= 8
    # batches with fp32 tables on a flat index of 4-bit codes take their candidates from the matrix-core scan
    # over the 8-bit tables and re-score them in fp32 (exact, see include/avq.h)
    small = not n_leaves and B <= (35 if bits == 4 else 8)
    prefiltered = bits == 4 and not n_leaves and not small and nb in SPECIAL_NB and M <= 64
    grouped = (bool(n_leaves) and bits == 4 and B >= 64 and B * Lp >= 131072 and nb in SPECIAL_NB and M <= 64
               and 16 <= Lp <= 512)   # the library's rule
    n_pad = float((n + 255) // 256 * 256)
    b_pad = float((B + 31) // 32 * 32)
    # the sparse matrix instruction multiplies 32 points x 32 queries over 32 stored positions (64 logical ones: two
    # code bytes, four subspaces); ceil(NB / 2) instructions per (32, 32): the multiply-adds the kernel executes
    steps_per_pair = (nb + 1) // 2
    mfma_executed = 2.0 * (scanned if n_leaves else n_pad) * b_pad * steps_per_pair * 32

    tiled = bits == 8 and not n_leaves and not small and nb in SPECIAL_NB   # batches of 8-bit codes: block bounds, 16 queries per tile

    def lds_roofline(ms, batch, every_point=False):
        """A scan that forms its sums from tables in LDS: bound by the plain ALU (adds) and the LDS gather."""
        adds = (2.0 if nib_tile else 1.0) * nb * scanned * batch
        lds_bytes = (8.0 if nib_tile else 4.0) * nb * scanned * batch
        if tiled and not every_point:
            # byte tables of seven bits, sixteen queries per 16-byte entry: one byte of LDS per query, point and code byte;
            # entries of two code bytes are added as packed bytes, then spread into 16-bit sums
            # byte-sized integer additions, four to a 32-bit lane operation: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz x 4
            r = {"bound": "alu", "achieved": 2.0 * M * scanned * batch / (ms * 1e-3) / 1e12, "peak": VALU_PEAK_TOPS * 4,
                 "unit": "TOP/s", "traffic": None, "kernel": "block_bound_tile_kernel<%d,2>" % nb, "avg_launch_ms": ms,
                 "note": "the method's M lookups + M additions per query and point against the peak of byte-sized integer adds "
                         "(four to a 32-bit lane operation: 4 x 78.6 TOP/s); the kernel reads one 16-byte LDS entry per point and "
                         "code byte for sixteen queries, adds the entries of two code bytes as packed bytes and forms block maxima "
                         "of these 7-bit table sums (bounds); exact scores are formed afterwards for the blocks that can reach the "
                         "R-th best",
                 "lds_gather": {"achieved_GBs": nb * scanned * batch / (ms * 1e-3) / 1e9, "peak_GBs": LDS_PEAK_GBS,
                                "frac": nb * scanned * batch / (ms * 1e-3) / 1e9 / LDS_PEAK_GBS},
                 "code_stream_GBs": nb * scanned * ((batch + 15) // 16) / (ms * 1e-3) / 1e9}
            r["frac"] = r["achieved"] / r["peak"]
            r["traffic"], r["traffic_source"] = traffic_from_profiles(r["kernel"], "%s_b%d" % (workload, batch))
            return r
        if n_leaves:
            kern = "adc_scan_kernel<1,false,%d,1>" % (nb if nb in SPECIAL_NB else 0)
        else:
            kern = "adc_scan_kernel<%d,false,%d,0>" % (8 if nib_tile else 4, nb if nb in SPECIAL_NB else 0)
        r = {"bound": "alu", "achieved": 2.0 * M * scanned * batch / (ms * 1e-3) / 1e12, "peak": VALU_PEAK_TOPS,
             "unit": "TOP/s", "traffic": None, "kernel": kern, "avg_launch_ms": ms,
             "note": "the method's M lookups + M additions per query and point against the fp32 add peak; the kernel "
                     "executes %.0f fp32 adds per point (entries of a code byte are added first) and gathers %.0f B of "
                     "LDS per point and query" % (adds / (scanned * batch), lds_bytes / (scanned * batch)),
             "lds_gather": {"achieved_GBs": lds_bytes / (ms * 1e-3) / 1e9, "peak_GBs": LDS_PEAK_GBS,
                            "frac": lds_bytes / (ms * 1e-3) / 1e9 / LDS_PEAK_GBS}}
        r["frac"] = r["achieved"] / r["peak"]
        r["traffic"], r["traffic_source"] = traffic_from_profiles(kern, "%s_b%d" % (workload, batch))
        return r

    def mfma_roofline(ms, kernel, extra):
        r = {"bound": "mfma", "achieved": method_ops / (ms * 1e-3) / 1e12, "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s",
             "kernel": kernel, "avg_launch_ms": ms,
             "mfma_pipe_util": mfma_executed / (ms * 1e-3) / 1e12 / MFMA_I8_PEAK_TOPS,
             "note": "achieved = the method's work, M table lookups + M additions per query and scanned point, per second, "
                     "against the dense int8 matrix peak. The kernel forms the sums as a one-hot contraction on "
                     "v_smfmac_i32_32x32x64_i8 and executes 8 multiply-adds per useful table add (mfma_pipe_util = "
                     "executed operations / peak). For scale: the plain-ALU ceiling of the same sums is %.1f TOP/s "
                     "(fp32 add peak), so the rate here is %.1fx that ceiling"
                     % (VALU_PEAK_TOPS, method_ops / (ms * 1e-3) / 1e12 / VALU_PEAK_TOPS)}
        r["frac"] = r["achieved"] / r["peak"]
        r.update(extra)
        return r

    fp32_direct = None
    if grouped:
        unverified = idx.debug_unverified_queries(reasons=True)
        kern = "adc_mfma_scan_kernel<%d,false,true,true>" % nb
        traffic, src = traffic_from_profiles(kern, workload)
        batch_roof = mfma_roofline(scan_ms, kern, {
            "traffic": traffic, "traffic_source": src, "sample_stage_ms": stage_ms.get("sample", 0.0),
            "queries_scanned_again": unverified[0],
            "stages_note": "before the scan over leaves, timed apart (sample_stage_ms): the bounds pass (leaf_bound_kernel "
                           "over each query's best leaves) and the regrouping of the (query, leaf) pairs"})
    elif prefiltered:
        unverified = idx.debug_unverified_queries(reasons=True)
        kern = "adc_mfma_scan_kernel<%d,false,false,true>" % nb
        traffic, src = traffic_from_profiles(kern, "%s_b%d" % (workload, B))
        batch_roof = mfma_roofline(scan_ms, kern, {
            "traffic": traffic, "traffic_source": src, "sample_stage_ms": stage_ms.get("sample", 0.0),
            "queries_scanned_again_with_fp32_tables": unverified[0],
            "of_which_too_many_kept_or_bound_too_high_or_other": unverified[1:],
            "stages_note": "the launch over all blocks of the candidate scan over the 8-bit tables; before it, timed apart "
                           "(sample_stage_ms): margins, a launch over a sample of the blocks and the bounds guessed from it; "
                           "the fp32 scores are formed for the kept points only (rescan stage)"})
        # the same step with every point scored in fp32 (the kernel the candidate scan replaces)
        idx.set_tuning("scan_prefilter", 1)
        dt_d, stage_d = timed_batch(avq.LUT_F32, max(2, args.steps // 5))
        idx.set_tuning("scan_prefilter", 0)
        fp32_direct = {"queries_per_s": B * max(2, args.steps // 5) / dt_d, "stage_ms": stage_d,
                       "roofline": lds_roofline(stage_d["scan"], B)}
        log("[bench] fp32 batch %d, every point scored in fp32: %.0f q/s, stages(ms) %s"
            % (B, fp32_direct["queries_per_s"], stage_d))
    else:
        batch_roof = lds_roofline(scan_ms, B)
        if tiled:
            idx.set_tuning("scan_prefilter", 1)
            dt_d, stage_d = timed_batch(avq.LUT_F32, max(2, args.steps // 5))
            idx.set_tuning("scan_prefilter", 0)
            fp32_direct = {"queries_per_s": B * max(2, args.steps // 5) / dt_d, "stage_ms": stage_d,
                           "roofline": lds_roofline(stage_d["scan"], B, every_point=True)}
            log("[bench] fp32 batch %d, every point scored in fp32: %.0f q/s, stages(ms) %s"
                % (B, fp32_direct["queries_per_s"], stage_d))
    log("[bench] fp32 batch %d: %.2f ms/step, %.0f q/s, stages(ms) %s" % (B, ms_per_step, qps, stage_ms))

    # ---- same with 8-bit tables ---------------------------------------------------------------
    steps8 = max(2, args.steps // 2)
    dt8, stage8_ms = timed_batch(avq.LUT_U8, steps8)
    qps8 = B * steps8 / dt8
    log("[bench] u8   batch %d: %.0f q/s, stages(ms) %s" % (B, qps8, stage8_ms))
    u8_roof = None
    if prefiltered:
        u8_roof = mfma_roofline(stage8_ms["scan"], "adc_mfma_scan_kernel<%d,false,false,true>" % nb,
                                {"traffic": None, "sample_stage_ms": stage8_ms.get("sample", 0.0)})

    # ---- other batch sizes the configuration names -----------------------------------------------
    extra = {}
    for bs in [int(v) for v in args.extra_batches.split(",") if v]:
        qq = qd_all[:bs].contiguous() if bs <= qd_all.shape[0] else None
        if qq is None:
            continue
        st_ = max(5, args.steps)
        dtb, stb = timed_batch(avq.LUT_F32, st_, qq)
        dtb8, stb8 = timed_batch(avq.LUT_U8, st_, qq)
        extra[str(bs)] = {"queries_per_s": bs * st_ / dtb, "ms_per_step": dtb / st_ * 1e3, "stage_ms": stb,
                          "u8_queries_per_s": bs * st_ / dtb8, "u8_stage_ms": stb8}
        log("[bench] fp32 batch %d: %.3f ms/step, stages(ms) %s" % (bs, dtb / st_ * 1e3, stb))

    # ---- timed region 2: single queries (the HBM-bound regime) ---------------------------------
    dt1, stage1_us = timed_single(avq.LUT_F32, args.b1_steps)
    code_bytes = float(nb) * scanned             # algorithmic bytes of one single-query scan
    bound_scan = not n_leaves and nb in SPECIAL_NB
    if n_leaves:
        # up to 80 queries on a partitioned index of these code sizes: exact block maxima over the probed leaves
        b1_kernel = ("leaf_block_max_kernel<false,%d>" % nb) if (bits == 4 and nb in SPECIAL_NB) else "adc_scan_kernel<1,false,%d,1>" % nb
        scan1_us = stage1_us["scan"]
        timing = "HIP event pair around the scan stage of every call (includes the pair's own cost)"
        parts = None
    else:
        # a code array beyond the 256 MB Infinity Cache is scanned by the variant with nontemporal loads
        streamed = ((n + 255) // 256) * 256 * nb > (256 << 20)
        b1_kernel = (("block_bound_stream_kernel<%d>" if streamed else "block_bound_kernel<%d>") % nb) if bound_scan else (
            ("block_max_nibble_kernel<false,%d>" % (nb if nb in SPECIAL_NB else 0)) if bits == 4 else "block_max_kernel<false,%d>" % nb)
        scan1_us = launches_us(0, avq.LUT_F32)
        timing = "200 launches back to back on the stream inside one HIP event pair"
        parts = {"code_stream_only_us": launches_us(1, avq.LUT_F32),
                 "lookups_only_us": launches_us(2, avq.LUT_F32) if bound_scan else None,
                 "note": "the same launch shape: stream_codes_kernel loads every code byte and folds the words (no "
                         "lookups); lookup_only_kernel does the scan's table lookups and additions on made-up code "
                         "words (no code stream). Each is what that half of the scan costs by itself"}
    traffic, src = traffic_from_profiles(b1_kernel, workload)
    b1_roof = {"bound": "hbm", "achieved": code_bytes / (scan1_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
               "unit": "GB/s", "traffic": traffic, "traffic_source": src, "kernel": b1_kernel,
               "avg_launch_ms": scan1_us / 1e3, "timing": timing,
               "scan_stage_event_pair_us": stage1_us["scan"], "parts": parts,
               "note": "algorithmic bytes = %d B of codes per scanned point; repeated scans of a code array below "
                       "256 MB are served from the Infinity Cache (see cold)" % nb}
    b1_roof["frac"] = b1_roof["achieved"] / b1_roof["peak"]
    log("[bench] fp32 batch 1: %.1f us/query end to end, stages(us) %s; scan kernel %.2f us back to back"
        % (dt1 / args.b1_steps * 1e6, stage1_us, scan1_us))
    if parts:
        log("[bench] code stream alone %.2f us, lookups alone %s us" % (parts["code_stream_only_us"], parts["lookups_only_us"]))
        evict = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        cold_us = launches_us(0, avq.LUT_F32, evict=evict)
        ev_us = launches_us(1, avq.LUT_F32, reps=1)  # a lone launch inside its own pair, warm: what the pair adds
        del evict
        b1_roof["cold"] = {"avg_launch_ms": cold_us / 1e3, "achieved": code_bytes / (cold_us * 1e-6) / 1e9,
                           "note": "1 GiB read through the Infinity Cache before every launch; one launch per event pair, "
                                   "so the figure includes the pair's cost (a lone warm launch of the stream-only kernel "
                                   "in its own pair reads %.1f us)" % ev_us}
        log("[bench] fp32 batch 1, cold cache: scan %.1f us" % cold_us)
    dt1u, stage1u_us = timed_single(avq.LUT_U8, max(100, args.b1_steps // 2))
    log("[bench] u8   batch 1: %.1f us/query end to end, stages(us) %s"
        % (dt1u / max(100, args.b1_steps // 2) * 1e6, stage1u_us))

    # ---- recall against exact search (untimed) ---------------------------------------------------
    nr = min(args.recall_queries, B)
    gt_ids, _ = idx.brute_force(qd[:nr].contiguous(), k)
    recall = {}
    for name, mode in (("f32", avq.LUT_F32), ("u8", avq.LUT_U8)):
        got_ids, _ = idx.search(qd[:nr].contiguous(), k, R, mode, Lp)
        torch.cuda.synchronize()
        g, t = got_ids.cpu().numpy(), gt_ids.cpu().numpy()
        recall[name] = float(np.mean([len(set(g[i]) & set(t[i])) / k for i in range(nr)]))
    log("[bench] recall@%d over %d queries: %s" % (k, nr, recall))

    # ---- CPU oracle on this host, bounded sample of the same workload ------------------------------
    cpu = cpu1 = cpu_bf = None
    parity = None
    if not args.no_cpu_baseline and x is not None:
        import oracle
        threads = oracle.num_threads()
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
        gi, gs = idx.search(qd[:no].contiguous(), k, R, avq.LUT_F32, Lp)
        torch.cuda.synchronize()
        parity = bool(np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gs.cpu().numpy(), os_))
        n8 = min(16, B)
        o8, s8 = oracle.search(x, cb, codes, bits, q[:n8], k, R, avq.LUT_U8, **okw)
        g8, gs8 = idx.search(qd[:n8].contiguous(), k, R, avq.LUT_U8, Lp)
        torch.cuda.synchronize()
        parity = parity and bool(np.array_equal(g8.cpu().numpy(), o8) and np.array_equal(gs8.cpu().numpy(), s8))
        # single queries through the one-query path
        g1, gs1 = idx.search(qd[:1].contiguous(), k, R, avq.LUT_F32, Lp)
        torch.cuda.synchronize()
        parity = parity and bool(np.array_equal(g1.cpu().numpy(), oi[:1]) and np.array_equal(gs1.cpu().numpy(), os_[:1]))
        sample = ("%d of the %d queries against all %d points (table build, ADC, full sort to top-%d, exact re-rank)"
                  % (no, B, n, R))
        cpu = {"value": no / dto, "unit": "queries/s", "cores": threads, "kind": "oracle",
               "sample": sample + ", OpenMP over queries", "host_cpus": os.cpu_count(), "seconds": dto}
        log("[bench] oracle: %d queries in %.1fs on %d threads; GPU results identical: %s" % (no, dto, threads, parity))
        # one thread (the paper's own protocol, Section 5.3), a few seconds of work
        n1 = max(1, min(no, int(round(no / dto * 4.0 / threads))))
        oracle.set_num_threads(1)
        t0 = time.perf_counter()
        oracle.search(x, cb, codes, bits, q[:n1], k, R, avq.LUT_F32, **okw)
        dt1t = time.perf_counter() - t0
        cpu1 = {"value": n1 / dt1t, "unit": "queries/s", "cores": 1, "kind": "oracle",
                "sample": "%d queries, same work, one thread" % n1, "seconds": dt1t}
        # exact search on the CPU (Section 2.2.2: O(nd) per query against the O(kd + mn) of the quantized scan)
        nbf = max(1, min(n1, int(round(n1 * M / float(d)))))
        t0 = time.perf_counter()
        oracle.brute_force(x, q[:nbf], k)
        dtbf = time.perf_counter() - t0
        cpu_bf = {"value": nbf / dtbf, "unit": "queries/s", "cores": 1, "kind": "oracle brute force",
                  "sample": "%d queries, exact <q, x> of all %d points, one thread" % (nbf, n), "seconds": dtbf}
        oracle.set_num_threads(threads)
        log("[bench] oracle, one thread: %.2f q/s quantized, %.2f q/s exact" % (cpu1["value"], cpu_bf["value"]))

    scan_desc = ("int8 matrix-core candidate scan + fp32 re-scoring of the kept points (results equal a full fp32 scan)"
                 if (prefiltered or grouped) else
                 ("block bounds from 8-bit table sums, exact scores of the blocks that can reach the R-th best"
                  if ((small and bound_scan) or tiled) else "fp32 table sums of every point"))
    out = {
        "metric": "queries/sec at Recall@10 vs brute force; ADC codes/sec and % HBM BW",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: n=%d d=%d PQ %dx%d (%d-bit, %d B/point) T=0.2%s, batch %d, "
                               "ADC top-%d re-ranked to top-%d"
                               % (args.config, n, d, M, 1 << bits, bits, nb,
                                  (", %d leaves, %d searched" % (n_leaves, Lp)) if n_leaves else "", B, R, k),
                   "lut": "f32", "train_s": t_train, "encode_s": t_encode, "scan": scan_desc},
        "recall_at_k": recall["f32"], "recall_at_k_u8": recall["u8"], "recall_k": k, "recall_queries": nr,
        "recall_at_10": recall["f32"] if k == 10 else None,
        "adc_points_per_s": scanned * B / (scan_ms * 1e-3),
        "adc_codes_per_s": scanned * B * M / (scan_ms * 1e-3),
        "stage_ms": stage_ms,
        "fp32_every_point": fp32_direct,
        "u8": {"queries_per_s": qps8, "stage_ms": stage8_ms,
               "adc_codes_per_s": scanned * B * M / (stage8_ms["scan"] * 1e-3), "roofline": u8_roof},
        "other_batches": extra or None,
        "roofline": batch_roof,
        "roofline_batch1": b1_roof,
        "batch1": {"queries_per_s": args.b1_steps / dt1, "us_per_query": dt1 / args.b1_steps * 1e6,
                   "steps": args.b1_steps, "stage_us": stage1_us,
                   "adc_points_per_s": scanned / (scan1_us * 1e-6),
                   "adc_codes_per_s": scanned * M / (scan1_us * 1e-6),
                   "hbm_frac": b1_roof["frac"],
                   "u8_us_per_query": dt1u / max(100, args.b1_steps // 2) * 1e6, "u8_stage_us": stage1u_us},
        "cpu_baseline": cpu, "cpu_baseline_1thread": cpu1, "cpu_brute_force_1thread": cpu_bf,
        "matches_oracle": parity,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
