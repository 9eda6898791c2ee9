"""Quality of the quantisation on synthetic data, in the paper's own terms.

    python -m paper_1908_10396_amd.quality [--config glove] [--queries 256] [--n N] [--alternations K]

Encodes the same datapoints with the same k-means dictionaries -- once with the
reconstruction loss (eta = 1) and once with the anisotropic loss (eta from
T = 0.2, Section 3.2) -- then, with --alternations K, K more rounds of
Section 4.2's alternation (dictionary update with the codes fixed, then
re-assignment), and reports, for the ADC scores without re-ranking:

 * Recall 1@N: how often the exact top-1 of a query is among its N best ADC
   scores (the metric of Section 5.2 / Figure 2a);
 * the relative error |<q, x~> - <q, x>| / |<q, x>| of the inner-product
   estimate of the exact top-1 pair (Figure 2b), mean and median;
 * the same two for a sweep of the threshold T with the dictionary held fixed
   (Section 5.1, Figure 2a: T = 0 is the reconstruction loss).

Everything runs through the library's C ABI on the GPU (train, encode,
brute force, search with reorder_k = 0, inspection of ADC scores). The paper's
datasets are not available here; the inputs are the seeded synthetic ones of
synth_inputs.py, so the numbers show the direction of the effect, not the
paper's values.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


TOP_N = (1, 2, 5, 10, 20, 50, 100)


def measure(idx, xd, qd, top_n=TOP_N, gt=None):
    """Metrics of one encoded index (Section 5.2), all through the C ABI on the GPU.

    Returns (hits, rel, gt): hits[N] = number of queries whose exact top-1 datapoint is among the N best ADC
    scores (Recall 1@N = hits[N] / queries; ADC order without re-ranking, fp32 tables); rel[i] = relative error
    |<q_i, x~> - <q_i, x>| / |<q_i, x>| of the ADC estimate for query i's exact top-1 pair (Figure 2b);
    gt = (ids, scores) of the exact top-1, reusable for other encodings of the same data."""
    import numpy as np
    import torch
    from . import LUT_F32
    nq = qd.shape[0]
    if gt is None:
        gi, gs = idx.brute_force(qd, 1)
        gt = (gi.cpu().numpy()[:, 0], gs.cpu().numpy()[:, 0])
    gt_ids, gt_sc = gt
    kmax = min(max(top_n), idx.n)
    ids, _ = idx.search(qd, kmax, 0, LUT_F32)
    ids = ids.cpu().numpy()
    hits = {N: int(sum(gt_ids[i] in ids[i, :N] for i in range(nq))) for N in top_n if N <= kmax}
    rel = []
    for i0 in range(0, nq, 32):
        sc = idx.debug_adc_scores(qd[i0:i0 + 32].contiguous(), LUT_F32)
        rows = torch.arange(sc.shape[0], device="cuda")
        est = sc[rows, torch.from_numpy(gt_ids[i0:i0 + 32].astype(np.int64)).cuda()].cpu().numpy()
        rel.append(np.abs(est - gt_sc[i0:i0 + 32]) / np.abs(gt_sc[i0:i0 + 32]))
    return hits, np.concatenate(rel), gt


def sweep_T(xd, qd, d, M, bits, codebooks, Ts, seed=0, encode_passes=10, top_n=TOP_N):
    """Figure 2a's protocol: one dictionary (learned under the l2 loss), the datapoints re-assigned under the
    anisotropic loss for each threshold T (T = 0 is the reconstruction loss: eta = 1). {T: (hits, rel)}."""
    from . import Index
    out, gt = {}, None
    for T in Ts:
        idx = Index(d, M, bits, T=T, encode_passes=encode_passes, seed=seed)
        idx.set_codebooks(codebooks)
        idx.encode(xd)
        hits, rel, gt = measure(idx, xd, qd, top_n, gt)
        out[T] = (hits, rel)
        idx.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="glove", choices=["tiny", "glove", "large4"])
    ap.add_argument("--queries", type=int, default=256)
    ap.add_argument("--n", type=int, default=0, help="use only the first N points")
    ap.add_argument("--T", type=float, default=0.2)
    ap.add_argument("--T-sweep", default="0,0.1,0.2,0.3,0.5",
                    help="thresholds of the sweep of Section 5.1 (Figure 2a); empty: no sweep")
    ap.add_argument("--alternations", type=int, default=0,
                    help="rounds of (dictionary update, re-assignment) under the anisotropic loss")
    args = ap.parse_args()

    import torch
    import paper_1908_10396_amd as avq
    import synth_inputs as si

    cfg = dict(si.CONFIGS[args.config])
    if args.n:
        cfg["n"] = args.n
    n, d, M, bits = cfg["n"], cfg["d"], cfg["M"], cfg["bits"]
    x = si.make_data(cfg)
    q = si.make_queries(cfg, args.queries)
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    n_train = min(n, si.CHUNK)

    base = avq.Index(d, M, bits, T=args.T, kmeans_iters=20, encode_passes=10, seed=cfg["seed"])
    base.train(xd[:n_train])
    codebooks = base.get_codebooks()
    gt = None

    out = {"config": args.config, "n": n, "d": d, "M": M, "bits": bits, "T": args.T, "queries": args.queries,
           "eta_anisotropic": avq.eta(d, args.T, 1.0), "losses": {}, "T_sweep": {}}

    def report(name, hits, rel):
        recall = {"1@%d" % N: h / args.queries for N, h in hits.items()}
        print("%-36s %s  rel.err mean %.4f median %.4f" % (name, " ".join("%s=%.3f" % kv for kv in recall.items()),
                                                           rel.mean(), np.median(rel)), file=sys.stderr, flush=True)
        return {"recall": recall, "hits": {str(N): h for N, h in hits.items()}, "rel_error_top1_mean": float(rel.mean()),
                "rel_error_top1_median": float(np.median(rel))}

    variants = [("reconstruction (eta = 1)", dict(eta_mode=avq.ETA_EXPLICIT, eta_explicit=1.0), 0),
                ("anisotropic (T = %g)" % args.T, dict(eta_mode=avq.ETA_LIMIT), 0)]
    if args.alternations:
        variants.append(("anisotropic + %d dictionary updates" % args.alternations, dict(eta_mode=avq.ETA_LIMIT),
                         args.alternations))
    for name, kw, rounds in variants:
        idx = avq.Index(d, M, bits, T=args.T, kmeans_iters=20, encode_passes=10, seed=cfg["seed"], **kw)
        idx.set_codebooks(codebooks)
        idx.encode(xd)
        for r in range(rounds):
            t0 = time.time()
            iters, rel = idx.update_codebooks(xd, max_iters=2000, tol=1e-8)
            t1 = time.time()
            idx.encode(xd)
            torch.cuda.synchronize()
            print("  round %d: update %.3f s (%d CG iterations, residual %.1e), re-assignment %.3f s"
                  % (r + 1, t1 - t0, iters, rel, time.time() - t1), file=sys.stderr, flush=True)
        hits, rel, gt = measure(idx, xd, qd, TOP_N, gt)
        out["losses"][name] = report(name, hits, rel)
        idx.close()
    Ts = [float(t) for t in args.T_sweep.split(",") if t]
    if Ts:
        for T, (hits, rel) in sweep_T(xd, qd, d, M, bits, codebooks, Ts, seed=cfg["seed"]).items():
            out["T_sweep"]["%g" % T] = report("T = %g (eta = %.3f)" % (T, avq.eta(d, T, 1.0)), hits, rel)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
