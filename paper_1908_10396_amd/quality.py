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
   estimate of the exact top-1 pair (Figure 2b), mean and median.

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="glove", choices=["tiny", "glove", "large4"])
    ap.add_argument("--queries", type=int, default=256)
    ap.add_argument("--n", type=int, default=0, help="use only the first N points")
    ap.add_argument("--T", type=float, default=0.2)
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
    top_n = [1, 2, 5, 10, 20, 50, 100]
    kmax = min(max(top_n), n)

    base = avq.Index(d, M, bits, T=args.T, kmeans_iters=20, encode_passes=10, seed=cfg["seed"])
    base.train(xd[:n_train])
    codebooks = base.get_codebooks()
    gt_ids = gt_sc = None

    out = {"config": args.config, "n": n, "d": d, "M": M, "bits": bits, "T": args.T, "queries": args.queries,
           "eta_anisotropic": avq.eta(d, args.T, 1.0), "losses": {}}
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
        if gt_ids is None:                                     # exact top-1 (the same for both encodings)
            gi, gs = idx.brute_force(qd, 1)
            gt_ids, gt_sc = gi.cpu().numpy()[:, 0], gs.cpu().numpy()[:, 0]
        ids, _ = idx.search(qd, kmax, 0, avq.LUT_F32)          # ADC order, no re-ranking
        ids = ids.cpu().numpy()
        recall = {}
        for N in top_n:
            if N <= kmax:
                recall["1@%d" % N] = float(np.mean([gt_ids[i] in ids[i, :N] for i in range(args.queries)]))
        # ADC estimate of the exact top-1 pair, from the scores of every point
        rel = []
        step = 32
        for i0 in range(0, args.queries, step):
            sc = idx.debug_adc_scores(qd[i0:i0 + step].contiguous(), avq.LUT_F32)
            rows = torch.arange(sc.shape[0], device="cuda")
            est = sc[rows, torch.from_numpy(gt_ids[i0:i0 + step].astype(np.int64)).cuda()].cpu().numpy()
            rel.append(np.abs(est - gt_sc[i0:i0 + step]) / np.abs(gt_sc[i0:i0 + step]))
        rel = np.concatenate(rel)
        out["losses"][name] = {"recall": recall, "rel_error_top1_mean": float(rel.mean()),
                               "rel_error_top1_median": float(np.median(rel))}
        print("%-28s %s  rel.err mean %.4f median %.4f" % (name, " ".join("%s=%.3f" % kv for kv in recall.items()),
                                                           rel.mean(), np.median(rel)), file=sys.stderr, flush=True)
        idx.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
