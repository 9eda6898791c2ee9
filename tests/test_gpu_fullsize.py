"""GPU parity at the benchmark's full size and launch configuration.

The Glove-shaped workload (n = 1,183,514, d = 100, 50 x 16 codewords) is built by
the library itself exactly as bench.py builds it; the oracle then re-computes a
sample of the outputs from the library's own dictionaries and codes:
 * whole searches for a few queries (the oracle needs ~0.3 s per query at this n),
   taken out of the 10,000-query batch the benchmark times, and as single-query
   calls (the small-batch path);
 * ADC scores at sampled points, and properties that hold at any size.
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from util import unpack_codes

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
avq = pytest.importorskip("paper_1908_10396_amd")


@pytest.fixture(scope="module")
def glove():
    cfg = si.CONFIGS["glove"]
    x = si.make_data(cfg)
    q = si.make_queries(cfg, cfg["nq"])
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    idx = avq.Index(cfg["d"], cfg["M"], cfg["bits"], T=cfg["T"], kmeans_iters=20, encode_passes=10,
                    seed=cfg["seed"])
    idx.train(xd[: si.CHUNK])
    idx.encode(xd)
    cb = idx.get_codebooks()
    codes = unpack_codes(idx.get_codes(), cfg["M"], cfg["bits"])
    return dict(cfg=cfg, x=x, q=q, xd=xd, qd=qd, idx=idx, cb=cb, codes=codes)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_full_batch_matches_oracle_on_sampled_queries(glove, lut_mode):
    g = glove
    cfg = g["cfg"]
    k, R = cfg["k"], cfg["reorder_k"]
    ids, sc = g["idx"].search(g["qd"], k, R, lut_mode)          # the 10,000-query launch
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    sample = [0, 1, 4095, 5000, 9998, 9999]
    oi, os_ = oracle.search(g["x"], g["cb"], g["codes"], cfg["bits"], g["q"][sample], k, R, lut_mode)
    np.testing.assert_array_equal(ids[sample], oi)
    np.testing.assert_array_equal(sc[sample], os_)
    # properties at any size: ids valid and distinct, scores are the exact inner products, sorted
    assert ids.min() >= 0 and ids.max() < cfg["n"]
    assert all(len(set(row)) == k for row in ids[::97])
    assert np.all(np.diff(sc, axis=1) <= 0)
    rows = np.arange(0, cfg["nq"], 501)
    for r in rows:
        ex = oracle.exact_scores(g["x"][ids[r]], g["q"][r])
        np.testing.assert_array_equal(sc[r], ex)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_single_query_calls_match_oracle(glove, lut_mode):
    g = glove
    cfg = g["cfg"]
    k, R = cfg["k"], cfg["reorder_k"]
    sample = [3, 77, 2048]
    oi, os_ = oracle.search(g["x"], g["cb"], g["codes"], cfg["bits"], g["q"][sample], k, R, lut_mode)
    for j, qi in enumerate(sample):
        ids, sc = g["idx"].search(g["qd"][qi:qi + 1], k, R, lut_mode)
        np.testing.assert_array_equal(ids.cpu().numpy()[0], oi[j])
        np.testing.assert_array_equal(sc.cpu().numpy()[0], os_[j])
    # ADC candidates without re-ranking, R = 100 directly
    oi, os_ = oracle.search(None, g["cb"], g["codes"], cfg["bits"], g["q"][sample[:1]], R, 0, lut_mode)
    ids, sc = g["idx"].search(g["qd"][sample[0]:sample[0] + 1], R, 0, lut_mode)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_few_query_calls_repeat_the_batch_rows(glove, lut_mode):
    # the single-query and few-query paths (block maxima, block bounds of 16 queries a tile, the selections in one
    # workgroup) called again and again: every call returns the rows of the 10,000-query launch, which the
    # test above checks against the oracle. A race in one of those kernels shows as a row that differs now and then
    g = glove
    cfg = g["cfg"]
    k, R = cfg["k"], cfg["reorder_k"]
    ids, sc = g["idx"].search(g["qd"], k, R, lut_mode)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    for nq in (1, 2, 5, 16, 33, 40):
        for rep in range(150):
            lo = (61 * rep + 7 * nq) % (cfg["nq"] - nq)
            i1, s1 = g["idx"].search(g["qd"][lo:lo + nq], k, R, lut_mode)
            np.testing.assert_array_equal(i1.cpu().numpy(), ids[lo:lo + nq], err_msg="%d queries from %d, call %d" % (nq, lo, rep))
            np.testing.assert_array_equal(s1.cpu().numpy(), sc[lo:lo + nq])


def test_adc_scores_at_sampled_points(glove):
    g = glove
    cfg = g["cfg"]
    rng = np.random.default_rng(0)
    pts = np.concatenate([[0, 255, 256, cfg["n"] - 1], rng.integers(0, cfg["n"], 2000)])
    qsel = [0, 17]
    sf = g["idx"].debug_adc_scores(g["qd"][qsel].contiguous(), avq.LUT_F32).cpu().numpy()
    su = g["idx"].debug_adc_scores(g["qd"][qsel].contiguous(), avq.LUT_U8).cpu().numpy()
    for j, qi in enumerate(qsel):
        L = oracle.lut_f32(g["q"][qi], g["cb"])
        np.testing.assert_array_equal(sf[j][pts], oracle.adc_f32(L, g["codes"][pts], cfg["bits"]))
        Q8, _, _ = oracle.lut_u8(L)
        np.testing.assert_array_equal(su[j][pts], oracle.adc_u8(Q8, g["codes"][pts]).astype(np.int32))


def test_library_codes_are_the_oracles_codes_on_a_sample(glove):
    g = glove
    cfg = g["cfg"]
    rng = np.random.default_rng(1)
    pts = rng.integers(0, cfg["n"], 3000)
    want = oracle.encode(g["x"][pts], g["cb"], T=cfg["T"], passes=10)
    assert np.mean(np.any(want != g["codes"][pts], axis=1)) <= 1e-3
    # training sample: the library's dictionaries against the oracle's k-means on the same rows
    cb = oracle.train_pq(g["x"][: si.CHUNK], cfg["M"], 16, 20, seed=cfg["seed"])
    np.testing.assert_allclose(g["cb"], cb, rtol=0, atol=2e-6)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_full_partitioned_batch_matches_oracle_on_sampled_queries(lut_mode):
    # the partitioned Glove-shaped workload as bench.py --config glove_ivf runs it (2,000 leaves, 100
    # probed, 10,000 queries per launch: leaves scanned on the matrix cores, pairs regrouped by leaf)
    cfg = si.CONFIGS["glove_ivf"]
    x = si.make_data(cfg)
    q = si.make_queries(cfg, cfg["nq"])
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    idx = avq.Index(cfg["d"], cfg["M"], cfg["bits"], T=cfg["T"], n_leaves=cfg["n_leaves"], kmeans_iters=10,
                    encode_passes=5, seed=cfg["seed"])
    idx.train(xd[: si.CHUNK])
    idx.encode(xd)
    k, R, L = cfg["k"], cfg["reorder_k"], cfg["leaves_to_search"]
    ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    sample = [0, 1, 2500, 4097, 7777, 9999]
    oi, os_ = oracle.search(x, idx.get_codebooks(), unpack_codes(idx.get_codes(), cfg["M"], cfg["bits"]), cfg["bits"],
                            q[sample], k, R, lut_mode, centers=idx.get_leaf_centers(), assign=idx.get_leaf_assign(),
                            leaves_to_search=L)
    np.testing.assert_array_equal(ids[sample], oi)
    np.testing.assert_array_equal(sc[sample], os_)
    assert np.all(np.diff(sc, axis=1) <= 0)
    if lut_mode == 0:
        # leaf selection of the whole batch (10,000 queries: eight queries per workgroup, leaf_select_tile_kernel)
        lids, lip = idx.debug_leaf_select(qd, L)
        lids, lip = lids.cpu().numpy(), lip.cpu().numpy()
        centers = idx.get_leaf_centers()
        for qi in sample:
            li, lp = oracle.leaf_select(centers, q[qi], L)
            np.testing.assert_array_equal(lids[qi], li)
            np.testing.assert_array_equal(lip[qi], lp)
    back = idx.debug_unverified_queries()
    assert 0 <= back < cfg["nq"] // 4          # most queries stay on the regrouped path
    # the one-query-per-workgroup scan gives the same batch
    idx.set_tuning("scan_prefilter", 1)
    ids2, sc2 = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
    np.testing.assert_array_equal(ids2.cpu().numpy(), ids)
    np.testing.assert_array_equal(sc2.cpu().numpy(), sc)
    idx.set_tuning("scan_prefilter", 0)
    # single queries and a batch of 16 (block maxima over the ~290 blocks of the probed leaves) give the batch's rows
    for qi in sample[:4]:
        i1, s1 = idx.search(qd[qi:qi + 1], k, R, lut_mode, leaves_to_search=L)
        np.testing.assert_array_equal(i1.cpu().numpy()[0], ids[qi])
        np.testing.assert_array_equal(s1.cpu().numpy()[0], sc[qi])
    i16, s16 = idx.search(qd[4090:4106], k, R, lut_mode, leaves_to_search=L)
    np.testing.assert_array_equal(i16.cpu().numpy(), ids[4090:4106])
    np.testing.assert_array_equal(s16.cpu().numpy(), sc[4090:4106])
    # many times over: one call in ten once came back with a row wrong (the 16 waves of the workgroup that selects
    # the leaves did not all see the same narrowed key range)
    for rep in range(12):
        lo = 100 + 613 * rep
        for nq in (16, 80):
            ib, sb = idx.search(qd[lo:lo + nq], k, R, lut_mode, leaves_to_search=L)
            np.testing.assert_array_equal(ib.cpu().numpy(), ids[lo:lo + nq], err_msg="rows %d..%d" % (lo, lo + nq))
            np.testing.assert_array_equal(sb.cpu().numpy(), sc[lo:lo + nq])

    # 300 leaves: about 870 blocks of 256 points per query, more than the few-query selection of the blocks ranks
    # directly (it narrows the range of their maxima first)
    L3 = 300
    ids3, sc3 = idx.search(qd[:2048], k, R, lut_mode, leaves_to_search=L3)
    ids3, sc3 = ids3.cpu().numpy(), sc3.cpu().numpy()
    o3, os3 = oracle.search(x, idx.get_codebooks(), unpack_codes(idx.get_codes(), cfg["M"], cfg["bits"]), cfg["bits"],
                            q[[5, 2047]], k, R, lut_mode, centers=idx.get_leaf_centers(), assign=idx.get_leaf_assign(),
                            leaves_to_search=L3)
    np.testing.assert_array_equal(ids3[[5, 2047]], o3)
    np.testing.assert_array_equal(sc3[[5, 2047]], os3)
    for rep in range(10):
        lo = 11 + 197 * rep
        for nq in (1, 5, 16):
            ib, sb = idx.search(qd[lo:lo + nq], k, R, lut_mode, leaves_to_search=L3)
            np.testing.assert_array_equal(ib.cpu().numpy(), ids3[lo:lo + nq], err_msg="300 leaves, rows %d..%d" % (lo, lo + nq))
            np.testing.assert_array_equal(sb.cpu().numpy(), sc3[lo:lo + nq])


def test_leaf_select_for_few_queries_is_repeatable():
    # up to 32 queries take a kernel pair of their own (scores by many small workgroups, then one 1024-thread
    # workgroup per query that selects): same leaves as the batch kernels and the oracle, call after call
    cfg = si.CONFIGS["glove_ivf"]
    x = si.make_data(cfg)
    q = si.make_queries(cfg, 2048)
    xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    idx = avq.Index(cfg["d"], cfg["M"], cfg["bits"], T=cfg["T"], n_leaves=cfg["n_leaves"], kmeans_iters=10,
                    encode_passes=5, seed=cfg["seed"])
    idx.train(xd[: si.CHUNK])
    centers = idx.get_leaf_centers()
    for L in (1, 100, 512):
        ref_ids, ref_ip = idx.debug_leaf_select(qd, L)
        ref_ids, ref_ip = ref_ids.cpu().numpy(), ref_ip.cpu().numpy()
        for qi in (0, 777, 2047):
            li, lp = oracle.leaf_select(centers, q[qi], L)
            np.testing.assert_array_equal(ref_ids[qi], li)
            np.testing.assert_array_equal(ref_ip[qi], lp)
        for rep in range(60):
            lo = (53 * rep) % 2000
            for nq in (1, 5, 16, 32):
                ids, ip = idx.debug_leaf_select(qd[lo:lo + nq], L)
                np.testing.assert_array_equal(ids.cpu().numpy(), ref_ids[lo:lo + nq], err_msg="L=%d rows %d..%d" % (L, lo, lo + nq))
                np.testing.assert_array_equal(ip.cpu().numpy(), ref_ip[lo:lo + nq])
