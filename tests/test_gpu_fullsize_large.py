"""GPU parity at the two large configurations, in the launch shapes bench.py times.

 * Large 4-bit (10,000,000 x 128, 64 subspaces x 16 codewords, top-200 -> top-10): the
   index is built by the library at full size; the oracle recomputes whole searches
   for sampled queries of the 1,024-query launch, of a 64-query launch and of
   single-query calls, for both table kinds, from the library's own dictionaries and
   codes. At this size the matrix-core scan runs tens of chunks with 18-bit
   chunk-local ids and the single-query path ranks 39,063 block maxima.
 * Large 8-bit (256 dims, 32 subspaces x 256 codewords, per-point eta from log-normal
   norms, top-500 -> top-100): a slice of 4,000,123 points is trained, encoded and
   searched (batches of 1,024 and 1); separately the ADC scan and selection run over
   the full 50,000,000 points on synthetic uniformly drawn codes (no datapoints, so
   no exact re-ranking), which reaches the ids and block counts of the full size.
The oracle needs seconds per query here, so a handful of queries is compared
element by element; properties that hold at any size are checked on all of them.
"""
import gc

import numpy as np
import pytest

import oracle
import synth_inputs as si
from util import unpack_codes

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
avq = pytest.importorskip("paper_1908_10396_amd")


def log(msg):
    print("[fullsize-large] " + msg, flush=True)


# ---------------------------------------------------------------------------- large4

L4_SAMPLE = [0, 1, 31, 63, 500, 1023]      # the first four also lie in the 64-query launch


@pytest.fixture(scope="module")
def large4():
    cfg = si.CONFIGS["large4"]
    log("large4: generating %d x %d points" % (cfg["n"], cfg["d"]))
    x = si.make_data(cfg)
    q = si.make_queries(cfg, cfg["nq"])
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    idx = avq.Index(cfg["d"], cfg["M"], cfg["bits"], T=cfg["T"], kmeans_iters=20, encode_passes=10,
                    seed=cfg["seed"])
    idx.train(xd[: si.CHUNK])
    idx.encode(xd)
    log("large4: index built")
    cb = idx.get_codebooks()
    codes = unpack_codes(idx.get_codes(), cfg["M"], cfg["bits"])
    g = dict(cfg=cfg, x=x, q=q, xd=xd, qd=qd, idx=idx, cb=cb, codes=codes, want={})
    yield g
    idx.close()
    g.clear()
    del x, xd, codes
    gc.collect()
    torch.cuda.empty_cache()


def _large4_oracle(g, lut_mode):
    if lut_mode not in g["want"]:
        cfg = g["cfg"]
        log("large4: oracle on %d queries, lut_mode %d" % (len(L4_SAMPLE), lut_mode))
        g["want"][lut_mode] = oracle.search(g["x"], g["cb"], g["codes"], cfg["bits"], g["q"][L4_SAMPLE],
                                            cfg["k"], cfg["reorder_k"], lut_mode)
    return g["want"][lut_mode]


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_large4_batches_of_1024_64_and_1_match_oracle(large4, lut_mode):
    g = large4
    cfg = g["cfg"]
    k, R, n = cfg["k"], cfg["reorder_k"], cfg["n"]
    oi, os_ = _large4_oracle(g, lut_mode)
    # the 1,024-query launch
    ids, sc = g["idx"].search(g["qd"], k, R, lut_mode)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    np.testing.assert_array_equal(ids[L4_SAMPLE], oi)
    np.testing.assert_array_equal(sc[L4_SAMPLE], os_)
    assert ids.min() >= 0 and ids.max() < n
    assert all(len(set(row)) == k for row in ids)
    assert np.all(np.diff(sc, axis=1) <= 0)
    for r in range(0, cfg["nq"], 93):
        np.testing.assert_array_equal(sc[r], oracle.exact_scores(g["x"][ids[r]], g["q"][r]))
    # a 64-query launch (its chunks are shorter: another plan of the same kernels)
    ids64, sc64 = g["idx"].search(g["qd"][:64].contiguous(), k, R, lut_mode)
    ids64, sc64 = ids64.cpu().numpy(), sc64.cpu().numpy()
    np.testing.assert_array_equal(ids64, ids[:64])
    np.testing.assert_array_equal(sc64, sc[:64])
    in64 = [j for j, qi in enumerate(L4_SAMPLE) if qi < 64]
    np.testing.assert_array_equal(ids64[[L4_SAMPLE[j] for j in in64]], oi[in64])
    # single-query calls (block maxima, selection of the best blocks, rescan)
    for j, qi in enumerate(L4_SAMPLE):
        i1, s1 = g["idx"].search(g["qd"][qi:qi + 1], k, R, lut_mode)
        np.testing.assert_array_equal(i1.cpu().numpy()[0], oi[j])
        np.testing.assert_array_equal(s1.cpu().numpy()[0], os_[j])
    # single- and few-query calls again and again (selection split over many workgroups, the last one finishing):
    # always the rows of the 1,024-query launch
    for nq in (1, 3, 12, 20):
        for rep in range(60):
            lo = (37 * rep + nq) % (cfg["nq"] - nq)
            i1, s1 = g["idx"].search(g["qd"][lo:lo + nq], k, R, lut_mode)
            np.testing.assert_array_equal(i1.cpu().numpy(), ids[lo:lo + nq], err_msg="%d queries from %d, call %d" % (nq, lo, rep))
            np.testing.assert_array_equal(s1.cpu().numpy(), sc[lo:lo + nq])


def test_large4_adc_candidates_without_reranking(large4):
    # reorder_k = 0: the R best by ADC score, ids up to 10^7, both table kinds, batch and single
    g = large4
    cfg = g["cfg"]
    R = cfg["reorder_k"]
    sample = [5, 40]
    for lut_mode in (0, 1):
        oi, os_ = oracle.search(None, g["cb"], g["codes"], cfg["bits"], g["q"][sample], R, 0, lut_mode)
        ids, sc = g["idx"].search(g["qd"][:64].contiguous(), R, 0, lut_mode)
        np.testing.assert_array_equal(ids.cpu().numpy()[sample], oi)
        np.testing.assert_array_equal(sc.cpu().numpy()[sample], os_)
        i1, s1 = g["idx"].search(g["qd"][sample[0]:sample[0] + 1], R, 0, lut_mode)
        np.testing.assert_array_equal(i1.cpu().numpy()[0], oi[0])
        np.testing.assert_array_equal(s1.cpu().numpy()[0], os_[0])


def test_large4_adc_scores_and_codes_at_sampled_points(large4):
    g = large4
    cfg = g["cfg"]
    n = cfg["n"]
    rng = np.random.default_rng(4)
    pts = np.concatenate([[0, 255, 256, (1 << 18) - 1, 1 << 18, n - 257, n - 1], rng.integers(0, n, 3000)])
    qsel = [0, 900]
    sf = g["idx"].debug_adc_scores(g["qd"][qsel].contiguous(), avq.LUT_F32).cpu().numpy()
    for j, qi in enumerate(qsel):
        L = oracle.lut_f32(g["q"][qi], g["cb"])
        np.testing.assert_array_equal(sf[j][pts], oracle.adc_f32(L, g["codes"][pts], cfg["bits"]))
    del sf
    # 8-bit tables through the matrix-core kernel's store mode (32 queries: its smallest tile)
    q32 = g["qd"][:32].contiguous()
    su = g["idx"].debug_adc_scores(q32, avq.LUT_U8)[[0, 31]].cpu().numpy()
    for j, qi in enumerate([0, 31]):
        Q8, _, _ = oracle.lut_u8(oracle.lut_f32(g["q"][qi], g["cb"]))
        np.testing.assert_array_equal(su[j][pts], oracle.adc_u8(Q8, g["codes"][pts]).astype(np.int32))
    # the library's codes are the oracle's on a sample spread over the whole index
    pts = rng.integers(0, n, 2000)
    want = oracle.encode(g["x"][pts], g["cb"], T=cfg["T"], passes=10)
    assert np.mean(np.any(want != g["codes"][pts], axis=1)) <= 1e-3


# ---------------------------------------------------------------------------- large8

L8_N = 4_000_123
L8_SAMPLE = [0, 1, 512, 1023]


@pytest.fixture(scope="module")
def large8():
    cfg = dict(si.CONFIGS["large8"])
    log("large8: generating %d x %d points (slice of the 5e7-point configuration)" % (L8_N, cfg["d"]))
    x = si.make_data(cfg, L8_N)
    q = si.make_queries(cfg, cfg["nq"])
    xd = torch.from_numpy(x).cuda()
    qd = torch.from_numpy(q).cuda()
    idx = avq.Index(cfg["d"], cfg["M"], cfg["bits"], T=cfg["T"], kmeans_iters=20, encode_passes=10,
                    seed=cfg["seed"], borrow_x=True)
    idx.train(xd[: si.CHUNK])
    idx.encode(xd)
    log("large8: index built")
    cb = idx.get_codebooks()
    codes = idx.get_codes()
    g = dict(cfg=cfg, x=x, q=q, xd=xd, qd=qd, idx=idx, cb=cb, codes=codes)
    yield g
    idx.close()
    g.clear()
    del x, xd, codes
    gc.collect()
    torch.cuda.empty_cache()


def test_large8_norms_are_lognormal_and_codes_are_the_oracles(large8):
    g = large8
    cfg = g["cfg"]
    nrm = np.linalg.norm(g["x"][:100000].astype(np.float64), axis=1)
    assert abs(np.log(nrm).std() - 0.25) < 0.01 and abs(np.log(nrm).mean()) < 0.01
    rng = np.random.default_rng(8)
    pts = rng.integers(0, L8_N, 600)
    want = oracle.encode(g["x"][pts], g["cb"], T=cfg["T"], passes=10)      # eta per point from its own norm
    assert np.mean(np.any(want != g["codes"][pts], axis=1)) <= 2e-3
    # eta = 1 would give other codes for a good part of these points: the per-point eta matters
    l2 = oracle.encode(g["x"][pts[:100]], g["cb"], T=0.0, passes=10)
    assert np.mean(np.any(l2 != g["codes"][pts[:100]], axis=1)) > 0.2


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_large8_slice_batches_of_1024_and_1_match_oracle(large8, lut_mode):
    g = large8
    cfg = g["cfg"]
    k, R = cfg["k"], cfg["reorder_k"]
    log("large8: oracle on %d queries, lut_mode %d" % (len(L8_SAMPLE), lut_mode))
    oi, os_ = oracle.search(g["x"], g["cb"], g["codes"], cfg["bits"], g["q"][L8_SAMPLE], k, R, lut_mode)
    ids, sc = g["idx"].search(g["qd"], k, R, lut_mode)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    np.testing.assert_array_equal(ids[L8_SAMPLE], oi)
    np.testing.assert_array_equal(sc[L8_SAMPLE], os_)
    assert ids.min() >= 0 and ids.max() < L8_N
    assert all(len(set(row)) == k for row in ids[::37])
    assert np.all(np.diff(sc, axis=1) <= 0)
    for r in range(0, cfg["nq"], 171):
        np.testing.assert_array_equal(sc[r], oracle.exact_scores(g["x"][ids[r]], g["q"][r]))
    for j, qi in enumerate(L8_SAMPLE):
        i1, s1 = g["idx"].search(g["qd"][qi:qi + 1], k, R, lut_mode)
        np.testing.assert_array_equal(i1.cpu().numpy()[0], oi[j])
        np.testing.assert_array_equal(s1.cpu().numpy()[0], os_[j])
    for nq in (1, 2, 5):
        for rep in range(40):
            lo = (41 * rep + nq) % (cfg["nq"] - nq)
            i1, s1 = g["idx"].search(g["qd"][lo:lo + nq], k, R, lut_mode)
            np.testing.assert_array_equal(i1.cpu().numpy(), ids[lo:lo + nq], err_msg="%d queries from %d, call %d" % (nq, lo, rep))
            np.testing.assert_array_equal(s1.cpu().numpy(), sc[lo:lo + nq])


def test_large8_adc_scores_at_sampled_points(large8):
    g = large8
    cfg = g["cfg"]
    rng = np.random.default_rng(9)
    pts = np.concatenate([[0, 255, 256, L8_N - 1], rng.integers(0, L8_N, 3000)])
    qsel = [3, 700]
    sf = g["idx"].debug_adc_scores(g["qd"][qsel].contiguous(), avq.LUT_F32).cpu().numpy()
    su = g["idx"].debug_adc_scores(g["qd"][qsel].contiguous(), avq.LUT_U8).cpu().numpy()
    for j, qi in enumerate(qsel):
        L = oracle.lut_f32(g["q"][qi], g["cb"])
        np.testing.assert_array_equal(sf[j][pts], oracle.adc_f32(L, g["codes"][pts], cfg["bits"]))
        Q8, _, _ = oracle.lut_u8(L)
        np.testing.assert_array_equal(su[j][pts], oracle.adc_u8(Q8, g["codes"][pts]).astype(np.int32))


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_large8_full_size_adc_scan_and_selection_on_synthetic_codes(large8, lut_mode):
    # all 50,000,000 points: 1.6 GB of uniformly drawn 8-bit codes against the slice's dictionaries;
    # no datapoints are installed, so reorder_k = 0 and the R = 500 best ADC candidates are compared
    cfg = large8["cfg"]
    n, M, R = cfg["n"], cfg["M"], cfg["reorder_k"]
    log("large8: %d synthetic codes, lut_mode %d" % (n, lut_mode))
    codes = np.empty((n, M), np.uint8)
    for c, lo, hi in si._chunks(n):
        codes[lo:hi] = np.random.default_rng([cfg["seed"], 7, c]).integers(0, 256, (hi - lo, M), dtype=np.uint8)
    # the best possible code word for query 0 planted three times, far apart: equal scores at the very
    # top of its list, the lower id must come first (ids beyond 2^25 and the last point among them)
    best = np.argmax(oracle.lut_f32(large8["q"][0], large8["cb"]), axis=1).astype(np.uint8)
    codes[12345] = codes[31_000_000] = codes[n - 1] = best
    idx = avq.Index(cfg["d"], M, cfg["bits"], T=cfg["T"], seed=cfg["seed"])
    idx.set_codebooks(large8["cb"])
    idx.set_database(None, torch.from_numpy(codes).cuda())
    sample = [0, 7, 1023]
    oi, os_ = oracle.search(None, large8["cb"], codes, cfg["bits"], large8["q"][sample], R, 0, lut_mode)
    ids, sc = idx.search(large8["qd"], R, 0, lut_mode)
    ids, sc = ids.cpu().numpy(), sc.cpu().numpy()
    np.testing.assert_array_equal(ids[sample], oi)
    np.testing.assert_array_equal(sc[sample], os_)
    assert list(oi[0][:3]) == [12345, 31_000_000, n - 1]
    assert ids.min() >= 0 and ids.max() < n and ids.max() > (1 << 25)
    for j, qi in enumerate(sample[:2]):
        i1, s1 = idx.search(large8["qd"][qi:qi + 1], R, 0, lut_mode)
        np.testing.assert_array_equal(i1.cpu().numpy()[0], oi[j])
        np.testing.assert_array_equal(s1.cpu().numpy()[0], os_[j])
    idx.close()
