"""GPU parity: every stage of the HIP path against the CPU oracle, element by
element, on the same seeded inputs. All calls go through the C ABI (via the
ctypes binding). Bars: integer / index / byte results bit-exact; the fp32 path
follows the oracle's operation order, so it is held to exact equality too
(tighter than the 1e-5 relative tolerance the target states), and the
tolerance is asserted separately so a regression shows which bar broke.
"""
import os

import numpy as np
import pytest

import oracle
import synth_inputs as si
from util import unit_rows, unpack_codes

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
avq = pytest.importorskip("paper_1908_10396_amd")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_case(seed, n, d, M, bits, nq, train_iters=4, n_train=None):
    """Synthetic unit-norm data, oracle-trained dictionaries and oracle codes."""
    rng = np.random.default_rng(seed)
    x = unit_rows(rng, n, d)
    q = unit_rows(rng, nq, d)
    kc = 1 << bits
    nt = min(n, n_train or 4000)
    cb = oracle.train_pq(x[:max(nt, kc)], M, kc, train_iters, seed=seed)
    codes = oracle.encode(x, cb, T=0.2, passes=3)
    return dict(x=x, q=q, cb=cb, codes=codes, n=n, d=d, M=M, bits=bits, kc=kc)


def make_index(case, **kw):
    idx = avq.Index(case["d"], case["M"], case["bits"], T=0.2, **kw)
    idx.set_codebooks(case["cb"])
    xd = dev(case["x"])
    idx.set_database(xd, oracle.pack_codes(case["codes"], case["bits"]))
    return idx, xd


CASES = {
    # name: (n, d, M, bits, nq)  -- several 256-point blocks plus a ragged tail
    "tiny_nb8": (10_000, 32, 16, 4, 100),
    "glove_nb25": (6_011, 100, 50, 4, 37),
    "large4_nb32": (3_333, 128, 64, 4, 21),
    "large8_nb32": (2_500, 256, 32, 8, 19),
    "generic_nb7": (1_999, 28, 14, 4, 9),
    "odd_m_nb4": (1_030, 21, 7, 4, 5),
    "odd_m_nb25": (2_100, 98, 49, 4, 40),
    "bits100_nb13": (3_000, 100, 25, 4, 33),
    "bits8_nb3": (777, 12, 3, 8, 6),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    n, d, M, bits, nq = CASES[request.param]
    c = make_case(100 + list(CASES).index(request.param), n, d, M, bits, nq)
    c["name"] = request.param
    return c


def test_lut_tables_match(case):
    idx, _ = make_index(case)
    qd = dev(case["q"])
    L = idx.debug_lut(qd, avq.LUT_F32).cpu().numpy()
    Q8, scale, bias = (t.cpu().numpy() for t in idx.debug_lut(qd, avq.LUT_U8))
    for qi in range(case["q"].shape[0]):
        Lo = oracle.lut_f32(case["q"][qi], case["cb"])
        np.testing.assert_array_equal(L[qi], Lo)
        Qo, so, bo = oracle.lut_u8(Lo)
        np.testing.assert_array_equal(Q8[qi], Qo)
        assert scale[qi] == so and bias[qi] == bo


@pytest.mark.parametrize("nq", [1, 7, 32, 33])
def test_lut_tables_match_for_few_queries_and_for_batches(case, nq):
    # up to 32 queries take the table kernel made for latency, more the one made for throughput; queries with
    # repeated and zero components make equal table entries (the first minimum and maximum in index order count)
    idx, _ = make_index(case)
    rng = np.random.default_rng(77)
    q = np.resize(case["q"], (nq, case["q"].shape[1])).copy()
    q[0] = 0.0
    if nq > 1:
        q[1] = np.where(rng.random(q.shape[1]) < 0.5, 0.0, -0.0).astype(np.float32)
    if nq > 2:
        q[2] = np.round(q[2] * 2.0) / 2.0
    qd = dev(q)
    L = idx.debug_lut(qd, avq.LUT_F32).cpu().numpy()
    Q8, scale, bias = (t.cpu().numpy() for t in idx.debug_lut(qd, avq.LUT_U8))
    for qi in range(nq):
        Lo = oracle.lut_f32(q[qi], case["cb"])
        np.testing.assert_array_equal(L[qi].view(np.uint32), Lo.view(np.uint32))
        Qo, so, bo = oracle.lut_u8(Lo)
        np.testing.assert_array_equal(Q8[qi], Qo)
        assert np.float32(scale[qi]).view(np.uint32) == np.float32(so).view(np.uint32)
        assert np.float32(bias[qi]).view(np.uint32) == np.float32(bo).view(np.uint32)


@pytest.mark.parametrize("nq", [1, 3, None])
def test_adc_scores_match(case, nq):
    # nq = 1, 3: one query per workgroup; None: the full batch (query-tiled kernels)
    idx, _ = make_index(case)
    q = case["q"] if nq is None else case["q"][:nq]
    qd = dev(q)
    sf = idx.debug_adc_scores(qd, avq.LUT_F32).cpu().numpy()
    su = idx.debug_adc_scores(qd, avq.LUT_U8).cpu().numpy()
    for qi in range(q.shape[0]):
        kf, _, _ = oracle.adc_keys_flat(q[qi], case["cb"], case["codes"], case["bits"], 0)
        np.testing.assert_allclose(sf[qi], kf, rtol=1e-5, atol=1e-6)     # the stated tolerance
        np.testing.assert_array_equal(sf[qi], kf)                         # same operation order
        ku, _, _ = oracle.adc_keys_flat(q[qi], case["cb"], case["codes"], case["bits"], 1)
        np.testing.assert_array_equal(su[qi], ku.astype(np.int32))


@pytest.mark.parametrize("lut_mode", [0, 1])
@pytest.mark.parametrize("k,R", [(10, 0), (10, 100), (1, 1), (64, 128)])
def test_search_matches(case, lut_mode, k, R):
    idx, xd = make_index(case)
    qd = dev(case["q"])
    ids, sc = idx.search(qd, k, R, lut_mode)
    oi, os_ = oracle.search(case["x"], case["cb"], case["codes"], case["bits"], case["q"], k, R, lut_mode)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_allclose(sc.cpu().numpy(), os_, rtol=1e-5, atol=1e-6)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)
    # single-query calls take the one-query-per-workgroup path
    ids1, sc1 = idx.search(qd[:1].contiguous(), k, R, lut_mode)
    np.testing.assert_array_equal(ids1.cpu().numpy(), oi[:1])
    np.testing.assert_array_equal(sc1.cpu().numpy(), os_[:1])


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_search_is_deterministic_and_independent_of_launch_shape(case, lut_mode):
    idx, xd = make_index(case)
    qd = dev(case["q"])
    base = [t.cpu().numpy() for t in idx.search(qd, 10, 100, lut_mode)]
    again = [t.cpu().numpy() for t in idx.search(qd, 10, 100, lut_mode)]
    np.testing.assert_array_equal(base[0], again[0])
    np.testing.assert_array_equal(base[1], again[1])
    tiles = (1, 4, 8) if (lut_mode == 1 or case["bits"] == 4) else (1, 4)
    for name, val in (("scan_target_wgs", 64), ("scan_target_wgs", 4096), ("scan_waves", 2),
                      ("small_batch_max", 1), ("small_batch_max", 1000), ("scan_mfma", 1), ("scan_prefilter", 1),
                      ("scan_prefilter", 2), ("prefilter_cap", 128), ("prefilter_cap", 300), ("scan_sample", 1), ("scan_sample", 2)) + tuple(("scan_qt", t) for t in tiles):
        idx.set_tuning(name, val)
        got = [t.cpu().numpy() for t in idx.search(qd, 10, 100, lut_mode)]
        np.testing.assert_array_equal(base[0], got[0])
        np.testing.assert_array_equal(base[1], got[1])
        idx.set_tuning(name, 0)


@pytest.mark.parametrize("prefilter", [0, 1, 2])
def test_fp32_batches_with_flat_score_distributions(prefilter):
    # Batches with fp32 tables take their candidates from the 8-bit-table scan and must notice
    # when those cannot be proven complete: here 1,200 of 4,000 points are copies of three
    # vectors, so for queries near one of them hundreds of points share the best integer sum
    # (and the best fp32 score: ties go to the lower id), while other queries see ordinary data.
    rng = np.random.default_rng(51)
    n, d, M, bits, nq = 4000, 32, 16, 4, 48
    x = unit_rows(rng, n, d)
    protos = unit_rows(rng, 3, d)
    dup = rng.permutation(n)[:1200]
    x[dup] = protos[rng.integers(0, 3, 1200)]
    q = unit_rows(rng, nq, d)
    q[:24] = protos[rng.integers(0, 3, 24)] + 0.05 * rng.standard_normal((24, d)).astype(np.float32)
    cb = oracle.train_pq(x, M, 16, 4, seed=3)
    codes = oracle.encode(x, cb, T=0.2, passes=3)
    idx = avq.Index(d, M, bits, T=0.2)
    idx.set_codebooks(cb)
    idx.set_database(dev(x), oracle.pack_codes(codes, bits))
    idx.set_tuning("small_batch_max", 1)     # the batch kernels, not the block-maxima path of small batches
    idx.set_tuning("scan_prefilter", prefilter)
    for k, R in ((10, 100), (5, 0), (20, 128)):
        oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, 0)
        ids, sc = idx.search(dev(q), k, R, avq.LUT_F32)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)
    # the same data with 8-bit tables, where equal sums are the rule: matrix-core scan (prefilter
    # 0 and 2) and the LDS-table scan (1); equal scores inside one block of 256 points must
    # still come out by id
    idx.set_tuning("scan_mfma", 1 if prefilter == 1 else 0)
    for k, R in ((10, 100), (5, 0)):
        oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, 1)
        ids, sc = idx.search(dev(q), k, R, avq.LUT_U8)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.mark.parametrize("variant", ["default", "lists", "sample_lists", "odd_fail", "small_buffers"])
def test_fp32_batches_scan_against_sampled_bounds(variant):
    # Large chunks (here forced by asking for few waves) make the candidate scan of fp32-table
    # batches guess its bounds from a sample of the blocks and check the guess afterwards. 6,000
    # copies of one vector sit in the first blocks only: for queries near it the sample, which
    # takes blocks at equal distances, says little about the best scores, and the check must
    # notice where the guess was too high. Results must equal the oracle's in every variant.
    rng = np.random.default_rng(61)
    n, d, M, bits, nq = 300_000, 32, 16, 4, 64
    x = unit_rows(rng, n, d)
    proto = unit_rows(rng, 1, d)
    x[rng.permutation(12_000)[:6000]] = proto[0]
    q = unit_rows(rng, nq, d)
    q[:8] = proto[0] + 0.1 * rng.standard_normal((8, d)).astype(np.float32)
    idx = avq.Index(d, M, bits, T=0.2, kmeans_iters=4, encode_passes=2, seed=5)
    xd = dev(x)
    idx.train(xd[:20_000])
    idx.encode(xd)
    cb = idx.get_codebooks()
    codes = unpack_codes(idx.get_codes(), M, bits)
    idx.set_tuning("scan_target_wgs", 4)
    idx.set_tuning("small_batch_max", 1)     # the batch kernels, not the block-maxima path of small batches
    if variant == "lists":
        idx.set_tuning("scan_sample", 1)
    elif variant == "sample_lists":
        idx.set_tuning("scan_sample", 2)
    elif variant == "odd_fail":
        idx.set_tuning("scan_prefilter", 2)
    elif variant == "small_buffers":
        idx.set_tuning("prefilter_cap", 200)
    for k, R in ((10, 100), (5, 0), (10, 500)):
        oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, 0)
        ids, sc = idx.search(dev(q), k, R, avq.LUT_F32)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)
        unverified = idx.debug_unverified_queries()
        assert 0 <= unverified <= nq
        if variant == "odd_fail":
            assert unverified >= nq // 2
        if variant == "default" and R == 100:
            assert unverified < nq // 2          # the guess holds for ordinary queries
    # the 8-bit-table search goes the same way (kept keys ranked by their integer sums; the 6,000 copies
    # tie, far more of them than a list holds, and must come out by id)
    for k, R in ((10, 100), (5, 0)):
        oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, 1)
        ids, sc = idx.search(dev(q), k, R, avq.LUT_U8)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.mark.parametrize("nq", [16, 100, 700])
def test_mid_size_batches_sample_short_chunks(nq):
    # Few queries mean many short chunks (here 5 to 37 blocks each, default launch shape): the candidate scan
    # still takes its bounds from a sample (two or more blocks of every chunk); with lists every query would
    # keep more points than the refinement holds and be scanned again. Results equal the oracle's, and
    # ordinary queries are not handed back.
    rng = np.random.default_rng(77 + nq)
    n, d, M, bits = 300_000, 100, 50, 4
    x = unit_rows(rng, n, d)
    q = unit_rows(rng, nq, d)
    idx = avq.Index(d, M, bits, T=0.2, kmeans_iters=3, encode_passes=1, seed=9)
    xd = dev(x)
    idx.train(xd[:20_000])
    idx.encode(xd)
    cb = idx.get_codebooks()
    codes = unpack_codes(idx.get_codes(), M, bits)
    idx.set_tuning("small_batch_max", 1)     # the batch kernels also for the 16 queries
    qs = q[:min(nq, 48)]   # the oracle's share
    for k, R in ((10, 100), (10, 300)):
        for lut_mode in (avq.LUT_F32, avq.LUT_U8):
            ids, sc = idx.search(dev(q), k, R, lut_mode)
            if lut_mode == avq.LUT_F32:
                assert idx.debug_unverified_queries() <= max(1, nq // 50)
            oi, os_ = oracle.search(x, cb, codes, bits, qs, k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy()[:len(qs)], oi)
            np.testing.assert_array_equal(sc.cpu().numpy()[:len(qs)], os_)


@pytest.mark.parametrize("n,d,M,nq", [(280_001, 100, 50, 40), (300_300, 100, 25, 33), (270_000, 98, 49, 17)])
def test_fp32_batches_sampled_bounds_other_code_sizes(n, d, M, nq):
    # the same two-launch candidate scan for 25, 13 (odd M: a zero table at the end) and a
    # non-specialised number of code bytes (M = 49: the scan with fp32 tables of every point),
    # sizes that are no multiple of a block, batches that are no multiple of a tile
    rng = np.random.default_rng(62)
    x = unit_rows(rng, n, d)
    q = unit_rows(rng, nq, d)
    idx = avq.Index(d, M, 4, T=0.2, kmeans_iters=3, encode_passes=1, seed=6)
    xd = dev(x)
    idx.train(xd[:8_000])
    idx.encode(xd)
    cb = idx.get_codebooks()
    codes = unpack_codes(idx.get_codes(), M, 4)
    idx.set_tuning("scan_target_wgs", 4)
    idx.set_tuning("small_batch_max", 1)     # the batch kernels, not the block-maxima path of small batches
    for k, R in ((10, 100), (1, 0), (10, 257)):
        for lut_mode in (avq.LUT_F32, avq.LUT_U8):
            oi, os_ = oracle.search(x, cb, codes, 4, q, k, R, lut_mode)
            ids, sc = idx.search(dev(q), k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi)
            np.testing.assert_array_equal(sc.cpu().numpy(), os_)
    if M != 49:
        assert idx.debug_unverified_queries() >= 0      # the candidate path ran


def test_equal_scores_inside_a_block_with_8bit_codes():
    # 8-bit codes, both table kinds: duplicates make hundreds of equal scores per block
    rng = np.random.default_rng(52)
    n, d, M, bits, nq = 3000, 16, 4, 8, 24
    x = unit_rows(rng, n, d)
    protos = unit_rows(rng, 2, d)
    dup = rng.permutation(n)[:1500]
    x[dup] = protos[rng.integers(0, 2, 1500)]
    q = unit_rows(rng, nq, d)
    q[:12] = protos[rng.integers(0, 2, 12)] + 0.05 * rng.standard_normal((12, d)).astype(np.float32)
    cb = oracle.train_pq(x, M, 256, 3, seed=3)
    codes = oracle.encode(x, cb, T=0.2, passes=2)
    idx = avq.Index(d, M, bits, T=0.2)
    idx.set_codebooks(cb)
    idx.set_database(dev(x), oracle.pack_codes(codes, bits))
    for lut_mode in (0, 1):
        for k, R in ((10, 100), (5, 0)):
            oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, lut_mode)
            ids, sc = idx.search(dev(q), k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi)
            np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_small_batch_paths_agree_with_oracle(case, lut_mode):
    # a handful of queries: block-maxima scan + fused finish kernel (default), its
    # three-kernel variant, and the batch kernels forced onto the same queries
    idx, xd = make_index(case)
    nq = 5
    q = case["q"][:nq]
    qd = dev(q)
    for k, R in ((10, 100), (10, 0), (100, 512)):
        oi, os_ = oracle.search(case["x"], case["cb"], case["codes"], case["bits"], q, k, R, lut_mode)
        # scan_target_wgs = 2: two workgroups per query, so every wave loops over many blocks
        # select_split: the blocks to score exactly are chosen by several workgroups per query, 5 or 3 blocks each
        # (the slices start at every alignment of the 16-byte loads), as on a large index; rerank_split: the exact
        # scores of the candidates by several workgroups per query, 7 or 64 candidates each (1000: by one)
        for name, val in (("small_batch_impl", 0), ("small_batch_impl", 1), ("small_batch_max", 1),
                          ("scan_target_wgs", 2), ("select_split", 5), ("select_split", 3), ("select_split", 8192),
                          ("rerank_split", 7), ("rerank_split", 64), ("rerank_split", 1000),
                          ("stream_loads", 2)):  # the code stream with nontemporal loads, one block per wave (large arrays)
            idx.set_tuning(name, val)
            ids, sc = idx.search(qd, k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi, err_msg="%s=%d" % (name, val))
            np.testing.assert_array_equal(sc.cpu().numpy(), os_, err_msg="%s=%d" % (name, val))
            idx.set_tuning(name, 0)


def test_brute_force_matches(case):
    idx, xd = make_index(case)
    qd = dev(case["q"])
    for k in (1, 10, 100):
        ids, sc = idx.brute_force(qd, k)
        oi, os_ = oracle.brute_force(case["x"], case["q"], k)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)


def test_large_reorder_512():
    c = make_case(77, 5_000, 32, 16, 4, 12)
    idx, xd = make_index(c)
    qd = dev(c["q"])
    for lut_mode in (0, 1):
        for k, R in ((100, 500), (512, 512), (300, 0)):
            ids, sc = idx.search(qd, k, R, lut_mode)
            oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], 4, c["q"], k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi)
            np.testing.assert_array_equal(sc.cpu().numpy(), os_)


def test_degenerate_inputs():
    # fewer points than one block; k == n; duplicate points and an all-zero query give
    # massive ties that must break by lower id
    rng = np.random.default_rng(5)
    n, d, M, bits = 50, 16, 8, 4
    x = unit_rows(rng, n, d)
    x[10:20] = x[3]                      # duplicates
    cb = oracle.train_pq(x, M, 16, 3, seed=1)
    codes = oracle.encode(x, cb, T=0.2)
    q = unit_rows(rng, 4, d)
    q[1] = 0.0                           # every score equal
    idx = avq.Index(d, M, bits)
    idx.set_codebooks(cb)
    xd = dev(x)
    idx.set_database(xd, oracle.pack_codes(codes, bits))
    qd = dev(q)
    for lut_mode in (0, 1):
        for k, R in ((50, 50), (10, 0), (7, 20), (50, 0)):
            ids, sc = idx.search(qd, k, R, lut_mode)
            oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi)
            np.testing.assert_array_equal(sc.cpu().numpy(), os_)
    # one point
    idx1 = avq.Index(d, M, bits)
    idx1.set_codebooks(cb)
    x1 = dev(x[:1])
    idx1.set_database(x1, oracle.pack_codes(codes[:1], bits))
    ids, sc = idx1.search(qd, 1, 1, 0)
    assert ids.cpu().numpy().tolist() == [[0]] * 4


def test_error_paths():
    rng = np.random.default_rng(6)
    idx = avq.Index(16, 8, 4)
    q = dev(unit_rows(rng, 2, 16))
    with pytest.raises(avq.AvqError) as e:
        idx.search(q, 1, 0)
    assert e.value.code == avq.AVQ_ESTATE
    x = unit_rows(rng, 300, 16)
    with pytest.raises(avq.AvqError) as e:
        idx.encode(dev(x))
    assert e.value.code == avq.AVQ_ESTATE           # no dictionaries yet
    idx.train(dev(x))
    idx.encode(dev(x))
    for k, R in ((0, 0), (10, 5), (513, 0), (10, 600), (301, 0)):
        with pytest.raises(avq.AvqError) as e:
            idx.search(q, k, R)
        assert e.value.code == avq.AVQ_EINVAL
    with pytest.raises(avq.AvqError):
        idx.search(q, 1, 0, lut_mode=2)
    with pytest.raises(avq.AvqError):
        idx.train(dev(x[:8]))                        # fewer rows than codewords


# ---- training and encoding ---------------------------------------------------------

@pytest.mark.parametrize("name", ["tiny_nb8", "glove_nb25", "large8_nb32", "odd_m_nb4", "bits100_nb13", "bits8_nb3"])
def test_encode_matches(name):
    n, d, M, bits, nq = CASES[name]
    n = min(n, 3000)
    c = make_case(11, n, d, M, bits, 2)
    idx = avq.Index(d, M, bits, T=0.2, encode_passes=3)
    idx.set_codebooks(c["cb"])
    idx.encode(dev(c["x"]))
    got = unpack_codes(idx.get_codes(), M, bits)
    want = c["codes"]
    mism = np.any(got != want, axis=1)
    # fp64 on both sides: codes differ only at (near-)exact ties of the loss
    assert mism.mean() <= 1e-3
    if mism.any():
        eta = oracle.eta_limit(d, 0.2)
        xt_g = oracle.reconstruct(got[mism], c["cb"])
        xt_w = oracle.reconstruct(want[mism], c["cb"])
        for xi, a, b in zip(c["x"][mism], xt_g, xt_w):
            assert oracle.aniso_loss(xi, a, eta) == pytest.approx(oracle.aniso_loss(xi, b, eta), rel=1e-9)


def test_encode_eta_modes_and_norms():
    # varying norms: eta is taken per point; explicit eta = 1 is plain nearest codeword
    rng = np.random.default_rng(12)
    n, d, M, bits = 1500, 32, 16, 4
    x = unit_rows(rng, n, d) * np.exp(0.25 * rng.standard_normal((n, 1))).astype(np.float32)
    cb = oracle.train_pq(x, M, 16, 4, seed=2)
    for mode, kw in ((avq.ETA_LIMIT, {}), (avq.ETA_EXPLICIT, dict(eta_explicit=1.0)),
                     (avq.ETA_EXPLICIT, dict(eta_explicit=6.5)), (avq.ETA_EXACT, {})):
        idx = avq.Index(d, M, bits, T=0.2, eta_mode=mode, encode_passes=4, **kw)
        idx.set_codebooks(cb)
        nn = 200 if mode == avq.ETA_EXACT else n
        idx.encode(dev(x[:nn]))
        got = unpack_codes(idx.get_codes(), M, bits)
        want = oracle.encode(x[:nn], cb, T=0.2, eta_mode=mode, eta_explicit=kw.get("eta_explicit", 1.0), passes=4)
        assert np.mean(np.any(got != want, axis=1)) <= 2e-3


def test_train_matches():
    rng = np.random.default_rng(13)
    n, d, M, bits = 5000, 32, 16, 4
    x = unit_rows(rng, n, d)
    idx = avq.Index(d, M, bits, kmeans_iters=6, seed=9)
    idx.train(dev(x))
    got = idx.get_codebooks()
    want = oracle.train_pq(x, M, 16, 6, seed=9)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-6)
    # 8-bit dictionaries, wider subspaces
    idx = avq.Index(32, 4, 8, kmeans_iters=3, seed=3)
    idx.train(dev(x))
    np.testing.assert_allclose(idx.get_codebooks(), oracle.train_pq(x, 4, 256, 3, seed=3), rtol=0, atol=1e-6)


# ---- partitioned index --------------------------------------------------------------

def make_ivf_case(seed, n, d, M, bits, nq, n_leaves):
    rng = np.random.default_rng(seed)
    cfg = dict(si.CONFIGS["glove"])
    centers_mix = si.mixture_centers(40, d, seed)
    x = si.mixture(n, d, 40, 0.3, seed, centers=centers_mix)
    q = si.mixture(nq, d, 40, 0.3, seed, stream=si.STREAM_QUERIES, centers=centers_mix)
    centers = oracle.kmeans(x[:4000], n_leaves, iters=4, seed=seed)
    assign = oracle.assign_nearest(x, centers)
    cb = oracle.train_pq(x[:4000], M, 1 << bits, 4, seed, leaf_centers=centers, leaf_assign=assign[:4000])
    codes = oracle.encode(x, cb, T=0.2, passes=3, leaf_centers=centers, leaf_assign=assign)
    return dict(x=x, q=q, cb=cb, codes=codes, centers=centers, assign=assign, d=d, M=M, bits=bits,
                n_leaves=n_leaves)


@pytest.fixture(scope="module")
def ivf_case():
    return make_ivf_case(31, 9_001, 100, 50, 4, 33, 37)


def make_ivf_index(c):
    idx = avq.Index(c["d"], c["M"], c["bits"], n_leaves=c["n_leaves"])
    idx.set_codebooks(c["cb"])
    idx.set_leaf_centers(c["centers"])
    xd = dev(c["x"])
    idx.set_database(xd, oracle.pack_codes(c["codes"], c["bits"]), c["assign"])
    return idx, xd


def test_leaf_select_matches(ivf_case):
    c = ivf_case
    idx, _ = make_ivf_index(c)
    qd = dev(c["q"])
    for L in (1, 5, 37):
        ids, ip = idx.debug_leaf_select(qd, L)
        for qi in range(c["q"].shape[0]):
            oi, oip = oracle.leaf_select(c["centers"], c["q"][qi], L)
            np.testing.assert_array_equal(ids[qi].cpu().numpy(), oi)
            np.testing.assert_array_equal(ip[qi].cpu().numpy(), oip)


@pytest.mark.parametrize("lut_mode", [0, 1])
@pytest.mark.parametrize("k,R,L", [(10, 100, 5), (10, 0, 5), (20, 60, 37), (10, 100, 1)])
def test_partitioned_search_matches(ivf_case, lut_mode, k, R, L):
    c = ivf_case
    idx, xd = make_ivf_index(c)
    qd = dev(c["q"])
    ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
    oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], c["q"], k, R, lut_mode,
                            centers=c["centers"], assign=c["assign"], leaves_to_search=L)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.mark.parametrize("lut_mode", [0, 1])
@pytest.mark.parametrize("nq", [1, 3, 16, 17])
def test_partitioned_search_of_a_few_queries_matches(ivf_case, lut_mode, nq):
    # up to 16 queries: exact block maxima over the blocks of the probed leaves, the R best blocks scored again
    # (17: the scan with one workgroup per query); probing every leaf, one leaf, and fewer blocks than R
    c = ivf_case
    idx, xd = make_ivf_index(c)
    q = c["q"][:nq]
    qd = dev(q)
    for k, R, L in ((10, 100, 5), (10, 0, 5), (20, 60, 37), (10, 100, 1), (64, 512, 3), (1, 1, 37)):
        ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
        oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], q, k, R, lut_mode,
                                centers=c["centers"], assign=c["assign"], leaves_to_search=L)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi, err_msg="k=%d R=%d L=%d" % (k, R, L))
        np.testing.assert_array_equal(sc.cpu().numpy(), os_, err_msg="k=%d R=%d L=%d" % (k, R, L))
    idx.set_tuning("small_batch_impl", 1)   # the same through the scan with one workgroup per query
    ids, sc = idx.search(qd, 10, 100, lut_mode, leaves_to_search=5)
    oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], q, 10, 100, lut_mode,
                            centers=c["centers"], assign=c["assign"], leaves_to_search=5)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.fixture(scope="module")
def ivf_batch_case():
    # enough queries and probed leaves for the search that regroups the (query, leaf) pairs by leaf
    return make_ivf_case(33, 40_007, 32, 16, 4, 130, 150)


def test_leaf_select_for_batches_matches(ivf_batch_case):
    # a batch, every fifth query checked
    c = ivf_batch_case
    idx, _ = make_ivf_index(c)
    qd = dev(c["q"])
    for L in (1, 16, 100, 150):
        ids, ip = idx.debug_leaf_select(qd, L)
        ids, ip = ids.cpu().numpy(), ip.cpu().numpy()
        for qi in range(0, c["q"].shape[0], 7):
            oi, oip = oracle.leaf_select(c["centers"], c["q"][qi], L)
            np.testing.assert_array_equal(ids[qi], oi)
            np.testing.assert_array_equal(ip[qi], oip)


@pytest.mark.parametrize("which", ["d100", "d32"])
def test_leaf_select_for_thousands_of_queries_matches(ivf_case, ivf_batch_case, which):
    # from 768 queries on a workgroup scores the leaves for eight queries at once; the last workgroup here
    # holds two queries. d = 100 leaves a tail after the chunks of eight dimensions
    c = ivf_case if which == "d100" else ivf_batch_case
    idx, _ = make_ivf_index(c)
    rng = np.random.default_rng(5)
    nq = 2050
    q = c["q"][rng.integers(0, c["q"].shape[0], nq)] + rng.normal(0.0, 0.05, (nq, c["d"])).astype(np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    qd = dev(q)
    for L in (1, 16, min(100, c["n_leaves"]), c["n_leaves"]):
        ids, ip = idx.debug_leaf_select(qd, L)
        ids, ip = ids.cpu().numpy(), ip.cpu().numpy()
        for qi in list(range(0, nq, 97)) + [2047, 2048, 2049]:
            oi, oip = oracle.leaf_select(c["centers"], q[qi], L)
            np.testing.assert_array_equal(ids[qi], oi, err_msg="L=%d query %d" % (L, qi))
            np.testing.assert_array_equal(ip[qi], oip, err_msg="L=%d query %d" % (L, qi))


@pytest.mark.parametrize("lut_mode", [0, 1])
@pytest.mark.parametrize("variant", ["default", "plain", "odd_back", "small_buffers"])
def test_partitioned_batches_grouped_by_leaf(ivf_batch_case, lut_mode, variant):
    # batches of 64 queries or more probing 16 leaves or more (large ones by default, any when asked): leaves scanned on the matrix cores, 32
    # queries at a time, kept points scored per query; "plain": the one-query-per-workgroup scan;
    # "odd_back" / "small_buffers": every other query, or most of them, handed back to that scan
    c = ivf_batch_case
    idx, xd = make_ivf_index(c)
    idx.set_tuning("group_min_pairs", 1)   # regroup whatever the batch size (built in: from 100,000 pairs)
    if variant == "plain":
        idx.set_tuning("scan_prefilter", 1)
    elif variant == "odd_back":
        idx.set_tuning("scan_prefilter", 2)
    elif variant == "small_buffers":
        idx.set_tuning("prefilter_cap", 128)
    qd = dev(c["q"])
    for k, R, L in ((10, 100, 40), (10, 0, 16), (5, 300, 150), (100, 0, 25)):
        ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
        oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], c["q"], k, R, lut_mode,
                                centers=c["centers"], assign=c["assign"], leaves_to_search=L)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi, err_msg="k=%d R=%d L=%d" % (k, R, L))
        np.testing.assert_array_equal(sc.cpu().numpy(), os_, err_msg="k=%d R=%d L=%d" % (k, R, L))
    if variant == "odd_back":
        assert idx.debug_unverified_queries() >= 65


@pytest.fixture(scope="module", params=[(100, 25), (128, 64)], ids=["nb13", "nb32"])
def ivf_other_size_case(request):
    d, M = request.param
    return make_ivf_case(35, 12_345, d, M, 4, 140, 40)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_partitioned_search_at_other_code_sizes(ivf_other_size_case, lut_mode):
    # 13 and 32 code bytes per point (the cases above hold 25 and 8): a few queries (block maxima of the probed
    # leaves), the one-query-per-workgroup scan, and a batch regrouped by leaf
    c = ivf_other_size_case
    idx, xd = make_ivf_index(c)
    idx.set_tuning("group_min_pairs", 1)
    for nq in (2, 40, 140):
        q = c["q"][:nq]
        qd = dev(q)
        for k, R, L in ((10, 100, 16), (10, 0, 40), (30, 300, 7)):
            ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
            oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], q, k, R, lut_mode,
                                    centers=c["centers"], assign=c["assign"], leaves_to_search=L)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi, err_msg="nq=%d k=%d R=%d L=%d" % (nq, k, R, L))
            np.testing.assert_array_equal(sc.cpu().numpy(), os_, err_msg="nq=%d k=%d R=%d L=%d" % (nq, k, R, L))
    idx.set_tuning("small_batch_impl", 1)
    q = c["q"][:2]
    ids, sc = idx.search(dev(q), 10, 100, lut_mode, leaves_to_search=16)
    oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], q, 10, 100, lut_mode,
                            centers=c["centers"], assign=c["assign"], leaves_to_search=16)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.fixture(scope="module", params=[(64, 8), (24, 6)], ids=["nb8", "nb6"])
def ivf_wide_code_case(request):
    d, M = request.param
    return make_ivf_case(36, 6_007, d, M, 8, 70, 24)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_partitioned_search_with_8bit_codes(ivf_wide_code_case, lut_mode):
    # 256 codewords per subspace on a partitioned index: a few queries and a batch
    c = ivf_wide_code_case
    idx, xd = make_ivf_index(c)
    idx.set_tuning("group_min_pairs", 1)
    for nq in (1, 5, 70):
        q = c["q"][:nq]
        qd = dev(q)
        for k, R, L in ((10, 100, 6), (10, 0, 24), (25, 200, 16)):
            ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
            oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], c["bits"], q, k, R, lut_mode,
                                    centers=c["centers"], assign=c["assign"], leaves_to_search=L)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi, err_msg="nq=%d k=%d R=%d L=%d" % (nq, k, R, L))
            np.testing.assert_array_equal(sc.cpu().numpy(), os_, err_msg="nq=%d k=%d R=%d L=%d" % (nq, k, R, L))


@pytest.mark.parametrize("d,M", [(16, 8), (32, 16)])
@pytest.mark.parametrize("lut_mode", [0, 1])
def test_partitioned_search_pads_when_leaves_are_small(d, M, lut_mode):
    # more results asked for than the probed leaves hold: padded with id -1, score -inf (4 code bytes per point: the
    # scan with lists; 8: the block maxima of the probed leaves, with empty leaves among the 40)
    c = make_ivf_case(32, 400, d, M, 4, 7, 40)
    idx, xd = make_ivf_index(c)
    qd = dev(c["q"])
    for k, R, L in ((60, 100, 2), (5, 0, 1), (60, 60, 3)):
        ids, sc = idx.search(qd, k, R, lut_mode, leaves_to_search=L)
        oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], 4, c["q"], k, R, lut_mode, centers=c["centers"],
                                assign=c["assign"], leaves_to_search=L)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)
        if k == 60 and L == 2:
            assert (oi == -1).any()


def test_partitioned_train_and_encode(ivf_case):
    c = ivf_case
    x = c["x"]
    idx = avq.Index(c["d"], c["M"], c["bits"], n_leaves=12, kmeans_iters=4, leaf_kmeans_iters=4,
                    encode_passes=3, seed=4)
    xd = dev(x)
    idx.train(dev(x[:3000]))
    centers = oracle.kmeans(x[:3000], 12, iters=4, seed=4)
    np.testing.assert_allclose(idx.get_leaf_centers(), centers, rtol=0, atol=1e-6)
    # from here on use the library's own centers so later stages are compared like for like
    centers = idx.get_leaf_centers()
    assign_t = oracle.assign_nearest(x[:3000], centers)
    cb = oracle.train_pq(x[:3000], c["M"], 16, 4, 4, leaf_centers=centers, leaf_assign=assign_t)
    np.testing.assert_allclose(idx.get_codebooks(), cb, rtol=0, atol=1e-6)
    cb = idx.get_codebooks()
    idx.encode(xd)
    assign = oracle.assign_nearest(x, centers)
    got_assign = idx.get_leaf_assign()
    assert np.mean(got_assign != assign) <= 1e-3
    codes = oracle.encode(x, cb, T=0.2, passes=3, leaf_centers=centers, leaf_assign=got_assign)
    got = unpack_codes(idx.get_codes(), c["M"], c["bits"])
    assert np.mean(np.any(got != codes, axis=1)) <= 1e-3
    # and the index built by the library searches like the oracle on the library's own codes
    qd = dev(c["q"])
    ids, sc = idx.search(qd, 10, 100, 0, leaves_to_search=4)
    oi, os_ = oracle.search(x, cb, got, c["bits"], c["q"], 10, 100, 0, centers=centers,
                            assign=got_assign, leaves_to_search=4)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)


@pytest.mark.parametrize("n,d,M,bits", [(4000, 8, 4, 4), (3000, 100, 50, 4), (1200, 8, 2, 8)])
def test_update_codebooks_matches(n, d, M, bits):
    # Section 4.2's codeword update for all dictionaries at once (Appendix 7.5): the library solves
    # the normal equations by conjugate gradients without forming them, the oracle forms and
    # factorises them. Both in fp64, results rounded to fp32; the iteration stops at a relative
    # residual of 1e-12, far below fp32 resolution.
    rng = np.random.default_rng(31)
    x = unit_rows(rng, n, d) * np.exp(0.2 * rng.standard_normal((n, 1))).astype(np.float32)
    kc = 1 << bits
    cb = oracle.train_pq(x[:max(kc, min(n, 1500))], M, kc, 3, seed=4)
    cb[0, 5] = 9.0                                             # far from every point: never assigned
    idx = avq.Index(d, M, bits, T=0.2, encode_passes=3)
    idx.set_codebooks(cb)
    xd = dev(x)
    idx.encode(xd)
    codes = unpack_codes(idx.get_codes(), M, bits)
    eta = np.array([oracle.eta_limit(d, 0.2, float(np.linalg.norm(xi.astype(np.float64)))) for xi in x])
    want = oracle.pq_joint_update(x, codes, eta, cb)
    iters, rel = idx.update_codebooks(xd, max_iters=4000, tol=1e-12)
    got = idx.get_codebooks()
    assert rel <= 1e-12 and 0 < iters <= 4000
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=2e-6)
    # codewords that no point uses keep their value bit for bit
    used = np.zeros((M, kc), bool)
    for m in range(M):
        used[m, np.unique(codes[:, m])] = True
    assert not used[0, 5]
    np.testing.assert_array_equal(got[~used], cb[~used])
    # the update does not increase the loss it minimises
    def total(cbx):
        xt = oracle.reconstruct(codes, cbx)
        return sum(oracle.aniso_loss(x[i], xt[i], eta[i]) for i in range(n))
    assert total(got) <= total(cb) * (1 + 1e-9)
    # the codes in the index are untouched and searches use the new dictionaries
    np.testing.assert_array_equal(unpack_codes(idx.get_codes(), M, bits), codes)
    q = unit_rows(rng, 3, d)
    sc = idx.debug_adc_scores(dev(q), avq.LUT_F32).cpu().numpy()
    for i in range(3):
        np.testing.assert_array_equal(sc[i], oracle.adc_f32(oracle.lut_f32(q[i], got), codes, bits))


def test_update_codebooks_reconstruction_loss_is_the_cluster_mean():
    # eta = 1 everywhere: the normal equations are diagonal and the solution is the mean of the
    # sub-vectors assigned to each codeword (the k-means update, Section 4.2 with h_par = h_perp)
    rng = np.random.default_rng(32)
    n, d, M, bits = 2500, 16, 8, 4
    x = unit_rows(rng, n, d)
    cb = oracle.train_pq(x, M, 16, 2, seed=5)
    idx = avq.Index(d, M, bits, eta_mode=avq.ETA_EXPLICIT, eta_explicit=1.0)
    idx.set_codebooks(cb)
    xd = dev(x)
    idx.encode(xd)
    codes = unpack_codes(idx.get_codes(), M, bits)
    iters, rel = idx.update_codebooks(xd, max_iters=50, tol=1e-13)
    got = idx.get_codebooks()
    assert iters <= 2
    for m in range(M):
        for j in range(16):
            sel = codes[:, m] == j
            if sel.any():
                np.testing.assert_allclose(got[m, j], x[sel, 2 * m:2 * m + 2].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)


def test_update_codebooks_single_dictionary_is_the_vq_update():
    # M = 1: the joint system splits into one block per codeword, Theorem 4.2's closed form.
    # 256 codewords of 36 dimensions = 9216 unknowns: more than the per-workgroup accumulator
    # holds, so this also covers the variant that adds into device memory directly.
    rng = np.random.default_rng(34)
    n, d = 3000, 36
    x = unit_rows(rng, n, d) * np.exp(0.2 * rng.standard_normal((n, 1))).astype(np.float32)
    cb = oracle.train_pq(x, 1, 256, 2, seed=6)
    idx = avq.Index(d, 1, 8, T=0.2, encode_passes=2)
    idx.set_codebooks(cb)
    xd = dev(x)
    idx.encode(xd)
    codes = unpack_codes(idx.get_codes(), 1, 8)[:, 0]
    iters, rel = idx.update_codebooks(xd, max_iters=4000, tol=1e-12)
    got = idx.get_codebooks()
    assert rel <= 1e-12
    eta = np.array([oracle.eta_limit(d, 0.2, float(np.linalg.norm(xi.astype(np.float64)))) for xi in x])
    for j in range(256):
        sel = codes == j
        if sel.sum() == 0:
            np.testing.assert_array_equal(got[0, j], cb[0, j])
        else:
            want = oracle.vq_update(x[sel], eta[sel], np.ones(int(sel.sum())))
            np.testing.assert_allclose(got[0, j], want, rtol=2e-5, atol=2e-6)


def test_update_codebooks_alternation_lowers_the_loss_and_rejects_bad_calls():
    rng = np.random.default_rng(33)
    n, d, M, bits = 6000, 32, 16, 4
    x = unit_rows(rng, n, d)
    xd = dev(x)
    idx = avq.Index(d, M, bits, T=0.2, kmeans_iters=4, seed=2)
    idx.train(xd)
    eta = oracle.eta_limit(d, 0.2)
    losses = []
    for it in range(3):
        idx.encode(xd)
        codes = unpack_codes(idx.get_codes(), M, bits)
        xt = oracle.reconstruct(codes, idx.get_codebooks())
        losses.append(sum(oracle.aniso_loss(x[i], xt[i], eta) for i in range(n)))
        idx.update_codebooks(xd)
        xt = oracle.reconstruct(codes, idx.get_codebooks())
        losses.append(sum(oracle.aniso_loss(x[i], xt[i], eta) for i in range(n)))
    assert all(b <= a * (1 + 1e-7) for a, b in zip(losses, losses[1:])), losses
    assert losses[-1] < 0.97 * losses[0], losses
    with pytest.raises(avq.AvqError):
        idx.update_codebooks(xd[:100].contiguous())
    with pytest.raises(avq.AvqError):
        idx.update_codebooks(xd, max_iters=0)
    fresh = avq.Index(d, M, bits)
    fresh.set_codebooks(idx.get_codebooks())
    with pytest.raises(avq.AvqError):
        fresh.update_codebooks(xd)


@pytest.mark.parametrize("n,d,M,bits", [(1000, 16, 16, 4), (2100, 98, 49, 4), (3000, 100, 25, 4), (700, 24, 3, 8)])
def test_stream_codes_reads_every_code_byte_once(n, d, M, bits):
    # the measurement kernel folds a block's words with xor; a word holds the same code byte of
    # four consecutive points, padding points are all zero
    rng = np.random.default_rng(41)
    x = unit_rows(rng, n, d)
    idx = avq.Index(d, M, bits, kmeans_iters=2, encode_passes=1)
    idx.train(dev(x[:max(300, 1 << bits)]))
    idx.encode(dev(x))
    codes = idx.get_codes()
    NB = codes.shape[1]
    n_blocks = (n + 255) // 256
    padded = np.zeros((n_blocks * 256, NB), np.uint8)
    padded[:n] = codes
    by = np.bitwise_xor.reduce(np.bitwise_xor.reduce(padded.reshape(n_blocks, 64, 4, NB), axis=3), axis=1)
    want = by[:, 0].astype(np.uint32) | by[:, 1].astype(np.uint32) << 8 | by[:, 2].astype(np.uint32) << 16 \
        | by[:, 3].astype(np.uint32) << 24
    got = idx.debug_stream_codes().cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(got, want)


def test_anisotropic_encoding_reduces_the_error_of_large_inner_products():
    # The point of the score-aware loss (Section 3, Figure 2b): with the same dictionaries, codes
    # assigned under the anisotropic loss estimate the inner products that matter -- those of a
    # query with its best datapoints -- better than codes assigned by reconstruction error.
    # d = 32, T = 0.5: eta = 31 * 0.25 / 0.75 = 10.3 (Theorem 3.4's limit)
    rng = np.random.default_rng(7)
    n, d, M, nq = 20_000, 32, 16, 128
    x = unit_rows(rng, n, d)
    q = unit_rows(rng, nq, d)
    xd, qd = dev(x), dev(q)
    base = avq.Index(d, M, 4, T=0.5, kmeans_iters=8, seed=3)
    base.train(xd)
    cb = base.get_codebooks()
    errs = {}
    for name, kw in (("l2", dict(eta_mode=avq.ETA_EXPLICIT, eta_explicit=1.0)), ("aniso", dict(eta_mode=avq.ETA_LIMIT))):
        idx = avq.Index(d, M, 4, T=0.5, seed=3, **kw)
        idx.set_codebooks(cb)
        idx.encode(xd)
        gi, gs = idx.brute_force(qd, 1)
        sc = idx.debug_adc_scores(qd, avq.LUT_F32)
        est = sc[torch.arange(nq, device="cuda"), gi[:, 0].long()].cpu().numpy()
        exact = gs[:, 0].cpu().numpy()
        errs[name] = float(np.mean(np.abs(est - exact) / np.abs(exact)))
    assert errs["aniso"] < 0.9 * errs["l2"], errs


@pytest.mark.parametrize("bits,M,d", [(4, 50, 100), (4, 25, 100), (4, 64, 128), (8, 32, 256), (8, 8, 64)])
@pytest.mark.parametrize("lut_mode", [0, 1])
def test_small_batches_through_block_bounds_with_a_heap_of_equal_scores(bits, M, d, lut_mode):
    # A handful of queries at the code sizes whose full scan records block maxima of 8-bit sums (bounds of the
    # scores) instead of scores. 30,000 points share the code word that is best for query 0: more points reach
    # the bound than the candidate buffer of reorder_k = 100 holds (25,600), so that query's candidates are
    # rebuilt from the exact block maxima; ties are ordered by id. The other queries see the heap somewhere
    # in the middle of their ranking. Compared with the oracle and with the scan over exact block maxima.
    rng = np.random.default_rng(1000 + 10 * M + bits + lut_mode)
    n, kc, nq = 41_003, 1 << bits, 5
    x = unit_rows(rng, n, d)
    q = unit_rows(rng, nq, d)
    cb = oracle.train_pq(x[:2000], M, kc, 2, seed=7)
    codes = rng.integers(0, kc, (n, M), dtype=np.uint8)
    best = np.argmax(oracle.lut_f32(q[0], cb), axis=1).astype(np.uint8)
    codes[5_000:35_000] = best
    case = dict(x=x, q=q, cb=cb, codes=codes, n=n, d=d, M=M, bits=bits, kc=kc)
    idx, xd = make_index(case)
    qd = dev(q)
    for k, R in ((10, 100), (100, 0), (7, 7)):
        oi, os_ = oracle.search(x, cb, codes, bits, q, k, R, lut_mode)
        if R == 0:
            assert list(oi[0]) == list(range(5_000, 5_000 + k))
        for impl, split in ((0, 0), (2, 0), (0, 41)):   # 41: the blocks are selected by four workgroups per query
            idx.set_tuning("small_batch_impl", impl)
            idx.set_tuning("small_batch_max", 1000)
            idx.set_tuning("select_split", split)
            ids, sc = idx.search(qd, k, R, lut_mode)
            np.testing.assert_array_equal(ids.cpu().numpy(), oi)
            np.testing.assert_array_equal(sc.cpu().numpy(), os_)
            ids1, sc1 = idx.search(qd[:1].contiguous(), k, R, lut_mode)
            np.testing.assert_array_equal(ids1.cpu().numpy(), oi[:1])
            np.testing.assert_array_equal(sc1.cpu().numpy(), os_[:1])
        idx.set_tuning("small_batch_impl", 0)
        idx.set_tuning("select_split", 0)


def test_small_batch_block_bounds_degenerate_tables():
    # all dictionaries zero: every table entry, every 8-bit sum and every score is 0; every block is listed and
    # every point reaches the bound. The answer is the lowest ids.
    n, d, M = 30_001, 32, 16
    idx = avq.Index(d, M, 4, T=0.2)
    idx.set_codebooks(np.zeros((M, 16, d // M), np.float32))
    rng = np.random.default_rng(3)
    idx.set_database(None, rng.integers(0, 256, (n, M // 2), dtype=np.uint8))
    qd = dev(unit_rows(rng, 2, d))
    for lut_mode in (0, 1):
        ids, sc = idx.search(qd, 20, 0, lut_mode)
        np.testing.assert_array_equal(ids.cpu().numpy(), np.tile(np.arange(20, dtype=np.int32), (2, 1)))
        assert np.all(sc.cpu().numpy() == 0.0)


def test_quality_metrics_and_T_sweep_equal_the_oracles():
    # Section 5.1 / 5.2 on a 20,000-point slice of the Glove-shaped data: one dictionary learned under the l2
    # loss, the datapoints re-assigned under the anisotropic loss for T in {0, 0.1, 0.2, 0.3, 0.5} (T = 0: eta = 1,
    # the reconstruction loss). Recall 1@N hit counts and the relative error of the top-1 estimate from the
    # library (paper_1908_10396_amd.quality) against the oracle's, computed from the oracle's own encoding
    # under the same dictionary.
    from paper_1908_10396_amd import quality
    cfg = si.CONFIGS["glove"]
    n, nq, d, M, bits = 20_000, 64, cfg["d"], cfg["M"], cfg["bits"]
    x = si.make_data(cfg, n)
    q = si.make_queries(cfg, nq)
    xd, qd = dev(x), dev(q)
    base = avq.Index(d, M, bits, T=0.2, kmeans_iters=10, seed=5)
    base.train(xd)
    cb = base.get_codebooks()
    Ts = [0.0, 0.1, 0.2, 0.3, 0.5]
    got = quality.sweep_T(xd, qd, d, M, bits, cb, Ts, seed=5)
    top1_err = {}
    for T in Ts:
        codes = oracle.encode(x, cb, T=T, passes=10)
        hits, rel = oracle.quality_metrics(x, q, cb, codes, bits, top_n=quality.TOP_N)
        ghits, grel = got[T]
        assert ghits == hits, (T, ghits, hits)
        np.testing.assert_allclose(grel, rel, rtol=1e-6, atol=1e-9)
        top1_err[T] = rel.mean()
    # the direction Figure 2b shows: the estimate of the top inner product improves as T grows from 0
    assert top1_err[0.2] < top1_err[0.0] and top1_err[0.5] < top1_err[0.0], top1_err


@pytest.mark.parametrize("bits,M,d", [(4, 8, 16), (8, 3, 12)])
def test_update_codebooks_on_a_partitioned_index_matches(bits, M, d):
    # Appendix 7.5 with leaf centers: x~ = center + PQ(residual), the loss against x itself (Theorem 4.2's
    # weights come from x, the right-hand side from the residual)
    rng = np.random.default_rng(41 + bits)
    n, L, kc = 3000, 6, 1 << bits
    x = unit_rows(rng, n, d) * np.exp(0.2 * rng.standard_normal((n, 1))).astype(np.float32)
    xd = dev(x)
    idx = avq.Index(d, M, bits, T=0.3, n_leaves=L, kmeans_iters=3, leaf_kmeans_iters=3, encode_passes=3, seed=9)
    idx.train(xd)
    idx.encode(xd)
    cb, centers, assign = idx.get_codebooks(), idx.get_leaf_centers(), idx.get_leaf_assign()
    codes = unpack_codes(idx.get_codes(), M, bits)
    eta = np.array([oracle.eta_limit(d, 0.3, float(np.linalg.norm(xi.astype(np.float64)))) for xi in x])
    want = oracle.pq_joint_update(x, codes, eta, cb, centers, assign)
    iters, rel = idx.update_codebooks(xd, max_iters=4000, tol=1e-12)
    got = idx.get_codebooks()
    assert rel <= 1e-12 and iters > 0
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=2e-6)

    def total(cbx):
        xt = oracle.reconstruct(codes, cbx, centers, assign)
        return sum(oracle.aniso_loss(x[i], xt[i], eta[i]) for i in range(n))
    assert total(got) < total(cb)


def test_anisotropic_leaves_assignment_center_update_and_training():
    # Section 4 with the leaf centers as the codewords of a vector quantizer: assignment to the center of
    # smallest anisotropic loss (Definition 4.1), Theorem 4.2's update of every center, and avq_train's
    # alternation of the two; each piece against the oracle, the whole by the loss it lowers.
    rng = np.random.default_rng(51)
    n, d, M, L, T = 5000, 16, 8, 9, 0.5
    x = unit_rows(rng, n, d) * np.exp(0.15 * rng.standard_normal((n, 1))).astype(np.float32)
    xd = dev(x)
    l2 = avq.Index(d, M, 4, T=T, n_leaves=L, kmeans_iters=2, leaf_kmeans_iters=4, encode_passes=2, seed=3)
    l2.train(xd)
    centers = l2.get_leaf_centers()
    # assignment: an index whose leaves are anisotropic, given the same centers
    an = avq.Index(d, M, 4, T=T, n_leaves=L, kmeans_iters=2, leaf_kmeans_iters=4, encode_passes=2, seed=3,
                   leaf_aniso_iters=2)
    an.set_codebooks(l2.get_codebooks())
    an.set_leaf_centers(centers)
    an.encode(xd)
    got_assign = an.get_leaf_assign()
    want_assign = oracle.assign_aniso(x, centers, T)
    assert np.mean(got_assign != want_assign) <= 1e-3
    assert np.mean(want_assign != oracle.assign_nearest(x, centers)) > 0.01      # the loss changes the partition
    # Theorem 4.2 for every leaf, with that assignment
    iters, rel = an.update_leaf_centers(xd, max_iters=2000, tol=1e-12)
    assert rel <= 1e-12 and iters > 0
    want_centers = oracle.vq_centers_update(x, got_assign, centers, T)
    np.testing.assert_allclose(an.get_leaf_centers(), want_centers, rtol=2e-5, atol=2e-6)
    # training with the alternation lowers the anisotropic loss of the vector quantizer below Lloyd's
    tr = avq.Index(d, M, 4, T=T, n_leaves=L, kmeans_iters=2, leaf_kmeans_iters=4, encode_passes=2, seed=3,
                   leaf_aniso_iters=3)
    tr.train(xd)
    tr.encode(xd)
    eta = np.array([oracle.eta_limit(d, T, float(np.linalg.norm(xi.astype(np.float64)))) for xi in x])

    def vq_loss(c, a):
        return sum(oracle.aniso_loss(x[i], c[a[i]], eta[i]) for i in range(n))
    base = vq_loss(centers, oracle.assign_nearest(x, centers))
    trained = vq_loss(tr.get_leaf_centers(), tr.get_leaf_assign())
    assert trained < 0.995 * base, (trained, base)
    # searches on such an index equal the oracle's (the oracle takes the centers and the assignment as given)
    q = unit_rows(rng, 40, d)
    oi, os_ = oracle.search(x, tr.get_codebooks(), unpack_codes(tr.get_codes(), M, 4), 4, q, 10, 50, 0,
                            centers=tr.get_leaf_centers(), assign=tr.get_leaf_assign(), leaves_to_search=4)
    ids, sc = tr.search(dev(q), 10, 50, 0, leaves_to_search=4)
    np.testing.assert_array_equal(ids.cpu().numpy(), oi)
    np.testing.assert_array_equal(sc.cpu().numpy(), os_)
    with pytest.raises(avq.AvqError):
        avq.Index(d, M, 4).update_leaf_centers(xd)               # flat index


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_partitioned_batch_with_tight_leaves_far_from_the_origin(lut_mode):
    # Leaf centers of norm 50 and residuals of 1e-4: a unit of the 8-bit tables is far below the rounding of a
    # score (<q, center> + table sum), so points tie after rounding and the lower id wins; the scan over leaves
    # regrouped by leaf must keep every point that the rounding can lift to the bound. Against the oracle and
    # the one-query-per-workgroup scan.
    rng = np.random.default_rng(61)
    n, d, M, L, nq, probe = 20_000, 16, 8, 32, 128, 16
    centers = (unit_rows(rng, L, d) * 50.0).astype(np.float32)
    assign = rng.integers(0, L, n).astype(np.int32)
    cb = (rng.standard_normal((M, 16, d // M)) * 1e-4).astype(np.float32)
    codes = rng.integers(0, 16, (n, M), dtype=np.uint8)
    codes[1000:1400] = codes[1000]                   # exact duplicates inside and across blocks
    assign[1000:1400] = assign[1000]
    x = (centers[assign] + oracle.reconstruct(codes, cb).astype(np.float32)).astype(np.float32)
    q = unit_rows(rng, nq, d)
    idx = avq.Index(d, M, 4, T=0.2, n_leaves=L)
    idx.set_codebooks(cb)
    idx.set_leaf_centers(centers)
    xd = dev(x)
    idx.set_database(xd, oracle.pack_codes(codes, 4), assign)
    idx.set_tuning("group_min_pairs", 1)
    for k, R in ((10, 100), (50, 0)):
        oi, os_ = oracle.search(x, cb, codes, 4, q, k, R, lut_mode, centers=centers, assign=assign, leaves_to_search=probe)
        ids, sc = idx.search(dev(q), k, R, lut_mode, leaves_to_search=probe)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)
    assert idx.debug_unverified_queries() < nq      # the regrouped path served queries


@pytest.mark.parametrize("M,d", [(32, 256), (8, 64), (13, 26), (25, 50)])
@pytest.mark.parametrize("lut_mode", [0, 1])
def test_batches_of_8bit_codes_through_block_bounds(M, d, lut_mode):
    # Batches on a flat index of 8-bit codes: the full scan takes the queries sixteen at a time over 6-bit byte
    # tables and records block maxima; the blocks that can reach the R-th best are scored exactly per query.
    # 43 queries (two full tiles and one of 11), a ragged last block, a heap of 30,000 points that share the best
    # code word of query 0 (its candidate list overflows and is rebuilt), the same point planted at both ends.
    rng = np.random.default_rng(2000 + M + lut_mode)
    n, nq = 41_003, 43
    x = unit_rows(rng, n, d)
    q = unit_rows(rng, nq, d)
    cb = oracle.train_pq(x[:2000], M, 256, 2, seed=8)
    codes = rng.integers(0, 256, (n, M), dtype=np.uint8)
    best = np.argmax(oracle.lut_f32(q[0], cb), axis=1).astype(np.uint8)
    codes[5_000:35_000] = best
    codes[0] = codes[n - 1] = np.argmax(oracle.lut_f32(q[1], cb), axis=1).astype(np.uint8)
    case = dict(x=x, q=q, cb=cb, codes=codes, n=n, d=d, M=M, bits=8, kc=256)
    idx, xd = make_index(case)
    qd = dev(q)
    for k, R in ((10, 100), (100, 0), (7, 7)):
        oi, os_ = oracle.search(x, cb, codes, 8, q, k, R, lut_mode)
        if R == 0:
            assert list(oi[0]) == list(range(5_000, 5_000 + k)) and oi[1][0] == 0 and oi[1][1] == n - 1
        ids, sc = idx.search(qd, k, R, lut_mode)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_)
        idx.set_tuning("scan_prefilter", 1)                       # every point scored: the same answer
        ids2, sc2 = idx.search(qd, k, R, lut_mode)
        idx.set_tuning("scan_prefilter", 0)
        np.testing.assert_array_equal(ids2.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc2.cpu().numpy(), os_)
        idx.set_tuning("select_split", 37)                        # blocks chosen by five workgroups per query,
        idx.set_tuning("rerank_split", 16)                        # exact scores by several, sixteen candidates each,
        idx.set_tuning("bound_bits", 6 if k == 10 else 8)         # byte tables of six or eight bits (built in: seven)
        ids3, sc3 = idx.search(qd, k, R, lut_mode)
        idx.set_tuning("select_split", 0)
        idx.set_tuning("rerank_split", 0)
        idx.set_tuning("bound_bits", 0)
        np.testing.assert_array_equal(ids3.cpu().numpy(), oi)
        np.testing.assert_array_equal(sc3.cpu().numpy(), os_)


# ---- drawn configurations -------------------------------------------------------------

def draw_configuration(seed):
    rng = np.random.default_rng(1000 + seed)
    bits = int(rng.choice([4, 4, 8]))
    ds = int(rng.choice([1, 2, 2, 3, 4, 8]))
    M = int(rng.integers(2, 41)) if bits == 4 else int(rng.integers(2, 17))
    if rng.random() < 0.4:  # a code size with kernels of its own
        M = int(rng.choice([16, 25, 26, 50, 64])) if bits == 4 else int(rng.choice([8, 13, 25, 32]))
    while M * ds > 256:
        ds = max(1, ds // 2)
    n = int(np.exp(rng.uniform(np.log(300.0), np.log(40000.0))))
    nq = int(rng.choice([1, 2, 5, 16, 32, 33, 35, 36, 37, 64, 80, 81, 130, 300]))
    R = int(rng.choice([0, 1, 10, 64, 100, 257, 512]))
    k = int(rng.integers(1, max(1, min(R if R else 64, 100)) + 1))
    leaves = int(rng.integers(3, 30)) if rng.random() < 0.5 else 0
    L = int(rng.integers(1, leaves + 1)) if leaves else 0
    return dict(bits=bits, M=M, d=M * ds, n=n, nq=nq, k=k, R=R, n_leaves=leaves, L=L)


@pytest.mark.parametrize("seed", range(int(os.environ.get("AVQ_DRAWN_CONFIGS", "64"))))
def test_drawn_configurations_match(seed):
    # shapes, batch sizes, k, R and partitions drawn at random around the thresholds where the search
    # changes its kernels; both table kinds, ids and scores against the oracle's
    g = draw_configuration(seed)
    msg = str(g)
    if g["n_leaves"]:
        c = make_ivf_case(200 + seed, g["n"], g["d"], g["M"], g["bits"], g["nq"], g["n_leaves"])
        idx, xd = make_ivf_index(c)
        if seed % 2:
            idx.set_tuning("group_min_pairs", 1)
        kw = dict(centers=c["centers"], assign=c["assign"], leaves_to_search=g["L"])
        skw = dict(leaves_to_search=g["L"])
    else:
        c = make_case(200 + seed, g["n"], g["d"], g["M"], g["bits"], g["nq"], train_iters=2)
        idx, xd = make_index(c)
        kw, skw = {}, {}
    # every third configuration with launch shapes that the built-in choices reach on large indexes only
    trng = np.random.default_rng(5000 + seed)
    if seed % 3 == 2:
        for name, val in (("select_split", int(trng.integers(2, 12))), ("rerank_split", int(trng.integers(2, 50))),
                          ("scan_target_wgs", int(trng.integers(1, 9)))):
            if trng.random() < 0.6:
                idx.set_tuning(name, val)
                msg += " %s=%d" % (name, val)
    qd = dev(c["q"])
    for lut_mode in (0, 1):
        ids, sc = idx.search(qd, g["k"], g["R"], lut_mode, **skw)
        oi, os_ = oracle.search(c["x"], c["cb"], c["codes"], g["bits"], c["q"], g["k"], g["R"], lut_mode, **kw)
        np.testing.assert_array_equal(ids.cpu().numpy(), oi, err_msg=msg)
        np.testing.assert_array_equal(sc.cpu().numpy(), os_, err_msg=msg)
