"""Pins for the oracle's query path: tables, ADC, top-k, re-ranking, leaves.

What fixes the right answer here: the ADC score of a point is <q, x~> with x~
the point rebuilt from its codes (Section 4.1); searching with every point
re-ranked is brute-force MIPS (Section 1); top-k is a sort.
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si


def _setup(rng, n, d, M, bits, nq=8):
    kc = 1 << bits
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    cb = (0.3 * rng.standard_normal((M, kc, d // M))).astype(np.float32)
    codes = rng.integers(0, kc, size=(n, M)).astype(np.uint8)
    q = rng.standard_normal((nq, d)).astype(np.float32)
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    return x, cb, codes, q


@pytest.mark.parametrize("M,bits,ds", [(16, 4, 2), (7, 4, 3), (50, 4, 2), (8, 8, 4), (32, 8, 8)])
def test_lut_and_adc_equal_inner_product_with_reconstruction(M, bits, ds):
    rng = np.random.default_rng(M * 10 + bits)
    x, cb, codes, q = _setup(rng, 500, M * ds, M, bits)
    xt = oracle.reconstruct(codes, cb)                      # fp64
    for qi in range(q.shape[0]):
        L = oracle.lut_f32(q[qi], cb)
        # table entry = partial inner product of the query's subspace with the codeword
        want_L = np.einsum("ml,mjl->mj", q[qi].reshape(M, ds).astype(np.float64), cb.astype(np.float64))
        np.testing.assert_allclose(L, want_L, rtol=0, atol=ds * 1e-7)
        s = oracle.adc_f32(L, codes, bits)
        want = xt @ q[qi].astype(np.float64)
        # fp32 summation of M terms: error bounded by M * eps * sum |terms|
        bound = M * 6e-8 * np.abs(want_L).max() * M + 1e-7
        assert np.max(np.abs(s - want)) <= bound
        keys, _, _ = oracle.adc_keys_flat(q[qi], cb, codes, bits, 0)
        np.testing.assert_array_equal(keys, s)


def test_adc_index_mapping_is_not_transposed():
    # a table with one nonzero entry picks out exactly the points carrying that code
    M, kc = 5, 16
    rng = np.random.default_rng(3)
    codes = rng.integers(0, kc, size=(200, M)).astype(np.uint8)
    for m, j in ((0, 3), (1, 0), (4, 15), (3, 7)):
        L = np.zeros((M, kc), np.float32)
        L[m, j] = 2.5
        s = oracle.adc_f32(L, codes, 4)
        np.testing.assert_array_equal(s, np.where(codes[:, m] == j, np.float32(2.5), np.float32(0)))
        Q = np.zeros((M, kc), np.uint8)
        Q[m, j] = 200
        np.testing.assert_array_equal(oracle.adc_u8(Q, codes), np.where(codes[:, m] == j, 200, 0))


@pytest.mark.parametrize("M,bits,ds", [(16, 4, 2), (50, 4, 2), (32, 8, 8)])
def test_u8_lut_properties(M, bits, ds):
    rng = np.random.default_rng(40 + M)
    x, cb, codes, q = _setup(rng, 400, M * ds, M, bits)
    for qi in range(q.shape[0]):
        L = oracle.lut_f32(q[qi], cb)
        Q8, scale, bias = oracle.lut_u8(L)
        width = L.max(1) - L.min(1)
        # every subspace reaches 0 at its minimum; the widest reaches 255
        assert np.all(Q8.min(1) == 0)
        assert Q8[np.argmax(width)].max() == 255
        assert scale == pytest.approx(width.max() / 255, rel=1e-6)
        assert bias == pytest.approx(L.min(1).astype(np.float64).sum(), abs=1e-5)
        # monotone within a subspace
        for m in range(M):
            o = np.argsort(L[m], kind="stable")
            assert np.all(np.diff(Q8[m][o].astype(int)) >= 0)
        # de-quantised score within M * scale / 2 of the fp32 score
        acc = oracle.adc_u8(Q8, codes)
        s = oracle.adc_f32(L, codes, bits)
        err = np.abs(acc.astype(np.float64) * scale + bias - s)
        assert err.max() <= M * scale / 2 + 1e-5
        np.testing.assert_array_equal(acc, Q8[np.arange(M)[None, :], codes].astype(np.uint32).sum(1))
        keys, sc2, b2 = oracle.adc_keys_flat(q[qi], cb, codes, bits, 1)
        np.testing.assert_array_equal(keys, acc.astype(np.float32))
        assert (sc2, b2) == (scale, bias)


@pytest.mark.parametrize("offset,spread", [(0.0, 1.0), (50.0, 1.0), (1000.0, 0.01), (-3.0, 30.0)])
def test_points_outside_the_margin_of_the_integer_sums_cannot_rank_in_fp32(offset, spread):
    # What the library's fp32 batches rely on (4-bit codes): with acc the integer sums over the 8-bit
    # tables and acc_(R) the R-th largest of them, every one of the R best fp32 scores (ties by id)
    # has acc >= acc_(R) - margin, margin = ceil(M + 0.01 + 2.02 rho / scale) + 1,
    # rho = (NB + 2) 2^-24 1.01 sum_m max_j |L[m][j]|: rounding moves each of the M table entries by at
    # most half a unit of scale, and the fp32 sum is within rho of the real one. Tables with a large
    # common offset or a tiny spread make the fp32 rounding term matter.
    rng = np.random.default_rng(77)
    M, bits, n = 50, 4, 6000
    NB = M // 2
    codes = rng.integers(0, 16, (n, M)).astype(np.uint8)
    worst = 0
    for trial in range(6):
        L = (offset + spread * rng.standard_normal((M, 16))).astype(np.float32)
        Q8, scale, bias = oracle.lut_u8(L)
        acc = oracle.adc_u8(Q8, codes).astype(np.int64)
        s = oracle.adc_f32(L, codes, bits)
        rho = (NB + 2) * 2.0 ** -24 * 1.01 * float(np.abs(L).max(1).astype(np.float64).sum())
        margin = int(np.ceil(M + 0.01 + 2.02 * rho / float(scale))) + 1
        by_f32 = np.lexsort((np.arange(n), -s.astype(np.float64)))      # score descending, id ascending
        acc_sorted = np.sort(acc)[::-1]
        for R in (1, 10, 100, 500):
            need = acc_sorted[R - 1] - margin
            assert acc[by_f32[:R]].min() >= need, (trial, R, margin)
            worst = max(worst, int(acc_sorted[R - 1] - acc[by_f32[:R]].min()))
    assert worst > 0   # the two orders do differ: the margin is doing something


def test_u8_lut_rounding_half_even_and_degenerate():
    # one subspace, entries at exact multiples: (L - lo) * 255 / R lands on .5 values
    L = np.array([[0.0, 255.0, 0.5, 1.5, 2.5, 254.5, 100.0, 3.0] + [1.0] * 8], np.float32)
    Q8, scale, bias = oracle.lut_u8(L)
    np.testing.assert_array_equal(Q8[0, :8], [0, 255, 0, 2, 2, 254, 100, 3])
    assert scale == np.float32(1.0) and bias == np.float32(0.0)
    Q8, scale, bias = oracle.lut_u8(np.full((3, 16), 0.25, np.float32))
    assert not Q8.any() and scale == 0.0 and bias == np.float32(0.75)


def test_topk_is_a_sort_with_id_tiebreak():
    rng = np.random.default_rng(9)
    s = rng.integers(0, 20, size=300).astype(np.float32)       # many ties
    s[5] = -0.0
    s[6] = 0.0
    order = np.lexsort((np.arange(300), -s.astype(np.float64)))
    for k in (1, 10, 300):
        ids, sc = oracle.topk(s, k)
        np.testing.assert_array_equal(ids, order[:k])
        np.testing.assert_array_equal(sc, s[order[:k]])
    ids, sc = oracle.topk(s[:4], 6)
    assert list(ids[4:]) == [-1, -1] and np.all(np.isneginf(sc[4:]))
    # explicit ids
    my = rng.permutation(1000)[:300].astype(np.int32)
    ids, _ = oracle.topk(s, 300, ids=my)
    np.testing.assert_array_equal(ids, my[np.lexsort((my, -s.astype(np.float64)))])


def test_exact_scores_and_brute_force():
    rng = np.random.default_rng(10)
    x, _, _, q = _setup(rng, 3000, 100, 50, 4, nq=6)
    for qi in range(q.shape[0]):
        s = oracle.exact_scores(x, q[qi])
        np.testing.assert_allclose(s, x.astype(np.float64) @ q[qi].astype(np.float64), atol=2e-6)
    ids, sc = oracle.brute_force(x, q, 10)
    ref = x.astype(np.float64) @ q.T.astype(np.float64)
    for qi in range(q.shape[0]):
        top = np.argsort(-ref[:, qi], kind="stable")[:11]
        gaps = -np.diff(ref[top, qi])
        if gaps.min() > 1e-5:                                  # unambiguous in fp32
            np.testing.assert_array_equal(ids[qi], top[:10])
        np.testing.assert_allclose(sc[qi], ref[ids[qi], qi], atol=2e-6)


@pytest.mark.parametrize("bits,M,ds", [(4, 16, 2), (8, 8, 4)])
@pytest.mark.parametrize("lut_mode", [0, 1])
def test_search_reorder_all_equals_brute_force(bits, M, ds, lut_mode):
    # Section 1: re-ranking every point exactly is MIPS itself, whatever the codes are.
    rng = np.random.default_rng(21)
    x, cb, codes, q = _setup(rng, 700, M * ds, M, bits)
    ids, sc = oracle.search(x, cb, codes, bits, q, k=10, reorder_k=700, lut_mode=lut_mode)
    bids, bsc = oracle.brute_force(x, q, 10)
    np.testing.assert_array_equal(ids, bids)
    np.testing.assert_array_equal(sc, bsc)


@pytest.mark.parametrize("lut_mode", [0, 1])
def test_search_stages_compose(lut_mode):
    rng = np.random.default_rng(22)
    bits, M, ds = 4, 16, 2
    x, cb, codes, q = _setup(rng, 2000, M * ds, M, bits)
    k, R = 10, 50
    ids, sc = oracle.search(x, cb, codes, bits, q, k, R, lut_mode)
    aids, asc = oracle.search(None, cb, codes, bits, q, R, 0, lut_mode)
    for qi in range(q.shape[0]):
        keys, scale, bias = oracle.adc_keys_flat(q[qi], cb, codes, bits, lut_mode)
        order = np.lexsort((np.arange(2000), -keys.astype(np.float64)))[:R]
        np.testing.assert_array_equal(aids[qi], order)
        if lut_mode == 1:
            want = (keys[order].astype(np.float64) * scale + bias)
            np.testing.assert_allclose(asc[qi], want, atol=1e-5)
        else:
            np.testing.assert_array_equal(asc[qi], keys[order])
        ex = oracle.exact_scores(x[order], q[qi])
        o2 = np.lexsort((order, -ex.astype(np.float64)))[:k]
        np.testing.assert_array_equal(ids[qi], order[o2])
        np.testing.assert_array_equal(sc[qi], ex[o2])


def test_leaf_select_and_partitioned_search():
    rng = np.random.default_rng(23)
    bits, M, ds, n = 4, 8, 2, 1500
    d = M * ds
    x, cb, _, q = _setup(rng, n, d, M, bits)
    cb *= 0.3
    centers = oracle.kmeans(x, 12, iters=5, seed=2)
    assign = oracle.assign_nearest(x, centers)
    codes = oracle.encode(x, cb, T=0.2, leaf_centers=centers, leaf_assign=assign)
    xt = oracle.reconstruct(codes, cb, centers, assign)
    for qi in range(3):
        lids, lip = oracle.leaf_select(centers, q[qi], 5)
        ref = centers.astype(np.float64) @ q[qi].astype(np.float64)
        np.testing.assert_array_equal(lids, np.argsort(-ref, kind="stable")[:5])
        np.testing.assert_allclose(lip, ref[lids], atol=1e-6)
    # probing every leaf scans every point and the key is <q, x~> with x~ = center + PQ
    ids, sc = oracle.search(None, cb, codes, bits, q, k=20, reorder_k=0, lut_mode=0,
                            centers=centers, assign=assign, leaves_to_search=12)
    ref = xt @ q.T.astype(np.float64)
    for qi in range(q.shape[0]):
        np.testing.assert_allclose(sc[qi], ref[ids[qi], qi], atol=3e-6)
        worst_kept = ref[ids[qi], qi].min()
        others = np.setdiff1d(np.arange(n), ids[qi])
        assert ref[others, qi].max() <= worst_kept + 6e-6
    # probing L leaves returns only points of the L best leaves, and all of the best of those
    ids5, sc5 = oracle.search(x, cb, codes, bits, q, k=10, reorder_k=40, lut_mode=0,
                              centers=centers, assign=assign, leaves_to_search=3)
    for qi in range(q.shape[0]):
        lids, _ = oracle.leaf_select(centers, q[qi], 3)
        assert set(assign[ids5[qi]]) <= set(lids)
        np.testing.assert_array_equal(sc5[qi], oracle.exact_scores(x[ids5[qi]], q[qi]))
    # 8-bit tables on a partitioned index: key = acc * scale + bias + leaf_ip, close to fp32 key
    ids8, sc8 = oracle.search(None, cb, codes, bits, q, k=20, reorder_k=0, lut_mode=1,
                              centers=centers, assign=assign, leaves_to_search=12)
    for qi in range(q.shape[0]):
        L = oracle.lut_f32(q[qi], cb)
        _, scale, _ = oracle.lut_u8(L)
        np.testing.assert_allclose(sc8[qi], ref[ids8[qi], qi], atol=M * scale / 2 + 1e-5)


def test_search_on_tiny_config_shapes():
    cfg = si.CONFIGS["tiny"]
    x = si.make_data(cfg, 2000)
    q = si.make_queries(cfg, 5)
    assert x.shape == (2000, 32) and q.shape == (5, 32)
    np.testing.assert_allclose(np.linalg.norm(x, axis=1), 1.0, atol=1e-6)
    cb = oracle.train_pq(x, cfg["M"], 16, iters=5, seed=0)
    codes = oracle.encode(x, cb, T=cfg["T"])
    ids, sc = oracle.search(x, cb, codes, 4, q, 10, 100, 0)
    bids, _ = oracle.brute_force(x, q, 10)
    recall = np.mean([len(set(ids[i]) & set(bids[i])) / 10 for i in range(5)])
    assert recall > 0.5     # sanity only: quantized search finds most true neighbours


def test_quality_metrics_on_a_hand_made_example_and_in_the_exact_limit():
    # Recall 1@N (Section 5.2) and the relative error of the top-1 estimate (Section 5.1), pinned by a case
    # small enough to do by hand: d = 2, one subspace, 4-bit codes; the codewords are the points of a grid.
    cb = np.zeros((1, 16, 2), np.float32)
    cb[0, :4] = [[1.0, 0.0], [0.0, 1.0], [0.5, 0.5], [-1.0, 0.0]]
    x = np.array([[0.9, 0.1], [0.2, 0.8], [0.6, 0.5], [-0.7, 0.1]], np.float32)
    codes = np.array([[0], [1], [2], [3]], np.uint8)          # x~ = (1,0), (0,1), (.5,.5), (-1,0)
    q = np.array([[1.0, 0.0], [0.0, 1.0], [0.6, 0.6]], np.float32)
    # exact scores:   q0: .9 .2 .6 -.7 -> best 0;  q1: .1 .8 .5 .1 -> best 1;  q2: .6 .6 .66 -.36 -> best 2
    # quantized:      q0: 1 0 .5 -1 -> rank of 0 is 1;  q1: 0 1 .5 0 -> rank of 1 is 1;
    #                 q2: .6 .6 .6 -.6 -> three equal scores, ids ascending: 0, 1, 2 -> rank of 2 is 3
    hits, rel = oracle.quality_metrics(x, q, cb, codes, 4, top_n=(1, 2, 3, 4))
    assert hits == {1: 2, 2: 2, 3: 3, 4: 3}
    np.testing.assert_allclose(rel, [0.1 / 0.9, 0.2 / 0.8, 0.06 / 0.66], rtol=1e-6)
    # a quantizer that reproduces every point exactly ranks exactly and estimates without error
    rng = np.random.default_rng(0)
    pts = rng.standard_normal((16, 2)).astype(np.float32)
    cb2 = pts.reshape(1, 16, 2).copy()
    hits, rel = oracle.quality_metrics(pts, rng.standard_normal((20, 2)).astype(np.float32), cb2,
                                       np.arange(16, dtype=np.uint8).reshape(16, 1), 4, top_n=(1, 5))
    assert hits == {1: 20, 5: 20} and np.all(rel < 1e-6)
    # N = n: every datapoint is among the n best, whatever the quantizer
    xs = rng.standard_normal((300, 8)).astype(np.float32)
    cbs = oracle.train_pq(xs, 4, 16, 3, seed=1)
    cds = oracle.encode(xs, cbs, T=0.2, passes=2)
    hits, _ = oracle.quality_metrics(xs, rng.standard_normal((12, 8)).astype(np.float32), cbs, cds, 4, top_n=(1, 300))
    assert hits[300] == 12 and hits[1] <= 12
