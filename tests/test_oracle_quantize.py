"""Pins for the oracle's training, encoding and codebook updates.

The oracle is compared with brute force on tiny inputs, with special cases that
reduce to textbook routines (nearest codeword, cluster mean), with the worked
example the paper prints, and with optimality conditions checked numerically.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _loss_np(x, xt, eta):
    """Independent form of the loss: the quadratic form in the proof of Theorem 4.2."""
    x, xt = np.asarray(x, np.float64), np.asarray(xt, np.float64)
    A = (eta - 1) * np.outer(x, x) / (x @ x) + np.eye(x.size)
    return xt @ A @ xt - 2 * eta * (x @ xt) + eta * (x @ x)


def _rand_pq(rng, n, d, M, kc):
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    cb = (0.4 * rng.standard_normal((M, kc, d // M))).astype(np.float32)
    return x, cb


def test_worked_example_layout():
    # Appendix 7.5: c = (-1,-1,1,1,-2,-2,2,2); codes (0,1) -> (-1,-1,2,2); (1,0) -> (1,1,-2,-2)
    with open(os.path.join(GOLD, "pq_worked_example.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    c = np.array(rows[0], np.float32).reshape(2, 2, 2)   # [M][kc][ds]
    for r in rows[1:]:
        code = np.array([[int(r[0]), int(r[1])]], np.uint8)
        want = np.array(r[2:], np.float64)
        np.testing.assert_array_equal(oracle.reconstruct(code, c)[0], want)


def test_pack_codes_layout():
    codes = np.array([[1, 2, 3, 4, 5], [15, 0, 9, 8, 7]], np.uint8)
    p4 = oracle.pack_codes(codes, 4)
    # even subspace in the low nibble; odd M leaves the last high nibble zero
    np.testing.assert_array_equal(p4, [[0x21, 0x43, 0x05], [0x0F, 0x89, 0x07]])
    np.testing.assert_array_equal(oracle.pack_codes(codes, 8), codes)


def test_encode_eta1_is_nearest_codeword():
    # eta = 1 makes the loss the reconstruction error, which separates over
    # subspaces: the encoding is the nearest codeword in every subspace.
    rng = np.random.default_rng(11)
    x, cb = _rand_pq(rng, 300, 24, 6, 16)
    got = oracle.encode(x, cb, T=0.2, eta_mode=2, eta_explicit=1.0, passes=5)
    xs = x.reshape(300, 6, 1, 4).astype(np.float64)
    want = np.argmin(((xs - cb[None].astype(np.float64)) ** 2).sum(-1), axis=-1)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("M,kc,ds", [(1, 16, 4), (2, 4, 2), (3, 4, 2), (2, 16, 1)])
def test_encode_vs_exhaustive_enumeration(M, kc, ds):
    rng = np.random.default_rng(12 + M)
    d = M * ds
    x, cb = _rand_pq(rng, 40, d, M, kc)
    eta = 4.125
    cd = oracle.encode(x, cb, T=0.2, eta_mode=2, eta_explicit=eta, passes=20)
    for i in range(x.shape[0]):
        # brute force over all kc^M code vectors with the independent loss
        best, bestv = None, np.inf
        for code in itertools.product(range(kc), repeat=M):
            xt = np.concatenate([cb[m, code[m]] for m in range(M)]).astype(np.float64)
            v = _loss_np(x[i], xt, eta)
            if v < bestv - 1e-15:
                best, bestv = code, v
        ex_code, ex_v = oracle.encode_exhaustive(x[i], cb, eta)
        assert tuple(ex_code) == best
        assert ex_v == pytest.approx(bestv, rel=1e-9, abs=1e-12)
        xt_cd = oracle.reconstruct(cd[i:i + 1], cb)[0]
        v_cd = _loss_np(x[i], xt_cd, eta)
        assert v_cd >= bestv - 1e-12
        if M == 1:
            assert tuple(cd[i]) == best
        # coordinate-wise optimal: no single-subspace change lowers the loss
        for m in range(M):
            for j in range(kc):
                alt = cd[i].copy()
                alt[m] = j
                v = _loss_np(x[i], oracle.reconstruct(alt[None], cb)[0], eta)
                assert v >= v_cd - 1e-12


def test_encode_loss_non_increasing_in_passes_and_beats_l2_codes():
    rng = np.random.default_rng(13)
    x, cb = _rand_pq(rng, 200, 32, 16, 16)
    eta = oracle.eta_limit(32, 0.2)
    prev = None
    for passes in (0, 1, 2, 3, 10):
        codes = oracle.encode(x, cb, T=0.2, passes=passes)
        xt = oracle.reconstruct(codes, cb)
        loss = np.array([_loss_np(x[i], xt[i], eta) for i in range(x.shape[0])])
        if prev is not None:
            assert np.all(loss <= prev + 1e-12)
        prev = loss
    # passes = 0 is the l2 start; the anisotropic codes must differ somewhere and be no worse
    l2 = oracle.encode(x, cb, T=0.2, passes=0)
    assert np.any(l2 != codes)


def test_encode_uses_per_point_norm():
    # Theorem 3.2: the weights depend on ||x_i||. A point scaled by c with codebooks
    # scaled by c must get the codes of the unscaled problem run at threshold T/c.
    rng = np.random.default_rng(14)
    x, cb = _rand_pq(rng, 100, 16, 8, 16)
    a = oracle.encode(x, cb, T=0.5)
    b = oracle.encode(2 * x, 2 * cb, T=1.0)
    np.testing.assert_array_equal(a, b)
    c = oracle.encode(2 * x, 2 * cb, T=0.5)       # different eta: some codes change
    assert np.any(a != c)


def test_encode_with_leaf_centers_vs_enumeration():
    rng = np.random.default_rng(15)
    M, kc, ds = 2, 4, 2
    x, cb = _rand_pq(rng, 30, M * ds, M, kc)
    cb *= 0.3
    centers = (x[:3] + 0.05 * rng.standard_normal((3, M * ds))).astype(np.float32)
    assign = rng.integers(0, 3, size=30).astype(np.int32)
    eta = 3.0
    for i in range(30):
        ce = centers[assign[i]]
        best, bestv = None, np.inf
        for code in itertools.product(range(kc), repeat=M):
            xt = ce.astype(np.float64) + np.concatenate([cb[m, code[m]] for m in range(M)])
            v = _loss_np(x[i], xt, eta)
            if v < bestv - 1e-15:
                best, bestv = code, v
        ex_code, ex_v = oracle.encode_exhaustive(x[i], cb, eta, center=ce)
        assert tuple(ex_code) == best
    cd = oracle.encode(x, cb, T=0.2, eta_mode=2, eta_explicit=eta, leaf_centers=centers,
                       leaf_assign=assign)
    xt = oracle.reconstruct(cd, cb, centers, assign)
    for i in range(30):
        ex_code, ex_v = oracle.encode_exhaustive(x[i], cb, eta, center=centers[assign[i]])
        assert _loss_np(x[i], xt[i], eta) >= ex_v - 1e-12


def test_init_indices_distinct_and_stratified():
    for n, k in ((16, 16), (1000, 16), (262144, 256)):
        idx = [oracle.init_index(7, 3, j, k, n) for j in range(k)]
        assert len(set(idx)) == k
        for j, i in enumerate(idx):
            assert (j * n) // k <= i < ((j + 1) * n) // k
    assert oracle.init_index(7, 3, 5, 16, 1000) != oracle.init_index(8, 3, 5, 16, 1000) or \
        oracle.init_index(7, 3, 6, 16, 1000) != oracle.init_index(8, 3, 6, 16, 1000)


def test_kmeans_recovers_separated_clusters_and_is_fixed_point():
    rng = np.random.default_rng(16)
    k, d, per = 8, 5, 200
    true = 10.0 * rng.standard_normal((k, d))
    lab = np.repeat(np.arange(k), per)
    perm = rng.permutation(k * per)
    # interleave so every stratum of the initial draw contains every cluster; the test
    # only relies on the result being a fixed point with the textbook update
    x = (true[lab] + 0.1 * rng.standard_normal((k * per, d))).astype(np.float32)[perm]
    c = oracle.kmeans(x, k, iters=25, seed=3)
    a = oracle.assign_nearest(x, c)
    # Lloyd fixed point: every center is the mean of the points assigned to it
    for j in range(k):
        if np.any(a == j):
            np.testing.assert_allclose(c[j], x[a == j].astype(np.float64).mean(0), rtol=0, atol=2e-6)
    # assignment is the nearest center (fp64), ties aside
    d2 = ((x[:, None, :].astype(np.float64) - c[None].astype(np.float64)) ** 2).sum(-1)
    np.testing.assert_array_equal(a, d2.argmin(1))


def test_kmeans_objective_non_increasing():
    rng = np.random.default_rng(17)
    x = rng.standard_normal((2000, 4)).astype(np.float32)
    prev = np.inf
    for it in range(0, 8):
        c = oracle.kmeans(x, 16, iters=it, seed=1)
        d2 = ((x[:, None, :].astype(np.float64) - c[None]) ** 2).sum(-1).min(1).sum()
        assert d2 <= prev + 1e-6
        prev = d2


def test_train_pq_is_per_subspace_kmeans_and_residual_mode():
    rng = np.random.default_rng(18)
    x = rng.standard_normal((1500, 8)).astype(np.float32)
    cb = oracle.train_pq(x, M=4, kc=16, iters=6, seed=5)
    assert cb.shape == (4, 16, 2)
    # each subspace's dictionary is a set of means of its own columns only:
    # changing other columns must not change it
    x2 = x.copy()
    x2[:, 2:] = rng.standard_normal((1500, 6)).astype(np.float32)
    cb2 = oracle.train_pq(x2, M=4, kc=16, iters=6, seed=5)
    np.testing.assert_array_equal(cb[0], cb2[0])
    assert np.any(cb[1] != cb2[1])
    # residual mode equals plain mode on explicitly subtracted data
    centers = rng.standard_normal((5, 8)).astype(np.float32)
    assign = rng.integers(0, 5, 1500).astype(np.int32)
    resid = (x.astype(np.float64) - centers[assign].astype(np.float64))
    cb_r = oracle.train_pq(x, 4, 16, 6, 5, leaf_centers=centers, leaf_assign=assign)
    cb_e = oracle.train_pq(resid.astype(np.float32), 4, 16, 6, 5)
    np.testing.assert_allclose(cb_r, cb_e, atol=1e-5)


def test_vq_update_reduces_to_mean_and_has_zero_gradient():
    rng = np.random.default_rng(19)
    xm = rng.standard_normal((50, 6))
    # Section 4: equal weights -> weighted average; w = 1 -> plain mean
    h = rng.uniform(0.5, 2.0, 50)
    np.testing.assert_allclose(oracle.vq_update(xm, h, h), (h[:, None] * xm).sum(0) / h.sum(), rtol=1e-10)
    np.testing.assert_allclose(oracle.vq_update(xm, np.ones(50), np.ones(50)), xm.mean(0), rtol=1e-10)
    # Theorem 4.2: c* minimises sum_i h_par ||r_par||^2 + h_perp ||r_perp||^2
    hp, ho = 3.0 * h, h
    c = oracle.vq_update(xm, hp, ho)

    def total(cc):
        return sum(ho[i] * oracle.aniso_loss(xm[i], cc, hp[i] / ho[i]) for i in range(50))
    base = total(c)
    for l in range(6):
        e = np.zeros(6)
        e[l] = 1e-4
        g = (total(c + e) - total(c - e)) / 2e-4
        assert abs(g) < 1e-6 * max(1.0, abs(base))
        assert total(c + e) >= base and total(c - e) >= base


def test_pq_joint_update_properties():
    rng = np.random.default_rng(20)
    n, d, M, kc = 400, 6, 3, 4
    x, cb = _rand_pq(rng, n, d, M, kc)
    codes = oracle.encode(x, cb, T=0.2, eta_mode=2, eta_explicit=3.0)
    # eta = 1: the joint solve is the mean of the assigned sub-vectors (k-means update)
    cb1 = oracle.pq_joint_update(x, codes, np.ones(n), cb)
    for m in range(M):
        for j in range(kc):
            sel = codes[:, m] == j
            if sel.any():
                np.testing.assert_allclose(cb1[m, j], x[sel, 2 * m:2 * m + 2].astype(np.float64).mean(0), atol=1e-6)
            else:
                np.testing.assert_array_equal(cb1[m, j], cb[m, j])
    # eta > 1: total loss does not increase and the gradient vanishes
    eta = np.full(n, 3.0)
    cb3 = oracle.pq_joint_update(x, codes, eta, cb)

    def total(cbx):
        xt = oracle.reconstruct(codes, cbx)
        return sum(_loss_np(x[i], xt[i], 3.0) for i in range(n))
    assert total(cb3) <= total(cb) + 1e-9
    base = total(cb3)
    for idx in [(0, 0, 0), (1, 2, 1), (2, 3, 0)]:
        if not (codes[:, idx[0]] == idx[1]).any():
            continue
        up, dn = cb3.copy(), cb3.copy()
        up[idx] += 1e-3
        dn[idx] -= 1e-3
        assert abs(total(up) - total(dn)) / 2e-3 < 2e-3 * max(1.0, base)
        assert total(up) >= base - 1e-7 and total(dn) >= base - 1e-7


def _total_loss(x, xt, etas):
    return sum(oracle.aniso_loss(x[i], xt[i], etas[i]) for i in range(x.shape[0]))


def test_joint_update_with_leaf_centers_has_zero_gradient_and_reduces_to_the_flat_case():
    # Appendix 7.5 on a partitioned index: x~ = center + PQ(residual), loss against the original x.
    rng = np.random.default_rng(21)
    n, d, M, kc, L = 400, 6, 3, 4, 5
    x = rng.standard_normal((n, d)).astype(np.float32)
    x *= rng.uniform(0.5, 1.5, (n, 1)).astype(np.float32)
    centers = rng.standard_normal((L, d)).astype(np.float32) * 0.5
    assign = rng.integers(0, L, n).astype(np.int32)
    codes = rng.integers(0, kc, (n, M)).astype(np.uint8)
    cb0 = rng.standard_normal((M, kc, d // M)).astype(np.float32)
    etas = np.array([oracle.eta(0, d, 0.4, float(np.linalg.norm(r))) for r in x])
    cb = oracle.pq_joint_update(x, codes, etas, cb0, centers, assign)

    def loss(cbv):
        xt = oracle.reconstruct(codes, cbv.astype(np.float32), centers, assign)
        return _total_loss(x.astype(np.float64), xt, etas)

    base = loss(cb)
    assert base < loss(cb0)
    # a stationary point of a convex quadratic: central differences vanish, any step increases the loss
    h = 1e-3
    for _ in range(12):
        e = np.zeros_like(cb)
        idx = tuple(rng.integers(0, s) for s in cb.shape)
        e[idx] = h
        up, dn = loss(cb + e), loss(cb - e)
        assert abs(up - dn) / (2 * h) < 2e-3 * max(1.0, base), (idx, up, dn)
        assert up >= base - 1e-6 and dn >= base - 1e-6
    # zero centers: the flat update; eta = 1: the mean of the residuals of every codeword's members
    flat = oracle.pq_joint_update(x, codes, etas, cb0)
    np.testing.assert_allclose(oracle.pq_joint_update(x, codes, etas, cb0, np.zeros((L, d), np.float32), assign), flat,
                               rtol=0, atol=1e-6)
    ones = np.ones(n)
    cb1 = oracle.pq_joint_update(x, codes, ones, cb0, centers, assign)
    res = x - centers[assign]
    for m in range(M):
        for j in range(kc):
            mem = codes[:, m] == j
            np.testing.assert_allclose(cb1[m, j], res[mem][:, m * 2:(m + 1) * 2].mean(axis=0), rtol=0, atol=2e-6)


def test_anisotropic_leaf_assignment_and_center_update():
    rng = np.random.default_rng(22)
    n, d, L = 300, 8, 7
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    centers = rng.standard_normal((L, d)).astype(np.float32) * 0.6
    # eta = 1 (T = 0): the nearest center
    np.testing.assert_array_equal(oracle.assign_aniso(x, centers, 0.0), oracle.assign_nearest(x, centers))
    # T = 0.5: the arg min of the loss of Section 3.2 evaluated from its definition, by brute force
    a = oracle.assign_aniso(x, centers, 0.5)
    e = oracle.eta(0, d, 0.5, 1.0)
    for i in range(0, n, 7):
        losses = [oracle.aniso_loss(x[i], centers[j], oracle.eta(0, d, 0.5, float(np.linalg.norm(x[i])))) for j in range(L)]
        assert a[i] == int(np.argmin(losses))
    assert np.mean(a != oracle.assign_nearest(x, centers)) > 0.02 and e > 1.0   # the loss matters
    # Theorem 4.2 per partition: no other center of a partition has a smaller loss; the total loss falls
    new = oracle.vq_centers_update(x, a, centers, 0.5)
    etas = np.array([oracle.eta(0, d, 0.5, float(np.linalg.norm(r))) for r in x])
    before = _total_loss(x.astype(np.float64), centers[a].astype(np.float64), etas)
    after = _total_loss(x.astype(np.float64), new[a].astype(np.float64), etas)
    assert after < before
    for _ in range(10):
        pert = new + (rng.standard_normal(new.shape) * 1e-2).astype(np.float32)
        assert _total_loss(x.astype(np.float64), pert[a].astype(np.float64), etas) >= after - 1e-9
