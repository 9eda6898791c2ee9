"""Pins for the oracle's eta, residual decomposition and loss.

Each check compares the oracle with something it does not compute itself:
the constant the paper prints, numerical quadrature of the defining integrals,
algebraic identities of the decomposition, and a Monte-Carlo estimate of the
score-aware loss of Definition 3.1.
"""
import os

import numpy as np
import pytest
from scipy import integrate

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_eta_printed_constant():
    # Section 5.1: T = 0.2 corresponds to eta = 4.125 by the limit of Eq. 3 (d = 100).
    for d, T, norm, want in _rows("eta_printed.txt"):
        assert oracle.eta_limit(int(d), float(T), float(norm)) == pytest.approx(float(want), abs=1e-12)


def test_eta_special_case_T0():
    # Section 3.2: T = 0 gives eta = 1 (parallel and orthogonal error weighted equally).
    for d in (2, 3, 8, 32, 100, 255, 256):
        assert oracle.eta_exact(d, 0.0, 1.0) == pytest.approx(1.0, abs=1e-9)
        assert oracle.eta_limit(d, 0.0, 1.0) == 1.0


def _eta_quadrature(d, T, norm):
    # h_par / h_perp of Section 3.2 straight from the two integrals (main-text form).
    a = np.arccos(T / norm)
    hp = (d - 1) * integrate.quad(lambda t: np.sin(t) ** (d - 2) - np.sin(t) ** d, 0, a,
                                  epsabs=0, epsrel=1e-13, limit=400)[0]
    ho = integrate.quad(lambda t: np.sin(t) ** d, 0, a, epsabs=0, epsrel=1e-13, limit=400)[0]
    return hp / ho


@pytest.mark.parametrize("d", [2, 3, 4, 8, 31, 32, 100, 128, 256, 1000])
@pytest.mark.parametrize("T,norm", [(0.2, 1.0), (0.1, 1.0), (0.5, 1.0), (0.2, 0.7), (0.2, 2.0)])
def test_eta_exact_matches_quadrature(d, T, norm):
    assert oracle.eta_exact(d, T, norm) == pytest.approx(_eta_quadrature(d, T, norm), rel=1e-8)


def test_sin_power_integrals_satisfy_recursion():
    # Appendix (proof of Theorem 3.4): d I_d = (d-1) I_{d-2} - cos(alpha) sin^{d-1}(alpha),
    # with I_0 = alpha and I_1 = 1 - cos(alpha).
    for T in (0.1, 0.2, 0.5, 0.9):
        a = np.arccos(T)
        assert oracle.sin_power_integral(0, a) == pytest.approx(a, rel=1e-13)
        assert oracle.sin_power_integral(1, a) == pytest.approx(1 - np.cos(a), rel=1e-12)
        for d in (2, 3, 10, 33, 100, 256):
            lhs = d * oracle.sin_power_integral(d, a)
            rhs = (d - 1) * oracle.sin_power_integral(d - 2, a) - np.cos(a) * np.sin(a) ** (d - 1)
            assert lhs == pytest.approx(rhs, rel=1e-9)


def test_eta_exact_d2_closed_form():
    # d = 2: I_0 = alpha, I_2 = (alpha - sin alpha cos alpha)/2, eta = I_0/I_2 - 1.
    for T in (0.05, 0.2, 0.6):
        a = np.arccos(T)
        want = a / ((a - np.sin(a) * np.cos(a)) / 2) - 1
        assert oracle.eta_exact(2, T, 1.0) == pytest.approx(want, rel=1e-12)


def test_eta_ratio_monotone_to_limit():
    # Theorem 3.4 and its proof: eta/(d-1) is non-increasing in d and tends to
    # u/(1-u), u = (T/||x||)^2, from above; Theorem 3.3: eta >= 1.
    T = 0.2
    lim = T * T / (1 - T * T)
    for parity in (0, 1):
        prev = np.inf
        for d in range(2 + parity, 300, 6):
            r = oracle.eta_exact(d, T, 1.0) / (d - 1)
            assert r <= prev * (1 + 1e-9)
            assert r >= lim
            assert oracle.eta_exact(d, T, 1.0) >= 1.0
            prev = r
    assert oracle.eta_exact(4000, T, 1.0) / 3999 == pytest.approx(lim, rel=2e-2)


def test_eta_norm_scaling_and_degenerate():
    # eta depends on T and ||x|| only through T/||x||.
    assert oracle.eta_exact(64, 0.2, 1.0) == pytest.approx(oracle.eta_exact(64, 0.4, 2.0), rel=1e-12)
    assert oracle.eta_limit(64, 0.2, 1.0) == pytest.approx(oracle.eta_limit(64, 0.4, 2.0), rel=1e-12)
    # readings: zero vector -> 1; T >= ||x|| -> finite clamp; proxy floored at 1
    assert oracle.eta_limit(64, 0.2, 0.0) == 1.0
    assert np.isfinite(oracle.eta_limit(64, 2.0, 1.0))
    assert oracle.eta_limit(10, 0.05, 1.0) == 1.0
    assert oracle.eta(2, 64, 0.2, 1.0, 3.5) == 3.5


def test_decomposition_identities():
    rng = np.random.default_rng(5)
    for d in (2, 7, 100):
        x = rng.standard_normal(d)
        xt = x + 0.3 * rng.standard_normal(d)
        rp, ro = oracle.residual_decompose(x, xt)
        r = x - xt
        np.testing.assert_allclose(rp + ro, r, atol=1e-14)
        assert abs(rp @ ro) < 1e-13
        # r_par is a multiple of x, r_perp is orthogonal to x
        assert abs(ro @ x) < 1e-13
        assert np.linalg.matrix_rank(np.stack([rp, x]), tol=1e-10) == 1
        assert rp @ rp == pytest.approx((r @ x) ** 2 / (x @ x), rel=1e-12)


def test_loss_equals_quadratic_form():
    # Proof of Theorem 4.2: h_par||r_par||^2 + h_perp||r_perp||^2 =
    # x~^T((h_par-h_perp) x x^T/||x||^2 + h_perp I) x~ - 2 h_par x^T x~ + h_par ||x||^2
    rng = np.random.default_rng(6)
    for d in (3, 16, 100):
        x = rng.standard_normal(d)
        xt = rng.standard_normal(d)
        eta = 4.125
        A = (eta - 1) * np.outer(x, x) / (x @ x) + np.eye(d)
        want = xt @ A @ xt - 2 * eta * (x @ xt) + eta * (x @ x)
        assert oracle.aniso_loss(x, xt, eta) == pytest.approx(want, rel=1e-10)


def test_loss_eta1_is_reconstruction_error():
    rng = np.random.default_rng(7)
    x, xt = rng.standard_normal(20), rng.standard_normal(20)
    assert oracle.aniso_loss(x, xt, 1.0) == pytest.approx(np.sum((x - xt) ** 2), rel=1e-12)


def test_loss_matches_score_aware_definition_monte_carlo():
    # Definition 3.1 with w = I(t >= T), q uniform on the unit sphere:
    # l(x, x~) = E[w(<q,x>) <q, x - x~>^2] is proportional to
    # eta ||r_par||^2 + ||r_perp||^2 with eta the exact ratio. Compare the ratio
    # of the losses of two different quantizations against a direct estimate.
    d, T = 8, 0.2
    rng = np.random.default_rng(8)
    x = rng.standard_normal(d)
    x /= np.linalg.norm(x)
    ortho = rng.standard_normal(d)
    ortho -= (ortho @ x) * x
    ortho /= np.linalg.norm(ortho)
    xt_a = x - 0.3 * x                      # purely parallel residual
    xt_b = x - 0.3 * ortho                  # purely orthogonal residual, same length
    xt_c = x - 0.2 * x - 0.25 * ortho       # mixed
    est = np.zeros(3)
    cnt = 0
    for _ in range(8):
        q = rng.standard_normal((1_000_000, d))
        q /= np.linalg.norm(q, axis=1, keepdims=True)
        w = (q @ x) >= T
        for i, xt in enumerate((xt_a, xt_b, xt_c)):
            est[i] += np.sum(w * (q @ (x - xt)) ** 2)
        cnt += q.shape[0]
    eta = oracle.eta_exact(d, T, 1.0)
    la, lb, lc = (oracle.aniso_loss(x, xt, eta) for xt in (xt_a, xt_b, xt_c))
    assert est[0] / est[1] == pytest.approx(la / lb, rel=0.02)   # this ratio is eta itself
    assert la / lb == pytest.approx(eta, rel=1e-9)
    assert est[2] / est[1] == pytest.approx(lc / lb, rel=0.02)
