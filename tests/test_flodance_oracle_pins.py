"""Pins for the CPU oracle of the principal-minor sequence and the FLODANCE fit
(oracle/flodance_oracle.py; Sec. 3.2, Alg. 2): each test ties it to something other
than itself.  Nothing here touches the GPU library.
"""
import math

import mpmath as mp
import numpy as np
import pytest

import oracle
from oracle import flodance_oracle as F


# ---- ell_k = log|det| of the leading k x k block ----------------------------
def test_principal_logdets_match_slogdet_of_every_leading_block():
    rng = np.random.default_rng(11)
    n = 40
    g = rng.standard_normal((n, n + 8))
    a = g @ g.T / n + 0.05 * np.eye(n)
    a[5, 5] -= 3.0                       # indefinite from the 6th block on: exercises |.|
    a = np.tril(a) + np.tril(a, -1).T
    diag = oracle.ldlt_logdet(a, want_diag=True).diag
    ell = F.principal_logdets(diag)
    signs = set()
    for k in range(1, n + 1):
        sg, lad = np.linalg.slogdet(a[:k, :k])
        signs.add(sg)
        assert abs(ell[k - 1] - lad) <= 1e-10 * max(1.0, abs(lad))
    assert signs == {1.0, -1.0}


def test_principal_logdets_of_the_kms_matrix_closed_form():
    # KMS matrix rho^|i-j|: det of the k x k block is (1 - rho^2)^(k-1)
    rho, n = 0.7, 300
    idx = np.arange(n)
    a = rho ** np.abs(idx[:, None] - idx[None, :])
    diag = oracle.ldlt_logdet(a, want_diag=True).diag
    ell = F.principal_logdets(diag)
    want = (idx) * math.log(1.0 - rho * rho)
    assert np.max(np.abs(ell - want)) <= 1e-11 * n


# ---- the regression ----------------------------------------------------------
def _ell_from_ratio_law(ell_1, C, nu, n_max):
    """ell_n when det K_n / det K_{n-1} = C n^-nu holds exactly (Assumption 1, Eq. (5)),
    built from the recurrence itself: no factorial, no log-gamma."""
    k = np.arange(2, n_max + 1, dtype=np.float64)
    steps = np.log(C) - nu * np.log(k)
    return np.concatenate([[ell_1], ell_1 + np.cumsum(steps.astype(np.longdouble)).astype(np.float64)])


def test_exact_scaling_law_is_recovered_and_extrapolated():
    # with the ratio law exact, Prop. 1 holds with c_0 = log C - ell_1 and no error
    # term, so q = 0 and n_0 = 1 must return (c_0, nu) and extrapolate exactly
    ell_1, C, nu = -0.8, 5.0, 1.7
    ell = _ell_from_ratio_law(ell_1, C, nu, 20000)
    f = F.fit(ell[:2000], d=1, n_0=1, n_s=2000, q=0)
    assert abs(f.beta[0] - (math.log(C) - ell_1)) <= 1e-9
    assert abs(f.beta[1] - nu) <= 1e-10
    assert f.residual <= 1e-9
    for n in (2000, 7777, 20000):
        assert abs(f.eval(float(n)) * n - ell[n - 1]) <= 1e-9 * abs(ell[n - 1])


def test_higher_order_terms_are_recovered():
    # nu(n) = nu_0 + nu_1 / n + nu_2 / n^2 in the curve of App. "Derivation of FLODANCE
    # Parameterization"; the fit with q = 2 returns all five coefficients
    L1, c0, nus = 0.3, 2.5, (1.2, -4.0, 9.0)
    n = np.arange(1, 3001, dtype=np.float64)
    lg = np.array([float(mp.loggamma(int(v) + 1)) for v in n])
    L = L1 + (1 - 1 / n) * c0 - (nus[0] + nus[1] / n + nus[2] / n ** 2) * lg / n
    f = F.fit(L * n, d=1, n_0=1, n_s=3000, q=2)
    assert np.allclose(f.beta, [c0, *nus], rtol=0, atol=2e-6)
    assert abs(f.eval(50000.0) - (L1 + (1 - 1 / 5e4) * c0 - (nus[0] + nus[1] / 5e4 + nus[2] / 25e8)
                                  * float(mp.loggamma(50001)) / 5e4)) <= 1e-9


def test_fit_equals_the_normal_equations_in_50_digit_arithmetic():
    # beta = (X^T X)^-1 X^T y exactly as Alg. 2 writes it, every quantity formed in
    # 50-digit arithmetic from the same ell, on a noisy sequence with burn-in and d > 1
    mp.mp.dps = 50
    rng = np.random.default_rng(5)
    d, n_0, n_s, q = 3, 7, 160, 2
    n = np.arange(1, n_s + 1, dtype=np.float64)
    L = 1.0 + (1 - 1 / n) * 2.0 - 1.4 * np.array([math.lgamma(v + 1) for v in n]) / n
    L += 1e-3 * rng.standard_normal(n_s) / np.sqrt(n)
    ell = np.full(n_s * d, np.nan)
    ell[d - 1::d] = L * n                 # only every d-th entry may be read
    f = F.fit(ell, d=d, n_0=n_0, n_s=n_s, q=q)

    Lmp = [mp.mpf(float(ell[j * d - 1])) / j for j in range(1, n_s + 1)]
    rows, ys = [], []
    for nj in range(n_0 + 1, n_s + 1):
        r = mp.sqrt(nj - 1)
        lg = mp.loggamma(nj + 1)
        rows.append([r] + [-lg / (r * mp.mpf(nj) ** (i - 1)) for i in range(1, q + 2)])
        ys.append(mp.mpf(nj) / r * (Lmp[nj - 1] - Lmp[n_0 - 1]))
    X = mp.matrix(rows)
    y = mp.matrix(ys)
    beta = mp.lu_solve(X.T * X, X.T * y)
    for i in range(q + 2):
        assert abs(f.beta[i] - float(beta[i])) <= 1e-9 * max(1.0, abs(float(beta[i])))
    n_big = 5000
    want = Lmp[n_0 - 1] + beta[0] * (1 - mp.mpf(1) / n_big) - sum(
        beta[i] * mp.loggamma(n_big + 1) / mp.mpf(n_big) ** i for i in range(1, q + 2))
    assert abs(f.eval(float(n_big)) - float(want)) <= 1e-10 * abs(float(want))


def test_eval_on_hand_computed_numbers():
    # q = 0: Lhat_4 = L_n0 + c_0 (3/4) - nu_0 log(24) / 4
    f = F.FlodanceFit(beta=np.array([2.0, 0.5]), L_n0=1.0, q=0, residual=0.0)
    assert abs(f.eval(4.0) - (1.0 + 1.5 - 0.5 * math.log(24.0) / 4.0)) <= 1e-15
    # q = 1 adds - nu_1 log(24) / 16
    f1 = F.FlodanceFit(beta=np.array([2.0, 0.5, 3.0]), L_n0=1.0, q=1, residual=0.0)
    assert abs(f1.eval(4.0) - (1.0 + 1.5 - 0.5 * math.log(24.0) / 4.0 - 3.0 * math.log(24.0) / 16.0)) <= 1e-15


def test_design_rows_on_hand_computed_numbers():
    # d = 2, n_0 = 1, n_s = 3: L_1 = ell_2, L_2 = ell_4 / 2, L_3 = ell_6 / 3
    ell = np.array([9.0, 1.0, 9.0, 6.0, 9.0, 12.0])
    X, y, L_n0 = F.design(ell, d=2, n_0=1, n_s=3, q=1)
    assert L_n0 == 1.0 and X.shape == (2, 3)
    # n = 2: y = 2/sqrt(1) (3 - 1), X = [1, -log 2, -log(2)/2]
    assert y[0] == 4.0
    assert np.allclose(X[0], [1.0, -math.log(2.0), -math.log(2.0) / 2.0], rtol=1e-15, atol=0)
    # n = 3: y = 3/sqrt(2) (4 - 1), X = [sqrt 2, -log(6)/sqrt 2, -log(6)/(3 sqrt 2)]
    assert abs(y[1] - 9.0 / math.sqrt(2.0)) <= 1e-15
    assert np.allclose(X[1], [math.sqrt(2.0), -math.log(6.0) / math.sqrt(2.0),
                              -math.log(6.0) / (3.0 * math.sqrt(2.0))], rtol=1e-15, atol=0)


def test_shift_of_the_sequence_moves_only_the_level():
    rng = np.random.default_rng(3)
    n = np.arange(1, 801, dtype=np.float64)
    L = 0.2 * np.log(n) + 1e-2 * rng.standard_normal(800)
    f = F.fit(L * n, d=1, n_0=20, n_s=800, q=1)
    g = F.fit((L + 7.5) * n, d=1, n_0=20, n_s=800, q=1)
    assert np.allclose(f.beta, g.beta, rtol=1e-8, atol=1e-8)
    assert abs((g.eval(5000.0) - f.eval(5000.0)) - 7.5) <= 1e-8


def test_bad_arguments_are_rejected():
    ell = np.zeros(100)
    for kw in (dict(d=1, n_0=0, n_s=50, q=0), dict(d=1, n_0=50, n_s=50, q=0),
               dict(d=3, n_0=1, n_s=40, q=0), dict(d=1, n_0=1, n_s=50, q=-1)):
        with pytest.raises(ValueError):
            F.design(ell, **kw)
