"""Pins for the positive-definite form of the CPU oracle (oracle.cholesky_logdet: unblocked
Cholesky in long double; the paper's algorithm for symmetric positive-definite matrices,
App. D: M = L L^T gives logdet(M[:k,:k]) = 2 sum_{i<=k} log L_ii).  Nothing here touches
the GPU library.
"""
import math

import numpy as np
import pytest

import oracle
from conftest import read_golden


def _spd(rng, n, shift=0.1):
    g = rng.standard_normal((n, n + 5))
    return g @ g.T / n + shift * np.eye(n)


def test_hand_computed_two_by_two():
    # [[4, 2], [2, 5]] = [[2, 0], [1, 2]] [[2, 1], [0, 2]]
    r = oracle.cholesky_logdet(np.array([[4.0, 2.0], [2.0, 5.0]]), want_diag=True, want_L=True)
    assert r.status == 0 and np.array_equal(r.L, [[2.0, 0.0], [1.0, 2.0]])
    assert abs(r.logdet - math.log(16.0)) <= 1e-15
    assert np.allclose(r.cum_logdet, [math.log(4.0), math.log(16.0)], rtol=1e-15)


@pytest.mark.parametrize("n", [1, 2, 7, 40, 150])
def test_factor_and_logdet_against_numpy(n):
    a = _spd(np.random.default_rng(n), n)
    r = oracle.cholesky_logdet(a, want_diag=True, want_L=True)
    L = np.linalg.cholesky(a)
    assert np.max(np.abs(r.L - L)) <= 1e-12 * np.max(np.abs(L))
    sg, lad = np.linalg.slogdet(a)
    assert sg == 1.0 and abs(r.logdet - lad) <= 1e-11 * max(1.0, abs(lad))
    # App. D: the running sums are the log-determinants of the leading blocks
    for k in (1, n // 2, n):
        if k >= 1:
            assert abs(r.cum_logdet[k - 1] - np.linalg.slogdet(a[:k, :k])[1]) <= 1e-11 * max(1.0, abs(lad))


def test_kms_matrix_closed_form_factor():
    # rho^|i-j|: L_i0 = rho^i, L_ij = rho^(i-j) sqrt(1 - rho^2) for j >= 1
    rho, n = 0.6, 120
    idx = np.arange(n)
    a = rho ** np.abs(idx[:, None] - idx[None, :])
    r = oracle.cholesky_logdet(a, want_diag=True, want_L=True)
    want = np.tril(rho ** (idx[:, None] - idx[None, :]).clip(min=0)) * math.sqrt(1 - rho * rho)
    want[:, 0] = rho ** idx
    assert np.max(np.abs(r.L - want)) <= 1e-14
    assert abs(r.logdet - (n - 1) * math.log(1 - rho * rho)) <= 1e-12


@pytest.mark.parametrize("n", [3, 5, 8, 10])
def test_hilbert_matrix_exact_determinant(n):
    gold = read_golden("hilbert_logdet.txt")
    i, j = np.indices((n, n))
    h = 1.0 / (i + j + 1.0)
    r = oracle.cholesky_logdet(h)
    tol = {3: 1e-14, 5: 1e-11, 8: 1e-7, 10: 1e-4}[n]
    assert r.status == 0 and abs(r.logdet - float(gold[str(n)])) < tol


def test_agrees_with_the_ldlt_oracle_entry_by_entry():
    # L_chol = L_unit sqrt(D) and the same log-determinants of all leading blocks
    a = _spd(np.random.default_rng(9), 90, shift=1e-3)
    c = oracle.cholesky_logdet(a, want_diag=True, want_L=True)
    u = oracle.ldlt_logdet(a, want_diag=True, want_L=True)
    assert np.max(np.abs(c.L - u.L * np.sqrt(u.diag)[None, :])) <= 1e-13 * np.max(np.abs(c.L))
    assert np.max(np.abs(c.cum_logdet - u.cum_logabs)) <= 1e-12 * max(1.0, abs(u.logabsdet))
    assert np.max(np.abs(c.diag ** 2 - u.diag) / u.diag) <= 1e-14


def test_first_non_positive_pivot_is_reported():
    rng = np.random.default_rng(4)
    a = _spd(rng, 30)
    a[11, 11] -= 5.0                      # the 12 x 12 leading block becomes indefinite
    r = oracle.cholesky_logdet(a)
    u = oracle.ldlt_logdet(a, want_diag=True)
    first_neg = int(np.argmax(u.diag < 0))
    assert r.status == 3 and r.bad_pivot_index == first_neg == 11 and math.isnan(r.logdet)
    # an exactly singular leading block counts as not positive too
    s = np.array([[1.0, 1.0], [1.0, 1.0]])
    assert oracle.cholesky_logdet(s).bad_pivot_index == 1


def test_only_the_lower_triangle_is_read():
    a = _spd(np.random.default_rng(2), 25)
    b = np.tril(a) + np.triu(np.full_like(a, np.nan), 1)
    assert oracle.cholesky_logdet(b).logdet == oracle.cholesky_logdet(a).logdet


def test_float32_input_is_widened_exactly():
    a = _spd(np.random.default_rng(6), 33).astype(np.float32)
    assert oracle.cholesky_logdet(a).logdet == oracle.cholesky_logdet(a.astype(np.float64)).logdet
