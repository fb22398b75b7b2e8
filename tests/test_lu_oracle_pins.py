"""Pins for the generic form of the CPU oracle (oracle.lu_logdet: A[perm, :] = L U with the
pivot of each column taken among the rows of its group of consecutive indices; Sec. 2.2,
Eq. 1 and Alg. 1: M = P L U, det M = sign(P) prod U_jj; pivoting inside a block, none
between blocks).  Nothing here touches the GPU library.
"""
import math

import numpy as np
import pytest

import oracle


def _lu(r, n):
    return np.tril(r.LU, -1) + np.eye(n), np.triu(r.LU)


def test_hand_computed_two_by_two():
    # [[0, 2], [3, 4]]: the second row comes first; L = [[1, 0], [0, 1]], U = [[3, 4], [0, 2]];
    # det = -(3 * 2) = -6
    r = oracle.lu_logdet(np.array([[0.0, 2.0], [3.0, 4.0]]), want_LU=True)
    assert r.status == 0 and r.perm.tolist() == [1, 0] and r.diag.tolist() == [3.0, 2.0]
    assert r.LU.tolist() == [[3.0, 4.0], [0.0, 2.0]]
    assert r.sign == -1 and abs(r.logabsdet - math.log(6.0)) <= 1e-15


def test_hand_computed_three_by_three():
    # partial pivoting picks 4 (row 2), then the larger of the two remaining entries of column 1
    a = np.array([[2.0, 1.0, 1.0], [1.0, 3.0, 2.0], [4.0, 1.0, 0.0]])
    r = oracle.lu_logdet(a, want_LU=True)
    assert r.perm.tolist() == [2, 1, 0]
    L, U = _lu(r, 3)
    assert np.allclose(L, [[1, 0, 0], [0.25, 1, 0], [0.5, 0.5 / 2.75, 1]], rtol=1e-15)
    det = 2 * (3 * 0 - 2 * 1) - 1 * (1 * 0 - 2 * 4) + 1 * (1 * 1 - 3 * 4)       # cofactors: -7
    assert r.sign == -1 and abs(r.logabsdet - math.log(abs(det))) <= 1e-15


@pytest.mark.parametrize("n,group", [(1, 64), (2, 64), (5, 2), (7, 3), (64, 64), (65, 64), (150, 64), (150, 16),
                                     (200, 200)])
def test_reconstruction_and_determinant(n, group):
    rng = np.random.default_rng(100 * n + group)
    a = rng.standard_normal((n, n))
    if n > 1:
        a[0, 0] = 0.0                       # no factorisation without a row exchange
    r = oracle.lu_logdet(a, group=group, want_LU=True)
    assert r.status == 0
    assert sorted(r.perm.tolist()) == list(range(n))
    assert np.array_equal(r.perm // group, np.arange(n) // group)        # no pivoting between groups
    L, U = _lu(r, n)
    assert np.max(np.abs(a[r.perm] - L @ U)) <= 1e-12 * max(1.0, np.max(np.abs(L)) * np.max(np.abs(U)))
    assert np.array_equal(np.diag(U), r.diag)
    sg, lad = np.linalg.slogdet(a)
    assert r.sign == sg and abs(r.logabsdet - lad) <= 1e-11 * max(1.0, abs(lad))
    assert r.negative_pivots == int(np.sum(r.diag < 0))
    # inside its group every multiplier is at most 1 (partial pivoting)
    for g0 in range(0, n, group):
        assert np.max(np.abs(np.tril(L[g0:g0 + group, g0:g0 + group], -1)), initial=0.0) <= 1.0


@pytest.mark.parametrize("n", [2, 3, 4, 6, 8])
def test_against_the_sum_over_permutations(n):
    a = np.random.default_rng(n).standard_normal((n, n))
    a[0, 0] = 0.0
    lad, sg, _ = oracle.leibniz_logdet(a)
    r = oracle.lu_logdet(a, group=n)
    assert r.sign == sg and abs(r.logabsdet - lad) <= 1e-13 * max(1.0, abs(lad))


def test_whole_matrix_as_one_group_is_lapack_s_partial_pivoting():
    scipy_linalg = pytest.importorskip("scipy.linalg")
    n = 120
    a = np.random.default_rng(3).standard_normal((n, n))
    lu, piv = scipy_linalg.lu_factor(a)
    r = oracle.lu_logdet(a, group=n, want_LU=True)
    perm = np.arange(n)
    for j, p in enumerate(piv):             # LAPACK's sequence of row exchanges
        perm[[j, p]] = perm[[p, j]]
    assert np.array_equal(r.perm, perm)
    assert np.max(np.abs(r.LU - lu)) <= 1e-12 * np.max(np.abs(lu))


def test_symmetric_positive_definite_input_agrees_with_the_symmetric_oracle():
    rng = np.random.default_rng(9)
    g = rng.standard_normal((80, 90))
    a = g @ g.T / 80 + 0.1 * np.eye(80)
    assert abs(oracle.lu_logdet(a).logabsdet - oracle.ldlt_logdet(a).logabsdet) <= 1e-12 * 80


def test_permutation_sign_alone():
    # a permutation matrix: every pivot is 1, the determinant is the sign of the permutation
    p = np.array([2, 0, 3, 1, 4])
    a = np.eye(5)[p]
    r = oracle.lu_logdet(a, group=5)
    inversions = sum(1 for i in range(5) for j in range(i + 1, 5) if p[i] > p[j])
    assert r.logabsdet == 0.0 and r.sign == (-1) ** inversions and np.all(r.diag == 1.0)


def test_column_of_zeros_inside_the_group_is_singular_and_the_upper_triangle_is_read():
    a = np.array([[0.0, 1.0], [0.0, 2.0]])
    r = oracle.lu_logdet(a)
    assert r.status == 1 and r.bad_pivot_index == 0 and r.sign == 0 and r.logabsdet == -math.inf
    # a pivot that only a row outside the group could supply
    b = np.array([[0.0, 1.0, 0.0], [0.0, 0.0, 1.0], [1.0, 0.0, 0.0]])
    assert oracle.lu_logdet(b, group=2).status == 1 and oracle.lu_logdet(b, group=3).status == 0
    c = np.array([[1.0, 5.0], [0.0, 1.0]])
    assert oracle.lu_logdet(c, want_LU=True).LU[0, 1] == 5.0
    c32 = np.random.default_rng(1).standard_normal((20, 20)).astype(np.float32)
    assert oracle.lu_logdet(c32).logabsdet == oracle.lu_logdet(c32.astype(np.float64)).logabsdet
