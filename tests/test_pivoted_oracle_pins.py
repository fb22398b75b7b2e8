"""Pins for the pivoted form of the CPU oracle (oracle.ldlt_pivoted: P A P^T = L D L^T
with the pivot taken from the diagonal inside a group of consecutive indices; Sec. 2.2:
the symmetric form handles permutations and the diagonal scaling, pivoting stays inside
a block; the software section lists `perm` among the outputs).  Nothing here touches
the GPU library.
"""
import math

import numpy as np
import pytest

import oracle


def _sym(rng, n):
    g = rng.standard_normal((n, n))
    return g + g.T


def _check_perm(perm, n, group):
    assert sorted(perm.tolist()) == list(range(n))
    assert np.array_equal(perm // group, np.arange(n) // group)    # no pivoting between groups


def test_hand_computed_two_by_two():
    # a_00 = 0: the second index is taken first.  d = (4, 0 - 2*2/4), l = 2/4
    r = oracle.ldlt_pivoted(np.array([[0.0, 2.0], [2.0, 4.0]]), want_L=True)
    assert r.status == 0 and r.perm.tolist() == [1, 0]
    assert r.diag.tolist() == [4.0, -1.0] and r.L.tolist() == [[1.0, 0.0], [0.5, 1.0]]
    assert r.sign == -1 and r.negative_pivots == 1 and abs(r.logabsdet - math.log(4.0)) <= 1e-16
    # without pivoting the same matrix has a zero pivot
    assert oracle.ldlt_logdet(np.array([[0.0, 2.0], [2.0, 4.0]])).status == 1


def test_hand_computed_three_by_three_with_a_tie():
    # diag (2, 2, 1): the first of the two equal entries is taken; then the Schur
    # complement [[2 - 1/2, 1 - 0], [1, 1]] -> 1.5 before 1
    a = np.array([[2.0, 1.0, 0.0], [1.0, 2.0, 1.0], [0.0, 1.0, 1.0]])
    r = oracle.ldlt_pivoted(a, want_L=True)
    assert r.perm.tolist() == [0, 1, 2]
    assert np.allclose(r.diag, [2.0, 1.5, 1.0 - 1.0 / 1.5], rtol=1e-15)
    assert abs(r.logabsdet - math.log(1.0)) <= 1e-15      # det = 2*(2-1) - 1*(1) = 1


@pytest.mark.parametrize("n,group", [(1, 64), (2, 64), (5, 2), (7, 4), (64, 64), (65, 64), (150, 64),
                                     (150, 16), (200, 1), (300, 128), (300, 256), (260, 320), (200, 200)])
def test_reconstruction_and_determinant(n, group):
    a = _sym(np.random.default_rng(100 * n + group), n)
    r = oracle.ldlt_pivoted(a, group=group, want_L=True)
    assert r.status == 0
    _check_perm(r.perm, n, group)
    pap = a[r.perm][:, r.perm]
    rec = r.L @ np.diag(r.diag) @ r.L.T
    assert np.max(np.abs(pap - rec)) <= 1e-12 * max(1.0, np.max(np.abs(r.L)) ** 2 * np.max(np.abs(r.diag)))
    assert np.array_equal(np.triu(r.L, 1), np.zeros_like(r.L)) and np.all(np.diag(r.L) == 1.0)
    sg, lad = np.linalg.slogdet(a)
    assert r.sign == sg and abs(r.logabsdet - lad) <= 1e-11 * max(1.0, abs(lad))
    assert r.negative_pivots == int(np.sum(r.diag < 0)) == int(np.sum(np.linalg.eigvalsh(a) < 0))
    assert np.all(r.slack == 1.0)


@pytest.mark.parametrize("n", [2, 3, 4, 6, 8])
def test_against_the_sum_over_permutations(n):
    a = _sym(np.random.default_rng(n), n)
    a[0, 0] = 0.0                                   # forces a swap at the first step
    lad, sg, _ = oracle.leibniz_logdet(a)
    r = oracle.ldlt_pivoted(a, group=n)
    assert r.sign == sg and abs(r.logabsdet - lad) <= 1e-13 * max(1.0, abs(lad))
    assert r.perm[0] != 0


def test_the_rule_is_the_largest_remaining_diagonal_entry():
    # replay by hand in numpy (float64) on a small matrix with well separated values
    rng = np.random.default_rng(5)
    n, group = 12, 6
    a = _sym(rng, n) + np.diag(rng.uniform(-6, 6, n))
    s = a.copy()
    order = []
    for j in range(n):
        cand = [k for k in range(n) if k not in order and (k // group) == (j // group)]
        p = max(cand, key=lambda k: (abs(s[k, k]), -k))
        order.append(p)
        l = s[:, p] / s[p, p]
        s = s - np.outer(l, s[p, :])
        s[p, :] = 0.0
        s[:, p] = 0.0
    r = oracle.ldlt_pivoted(a, group=group)
    assert r.perm.tolist() == order


def test_ties_go_to_the_candidate_that_came_first_in_the_input():
    # repeated magnitudes on a diagonal matrix: a stable sort by magnitude, whatever the
    # swaps of earlier steps did to the positions
    dv = np.array([1.0, -2.0, 2.0, 0.5, -2.0, 1.0, 3.0, 3.0] * 3)
    r = oracle.ldlt_pivoted(np.diag(dv), group=24)
    assert r.perm.tolist() == np.argsort(-np.abs(dv), kind="stable").tolist()
    assert np.array_equal(r.diag, dv[r.perm])


def test_diagonal_matrix_is_sorted_by_magnitude_inside_each_group():
    rng = np.random.default_rng(8)
    n, group = 40, 16
    dv = rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 3, n)
    r = oracle.ldlt_pivoted(np.diag(dv), group=group, want_L=True)
    want = np.concatenate([g0 + np.argsort(-np.abs(dv[g0:g0 + group]), kind="stable")
                           for g0 in range(0, n, group)])
    assert r.perm.tolist() == want.tolist() and np.array_equal(r.diag, dv[want])
    assert np.array_equal(r.L, np.eye(n))


def test_positive_definite_input_gives_bounded_multipliers_inside_a_group():
    # |a_ik| <= sqrt(a_ii a_kk) for every Schur complement of an SPD matrix, so with the
    # largest diagonal entry as the pivot the multipliers of the group's own rows are <= 1
    rng = np.random.default_rng(3)
    n, group = 96, 32
    g = rng.standard_normal((n, n + 3))
    a = g @ g.T
    r = oracle.ldlt_pivoted(a, group=group, want_L=True)
    for g0 in range(0, n, group):
        blk = r.L[g0:g0 + group, g0:g0 + group]
        assert np.max(np.abs(blk)) <= 1.0 + 1e-15
    assert np.all(r.diag > 0)
    assert abs(r.logabsdet - np.linalg.slogdet(a)[1]) <= 1e-11 * abs(r.logabsdet)


def test_without_choice_it_is_the_plain_factorisation_and_reports_the_slack():
    rng = np.random.default_rng(12)
    n = 70
    a = _sym(rng, n) + 30.0 * np.eye(n)
    plain = oracle.ldlt_logdet(a, want_diag=True, want_L=True)
    r = oracle.ldlt_pivoted(a, choose=False, want_L=True)
    assert r.perm.tolist() == list(range(n))
    assert np.max(np.abs(r.diag - plain.diag) / np.abs(plain.diag)) <= 1e-15
    assert np.max(np.abs(r.L - plain.L)) <= 1e-15
    assert abs(r.logabsdet - plain.logabsdet) <= 1e-13 * abs(plain.logabsdet)
    assert np.all(r.slack <= 1.0) and np.min(r.slack) < 1.0
    # a permutation found by the rule, checked through the other door: permute first,
    # factor without choice, every pivot was the largest candidate
    piv = oracle.ldlt_pivoted(a)
    again = oracle.ldlt_pivoted(a[piv.perm][:, piv.perm], choose=False)
    assert np.all(again.slack == 1.0) and np.array_equal(again.diag, piv.diag)


def test_all_candidates_zero_is_reported_as_singular():
    # the degenerate case of pivoting on the diagonal: [[0, 1], [1, 0]] has determinant -1
    # but no usable 1 x 1 pivot
    r = oracle.ldlt_pivoted(np.array([[0.0, 1.0], [1.0, 0.0]]))
    assert r.status == 1 and r.bad_pivot_index == 0 and r.sign == 0 and r.logabsdet == -math.inf
    # and an exactly singular matrix stops at the step where the rank runs out
    v = np.array([1.0, 2.0, -1.0, 0.5])
    r = oracle.ldlt_pivoted(np.outer(v, v))
    assert r.status == 1 and r.bad_pivot_index == 1


def test_only_the_lower_triangle_is_read_and_float32_is_widened_exactly():
    rng = np.random.default_rng(2)
    a = _sym(rng, 25)
    b = np.tril(a) + np.triu(np.full_like(a, np.nan), 1)
    ra, rb = oracle.ldlt_pivoted(a), oracle.ldlt_pivoted(b)
    assert ra.logabsdet == rb.logabsdet and np.array_equal(ra.perm, rb.perm)
    a32 = a.astype(np.float32)
    r32, r64 = oracle.ldlt_pivoted(a32), oracle.ldlt_pivoted(a32.astype(np.float64))
    assert r32.logabsdet == r64.logabsdet and np.array_equal(r32.perm, r64.perm)
