"""Pins for the CPU oracle: each test ties it to something other than itself.

The oracle (oracle/ldlt_oracle.c) is the unblocked long-double LDL^T of the
symmetric case of the paper's method (Sec. 2.2; App. D).  Nothing here touches
the GPU library.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W
from conftest import read_golden

REL = lambda a, b: abs(a - b) / max(1.0, abs(b))


def _sym(rng, n, scale=1.0):
    a = rng.standard_normal((n, n)) * scale
    return a + a.T


# ---- brute force ----------------------------------------------------------
def test_leibniz_on_hand_computed_determinants():
    # values worked by hand (cofactor expansion)
    assert oracle.leibniz_logdet(np.array([[2.0, 1.0], [1.0, 2.0]]))[2] == 3.0
    a = np.array([[2.0, -1.0, 0.0], [-1.0, 2.0, -1.0], [0.0, -1.0, 2.0]])
    assert oracle.leibniz_logdet(a)[2] == 4.0          # tridiagonal(−1,2,−1): det = n+1
    b = np.array([[0.0, 1.0], [1.0, 0.0]])
    lad, sg, det = oracle.leibniz_logdet(b)
    assert (sg, det, lad) == (-1, -1.0, 0.0)
    c = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0], [7.0, 8.0, 10.0]])  # non-symmetric
    assert oracle.leibniz_logdet(c)[2] == -3.0
    # a 3-cycle permutation matrix is even: det = +1 (catches a wrong parity rule)
    p = np.array([[0.0, 1.0, 0.0], [0.0, 0.0, 1.0], [1.0, 0.0, 0.0]])
    assert oracle.leibniz_logdet(p)[2] == 1.0


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7])
def test_ldlt_matches_leibniz_on_random_symmetric_indefinite(n):
    rng = np.random.default_rng(100 + n)
    seen_neg = 0
    for trial in range(12):
        a = _sym(rng, n)
        # unpivoted LDL^T needs nonzero leading minors: true with probability 1
        r = oracle.ldlt_logdet(a)
        lad, sg, _ = oracle.leibniz_logdet(a)
        assert r.sign == sg
        assert abs(r.logabsdet - lad) <= 1e-11 * max(1.0, abs(lad)) + 1e-11
        seen_neg += r.sign < 0
    if n >= 2:
        assert seen_neg > 0  # both signs exercised


def test_ldlt_matches_exact_rational_elimination():
    # integer symmetric matrices: the determinant is an exact integer
    rng = np.random.default_rng(7)
    for n in (3, 6, 9, 12):
        m = rng.integers(-4, 5, size=(n, n))
        a = (m + m.T + np.diag(rng.integers(6, 12, size=n))).astype(np.int64)
        fa = [[Fraction(int(x)) for x in row] for row in a]
        det = Fraction(1)
        for k in range(n):
            det *= fa[k][k]
            for i in range(k + 1, n):
                f = fa[i][k] / fa[k][k]
                for j in range(k, n):
                    fa[i][j] -= f * fa[k][j]
        r = oracle.ldlt_logdet(a.astype(np.float64))
        assert r.sign == (1 if det > 0 else -1)
        assert REL(r.logabsdet, math.log(abs(det))) < 1e-15 * n


def test_only_lower_triangle_is_read():
    rng = np.random.default_rng(3)
    a = _sym(rng, 9) + 9 * np.eye(9)
    b = np.tril(a) + np.triu(np.full((9, 9), np.nan), 1)
    assert oracle.ldlt_logdet(b).logabsdet == oracle.ldlt_logdet(a).logabsdet


# ---- closed forms ---------------------------------------------------------
def test_diagonal_and_scaled_identity():
    rng = np.random.default_rng(5)
    d = rng.uniform(0.1, 10.0, size=300) * rng.choice([-1.0, 1.0], size=300)
    r = oracle.ldlt_logdet(np.diag(d), want_diag=True)
    assert REL(r.logabsdet, float(np.sum(np.log(np.abs(d))))) < 1e-14
    assert r.sign == int(np.prod(np.sign(d)))
    assert np.array_equal(r.diag, d)
    assert r.negative_pivots == int(np.sum(d < 0))
    n, c = 777, 3.25
    r = oracle.ldlt_logdet(c * np.eye(n))
    assert REL(r.logabsdet, n * math.log(c)) < 1e-15


@pytest.mark.parametrize("n,rho", [(7, 0.3), (512, 0.5)])
def test_kms_closed_form_logdet_pivots_and_factor(n, rho):
    gold = read_golden("kms_closed_form.txt")
    a = W.kms(n, rho).dense()
    r = oracle.ldlt_logdet(a, want_diag=True, want_L=True)
    assert r.sign == 1
    assert REL(r.logabsdet, float(gold[f"{n}_{rho}"])) < 1e-14
    # every pivot and every entry of L is known in closed form
    d_exact = np.full(n, 1 - rho * rho)
    d_exact[0] = 1.0
    assert np.max(np.abs(r.diag - d_exact)) < 1e-15
    i, j = np.indices((n, n))
    L_exact = np.where(i >= j, rho ** np.abs(i - j).astype(float), 0.0)
    assert np.max(np.abs(r.L - L_exact)) < 1e-15
    # leading principal minors: (k-1) log(1-rho^2)
    k = np.arange(n)
    assert np.max(np.abs(r.cum_logabs - k * math.log1p(-rho * rho))) < 1e-12 * n


@pytest.mark.parametrize("n", [3, 5, 8, 10])
def test_hilbert_matrix_exact_determinant(n):
    # ill-conditioned (cond ~ 1e13 at n=10): long double keeps ~5 digits more than double
    gold = read_golden("hilbert_logdet.txt")
    i, j = np.indices((n, n))
    # entries 1/(i+j+1) are rounded to double on input; the determinant's relative
    # sensitivity to that rounding is ~ cond * 2^-53
    h = 1.0 / (i + j + 1.0)
    r = oracle.ldlt_logdet(h)
    tol = {3: 1e-14, 5: 1e-11, 8: 1e-7, 10: 1e-4}[n]
    assert r.sign == 1
    assert abs(r.logabsdet - float(gold[str(n)])) < tol


def test_higham_two_by_two_gram_matrix():
    # Sec. 2.1: J = [[1, eps], [1, 0]],  det(J J^T) = eps^2; once 1+eps^2 rounds
    # to 1 the stored Gram matrix is exactly singular.
    eps = 1e-3
    g = np.array([[1.0 + eps * eps, 1.0], [1.0, 1.0]])
    r = oracle.ldlt_logdet(g)
    # det of the stored matrix is exactly g00*1 - 1*1 (g00 - 1 is exact in binary)
    assert r.sign == 1 and REL(r.logabsdet, math.log(g[0, 0] - 1.0)) < 4e-15
    eps = 1e-9   # eps < sqrt(2^-53): fl(1+eps^2) == 1
    g = np.array([[1.0 + eps * eps, 1.0], [1.0, 1.0]])
    r = oracle.ldlt_logdet(g)
    assert (r.sign, r.status, r.bad_pivot_index) == (0, 1, 1)
    assert r.logabsdet == -math.inf
    # in float32 the same happens already for eps = 1e-4 (< sqrt(2^-24))
    g32 = np.array([[1.0 + 1e-8, 1.0], [1.0, 1.0]], dtype=np.float32)
    assert oracle.ldlt_logdet(g32).sign == 0


# ---- identities -----------------------------------------------------------
def test_scaling_identity():
    a = W.scaled_down(W.config(1), 200).dense()
    base = oracle.ldlt_logdet(a).logabsdet
    for c in (1e-30, 0.37, 4096.0, 1e25):
        r = oracle.ldlt_logdet(c * a)
        assert REL(r.logabsdet, 200 * math.log(c) + base) < 1e-14
    r = oracle.ldlt_logdet(-2.0 * a[:201 - 2, :201 - 2])   # odd order: sign flips
    assert r.sign == -1 and r.negative_pivots == 199


def test_block_schur_additivity():
    # Eq. 1: det M = det M11 * det S,  S = M22 - M21 M11^-1 M12
    a = W.scaled_down(W.config(1), 240).dense()
    for b in (1, 64, 100, 239):
        a11, a21, a22 = a[:b, :b], a[b:, :b], a[b:, b:]
        s = a22 - a21 @ np.linalg.solve(a11, a21.T)
        s = (s + s.T) / 2
        total = oracle.ldlt_logdet(a).logabsdet
        parts = oracle.ldlt_logdet(a11).logabsdet + oracle.ldlt_logdet(s).logabsdet
        assert REL(parts, total) < 1e-12


def test_leading_principal_minor_sequence():
    # App. D: the factorisation yields logdet of every leading principal block
    rng = np.random.default_rng(11)
    a = _sym(rng, 60) + 0.5 * np.eye(60)     # indefinite
    r = oracle.ldlt_logdet(a, want_diag=True)
    for k in (1, 2, 17, 59, 60):
        sg, lad = np.linalg.slogdet(a[:k, :k])
        assert REL(r.cum_logabs[k - 1], lad) < 1e-11
        assert int(np.prod(np.sign(r.diag[:k]))) == int(sg)


def test_cholesky_identity_on_spd():
    # App. D: logdet(M[:k,:k]) = 2 sum_{i<=k} log L_ii for the Cholesky factor
    a = W.scaled_down(W.config(2), 300).dense()
    c = np.linalg.cholesky(a)
    r = oracle.ldlt_logdet(a, want_diag=True)
    cum = 2 * np.cumsum(np.log(np.diag(c)))
    assert np.max(np.abs(r.cum_logabs - cum) / np.maximum(1, np.abs(cum))) < 1e-9
    assert r.negative_pivots == 0


def test_low_rank_plus_shift_identity():
    # logdet(F F^T/p + eps I_n) = (n-p) log eps + logdet(F^T F/p + eps I_p)
    w = W.scaled_down(W.config(3), 768)          # p = 192, decay 0.75, shift 1e-8
    f = w.factor()
    k = w.dense()
    small = f.T @ f / w.p + w.shift * np.eye(w.p)
    lhs = oracle.ldlt_logdet(k)
    rhs = (w.n - w.p) * math.log(w.shift) + oracle.ldlt_logdet(small).logabsdet
    assert lhs.sign == 1
    # K is rounded to double after forming F F^T: the 576 pivots of size 1e-8 each see
    # a relative perturbation ~ 2^-53 * |K| / 1e-8 ~ 1e-11, random in sign
    assert REL(lhs.logabsdet, rhs) < 1e-11


@pytest.mark.parametrize("cfg,n", [(1, 384), (2, 512), (3, 512), (4, 512)])
def test_against_library_slogdet_and_eigenvalues(cfg, n):
    a = W.scaled_down(W.config(cfg), n).dense().astype(np.float64)
    r = oracle.ldlt_logdet(a)
    sg, lad = np.linalg.slogdet(a)
    assert r.sign == int(sg)
    assert REL(r.logabsdet, lad) < 1e-9
    ev = np.linalg.eigvalsh(a)
    assert REL(r.logabsdet, float(np.sum(np.log(np.abs(ev))))) < 1e-7


def test_float32_input_is_read_exactly():
    a64 = W.scaled_down(W.config(1), 128).dense()
    a32 = a64.astype(np.float32)
    r32 = oracle.ldlt_logdet(a32)
    r64 = oracle.ldlt_logdet(a32.astype(np.float64))   # same bits, widened
    assert r32.logabsdet == r64.logabsdet and r32.sign == r64.sign


def test_planted_mistakes_are_caught_by_the_pins():
    """The pins above are sharp: numpy emulations of plausible slips in the
    recurrence (dropped D in the update, wrong sign) miss the KMS closed form."""
    n, rho = 24, 0.5
    a = W.kms(n, rho).dense()
    exact = (n - 1) * math.log1p(-rho * rho)

    def ldl(a, drop_d=False, plus=False):
        n = a.shape[0]
        l = np.eye(n)
        d = np.zeros(n)
        for j in range(n):
            w = l[j, :j] * (1.0 if drop_d else d[:j])
            s = l[j, :j] @ w
            d[j] = a[j, j] + s if plus else a[j, j] - s
            for i in range(j + 1, n):
                l[i, j] = (a[i, j] - l[i, :j] @ w) / d[j]
        return float(np.sum(np.log(np.abs(d))))

    assert abs(ldl(a) - exact) < 1e-12
    assert abs(ldl(a, drop_d=True) - exact) > 1e-3
    assert abs(ldl(a, plus=True) - exact) > 1e-3
    assert REL(oracle.ldlt_logdet(a).logabsdet, exact) < 1e-14
