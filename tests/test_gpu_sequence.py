"""GPU parity of the principal-minor sequence and the FLODANCE fit (Sec. 3.2, Alg. 2):
the HIP kernels, through the C ABI, against oracle/flodance_oracle.py on the same bits.

Tolerances (derived from the arithmetic):
* ell_k: both sides add k logarithms, each within a couple of ulp of the exact one, in
  different orders: |diff| <= 8 eps sum_{i<=k} |log|d_i||.
* regression: both sides solve the same least-squares problem with backward-stable
  methods, from covariates that differ by a few ulp (log-gamma, square roots): the
  coefficients agree to a small multiple of eps times the condition number of the
  column-scaled design matrix, measured in the scaled coordinates.
* Lhat_n from given coefficients: a handful of operations, 1e-13 relative.
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import workloads as W
from oracle import flodance_oracle as F

pytestmark = pytest.mark.gpu
EPS = np.finfo(np.float64).eps


@pytest.fixture(scope="module")
def M():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_04424_amd as m
    m.load()          # fails loudly if the HIP library is not built
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def synthetic_sequence(seed, n_s, d, noise=1e-3):
    """ell of length n_s d whose every d-th entry follows the curve of Prop. 1 with a
    1/n correction and martingale-like noise; the entries in between hold other values."""
    rng = np.random.default_rng(seed)
    n = np.arange(1, n_s + 1, dtype=np.float64)
    lg = np.array([math.lgamma(v + 1.0) for v in n])
    L = -2.0 + (1 - 1 / n) * 3.1 - (1.45 - 6.0 / n) * lg / n
    L += noise * np.cumsum(rng.standard_normal(n_s)) / n
    ell = rng.standard_normal(n_s * d) * 50.0
    ell[d - 1::d] = L * n
    return ell


# ---------------------------------------------------------------------------
# ell_k
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [1, 5, 256, 4096, 4097, 12289, 70001, 196608])
def test_principal_logdets_against_oracle(M, dtype, n):
    rng = np.random.default_rng(n + (7 if dtype == "f32" else 0))
    npdt = np.float64 if dtype == "f64" else np.float32
    d = (10.0 ** rng.uniform(-8, 3, n) * rng.choice([-1.0, 1.0], n)).astype(npdt)
    want = F.principal_logdets(d)
    got = M.mdet_principal_logdets(dev(d))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    bound = 8 * EPS * np.cumsum(np.abs(np.log(np.abs(d.astype(np.float64))))) + 1e-300
    assert np.all(np.abs(got - want) <= bound)


def test_principal_logdets_singular_pivot_gives_minus_infinity_from_there_on(M):
    d = np.array([2.0, 3.0, 0.0, 5.0])
    got = M.mdet_principal_logdets(dev(d)).cpu().numpy()
    assert abs(got[1] - math.log(6.0)) <= 1e-15 and np.all(np.isneginf(got[2:]))


def test_sequence_of_a_factorisation_matches_the_oracle(M):
    # pivots from the hot path itself -> running sum on the GPU, against the oracle's
    # log-determinants of the leading blocks of the same matrix
    w = W.config(1, "f64")
    a = w.dense()
    r_or = oracle.ldlt_logdet(a, want_diag=True)
    diag = torch.empty(w.n, dtype=torch.float64, device="cuda")
    res = M.mdet_logdet_device(dev(a), block_size=w.block_size, overwrite=True, diag=diag)
    assert res.status == 0
    ell = M.mdet_principal_logdets(diag).cpu().numpy()
    assert np.max(np.abs(ell - r_or.cum_logabs) / np.maximum(1.0, np.abs(r_or.cum_logabs))) <= 1e-10
    assert abs(ell[-1] - res.logabsdet) <= 1e-10 * abs(res.logabsdet)


# ---------------------------------------------------------------------------
# the regression
# ---------------------------------------------------------------------------
def _check_fit(M, ell, d, n0, ns, q, n_eval):
    want = F.fit(ell, d, n0, ns, q)
    coef = M.mdet_flodance_fit(dev(ell), d, n0, ns, q)
    pred = M.mdet_flodance_eval(coef, q, dev(np.asarray(n_eval, dtype=np.float64)))
    torch.cuda.synchronize()
    coef = coef.cpu().numpy()
    pred = pred.cpu().numpy()
    X, y, L_n0 = F.design(ell, d, n0, ns, q)
    scale = np.sqrt((X * X).sum(axis=0))
    cond = np.linalg.cond(X / scale)
    bs_want, bs_got = want.beta * scale, coef[:q + 2] * scale
    tol = 200 * EPS * cond
    assert np.linalg.norm(bs_got - bs_want) <= tol * max(np.linalg.norm(bs_want), np.linalg.norm(y))
    assert coef[q + 2] == L_n0
    # the residual norm: both are |y - X beta| of (nearly) the same minimiser
    assert abs(coef[q + 3] - want.residual) <= 1e-9 * max(np.linalg.norm(y), 1e-300)
    # fitted curve at and beyond the fitted range
    ref = want.eval(np.asarray(n_eval, dtype=np.float64))
    assert np.max(np.abs(pred - ref) / np.maximum(1.0, np.abs(ref))) <= max(1e-9, 10 * tol)
    return coef


@pytest.mark.parametrize("d,n0,ns,q", [
    (1, 1, 257, 0),        # exactly one workgroup of rows
    (1, 1, 301, 1),        # ragged second workgroup
    (3, 7, 160, 2),
    (10, 100, 5000, 4),    # the paper's usage: d = 10 classes, fit interval (1e2, 5e3), q = 4
    (2, 50, 5000, 10),     # the largest q the paper mentions
    (1, 1, 60001, 3),      # three levels of the reduction tree
    (4, 300, 20000, 6),
    (1, 5, 8, 1),          # as many samples as coefficients
])
def test_fit_and_extrapolation_against_oracle(M, d, n0, ns, q):
    ell = synthetic_sequence(1000 + ns + q, ns, d)
    _check_fit(M, ell, d, n0, ns, q, [n0 + 1, (n0 + ns) // 2, ns, 2 * ns, 10 * ns, 50000, 1e6])


def test_exact_law_is_recovered_on_the_gpu(M):
    # ratio law exact (Assumption 1): (c_0, nu) come back and the curve extrapolates
    ell_1, C, nu = -0.8, 5.0, 1.7
    k = np.arange(2, 20001, dtype=np.float64)
    ell = np.concatenate([[ell_1], ell_1 + np.cumsum(np.log(C) - nu * np.log(k))])
    coef = M.mdet_flodance_fit(dev(ell[:2000]), 1, 1, 2000, 0)
    pred = M.mdet_flodance_eval(coef, 0, dev(np.array([20000.0])))
    torch.cuda.synchronize()
    c = coef.cpu().numpy()
    assert abs(c[0] - (math.log(C) - ell_1)) <= 1e-9 and abs(c[1] - nu) <= 1e-10
    assert abs(pred.item() * 20000 - ell[-1]) <= 1e-9 * abs(ell[-1])


def test_eval_from_given_coefficients(M):
    rng = np.random.default_rng(2)
    for q in (0, 3, 10):
        beta = rng.standard_normal(q + 2)
        f = F.FlodanceFit(beta=beta, L_n0=0.75, q=q, residual=0.0)
        n = np.concatenate([[2.0, 3.0, 10.0], 10.0 ** rng.uniform(1, 7, 1000)])
        coef = dev(np.concatenate([beta, [0.75, 0.0]]))
        got = M.mdet_flodance_eval(coef, q, dev(n)).cpu().numpy()
        ref = f.eval(n)
        assert np.max(np.abs(got - ref) / np.maximum(1.0, np.abs(ref))) <= 1e-13


def test_end_to_end_from_a_matrix(M):
    # factorise (hot path) -> pivots -> sequence -> fit -> extrapolate, all on the GPU,
    # against the oracle chain on the same matrix
    w = W.scaled_down(W.config(2, "f64"), 2048, 256)
    a = w.dense()
    r_or = oracle.ldlt_logdet(a, want_diag=True)
    diag = torch.empty(w.n, dtype=torch.float64, device="cuda")
    res = M.mdet_logdet_device(dev(a), block_size=w.block_size, overwrite=True, diag=diag)
    assert res.status == 0
    ell = M.mdet_principal_logdets(diag)
    d, n0, ns, q = 4, 16, 400, 2
    coef = M.mdet_flodance_fit(ell, d, n0, ns, q)
    pred = M.mdet_flodance_eval(coef, q, dev(np.array([400.0, 512.0]))).cpu().numpy()
    want = F.fit(F.principal_logdets(r_or.diag), d, n0, ns, q)
    ref = want.eval(np.array([400.0, 512.0]))
    assert np.max(np.abs(pred - ref) / np.maximum(1.0, np.abs(ref))) <= 1e-7


def test_bad_arguments_and_small_workspace(M):
    ell = dev(np.zeros(1000))
    S = M.Status
    for kw, code in ((dict(d=1, n0=0, ns=50, q=0), S.EINVAL), (dict(d=1, n0=50, ns=50, q=0), S.EINVAL),
                     (dict(d=3, n0=1, ns=400, q=0), S.EINVAL), (dict(d=1, n0=1, ns=50, q=11), S.EINVAL),
                     (dict(d=1, n0=1, ns=50, q=-1), S.EINVAL), (dict(d=1, n0=10, ns=12, q=1), S.EINVAL)):
        with pytest.raises(M.MemdetError) as e:
            M.mdet_flodance_fit(ell, **kw)
        assert e.value.status == code
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MemdetError) as e:
        M.mdet_flodance_fit(ell, 1, 1, 900, 2, workspace=small)
    assert e.value.status == S.ENOMEM_DEVICE
    with pytest.raises(M.MemdetError) as e:
        M.mdet_principal_logdets(dev(np.ones(100000)), workspace=small)
    assert e.value.status == S.ENOMEM_DEVICE
