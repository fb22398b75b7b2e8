"""GPU parity of the pivoted form (MDET_FLAG_PIVOT: P A P^T = L D L^T with the pivot taken
from the diagonal inside each group of 64 consecutive indices; Sec. 2.2: the symmetric
form handles permutations, pivoting stays inside a block) against oracle.ldlt_pivoted.

What is compared.  The pivot is an argmax over floating-point values that the two sides
round differently (fp64 in blocked order on the GPU, long double unblocked in the
oracle), so where two candidates are within rounding of each other either choice is
right.  Every test therefore checks what is unique and that the rest is valid:
* perm is a permutation that maps each group of 64 onto itself;
* the oracle, given the matrix permuted by the GPU's perm and told to swap nothing,
  finds that every pivot taken was the largest candidate up to rounding (slack) and
  reproduces the GPU's pivots;
* log|det| and sign against the oracle's own pivoted run: 1e-10 relative in fp64,
  1e-4 in fp32 (the bar of the unpivoted path);
and on matrices whose candidates are well separated the permutations themselves must be
equal.
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import workloads as W

pytestmark = pytest.mark.gpu
TOL = {"f64": 1e-10, "f32": 1e-4}
GROUP = 64


def rel(a, b):
    return abs(a - b) / max(1.0, abs(b))


@pytest.fixture(scope="module")
def M():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_04424_amd as m
    m.load()          # fails loudly if the HIP library is not built
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def indefinite(seed, n, dtype=np.float64):
    """Symmetric, indefinite, well conditioned: a random symmetric part of norm about
    2.8 plus a diagonal of magnitudes in [4, 8] with random signs, some of them moved to
    zero so that the factorisation without pivoting meets a zero or tiny pivot."""
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((n, n))
    a = (g + g.T) / math.sqrt(n)
    dg = rng.uniform(4.0, 8.0, n) * rng.choice([-1.0, 1.0], n)
    a[np.arange(n), np.arange(n)] = dg
    if n > 1:
        a[0, 0] = 0.0
    if n > 70:
        a[64, 64] = 0.0
    return a.astype(dtype)


def check_against_oracle(a, perm, d, res, dtype="f64", want_equal_perm=False):
    n = a.shape[0]
    a64 = a.astype(np.float64)
    assert sorted(perm.tolist()) == list(range(n))
    assert np.array_equal(perm // GROUP, np.arange(n) // GROUP)
    o = oracle.ldlt_pivoted(a64)
    assert o.status == 0 and res.status == 0
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= TOL[dtype]
    assert res.negative_pivots == o.negative_pivots
    replay = oracle.ldlt_pivoted(a64[perm][:, perm], choose=False)
    eps = 1e-9 if dtype == "f64" else 1e-3
    assert replay.status == 0 and np.min(replay.slack) >= 1.0 - eps
    assert np.max(np.abs(d - replay.diag) / np.abs(replay.diag)) <= eps
    if want_equal_perm:
        assert np.array_equal(perm, o.perm)
    return o


# ---------------------------------------------------------------------------
# one block column through the single-step entry point
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("m,w", [(64, 64), (40, 40), (1, 1), (200, 64), (333, 128), (1000, 256), (100, 100)])
def test_block_column_factor_with_pivoting(M, dtype, m, w):
    npdt = np.float64 if dtype == "f64" else np.float32
    a = indefinite(m * 7 + w, m, npdt)
    ad = torch.zeros((m, (m + 3) // 4 * 4), dtype=dev(a).dtype, device="cuda")[:, :m]
    ad.copy_(dev(a))
    d = torch.zeros(w, dtype=ad.dtype, device="cuda")
    dinv = torch.zeros_like(d)
    perm = torch.full((w,), -1, dtype=torch.int32, device="cuda")
    flags = torch.full((2 + 1024,), -1, dtype=torch.int64, device="cuda")
    M.mdet_step_panel_factor_pivoted(ad, w, d, dinv, perm, flags)
    torch.cuda.synchronize()
    assert int(flags[0].item()) == -1
    pw = perm.cpu().numpy().astype(np.int64)
    assert sorted(pw.tolist()) == list(range(w)) and np.array_equal(pw // GROUP, np.arange(w) // GROUP)
    # the oracle on the whole matrix, permuted by the GPU's choice (rows below the block
    # column's diagonal block stay where they are), without further swaps
    full = np.concatenate([pw, np.arange(w, m)])
    a64 = a.astype(np.float64)
    r = oracle.ldlt_pivoted(a64[full][:, full], choose=False, want_L=True)
    tol = 1e-10 if dtype == "f64" else 2e-3
    assert np.min(r.slack[:w]) >= 1.0 - tol
    dd = d.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(dd - r.diag[:w]) / np.abs(r.diag[:w])) < tol
    assert np.max(np.abs(dinv.cpu().numpy().astype(np.float64) * r.diag[:w] - 1)) < tol
    got = ad.cpu().numpy().astype(np.float64)
    # the stored rows of a group keep the input order in the columns before the group
    for g0 in range(GROUP, w, GROUP):
        g1 = min(w, g0 + GROUP)
        got[g0:g1, :g0] = got[pw[g0:g1], :g0]
    i, j = np.indices((m, w))
    strict = i > j
    scale = max(1.0, np.max(np.abs(r.L[:, :w])))
    assert np.max(np.abs(got[:, :w] - r.L[:, :w])[strict], initial=0.0) < tol * scale
    # the oracle's own choice: the same determinant of the leading w x w block
    own = oracle.ldlt_pivoted(a64[:w, :w])
    assert abs(np.sum(np.log(np.abs(dd))) - own.logabsdet) <= tol * max(1.0, abs(own.logabsdet))


def test_leaf_with_separated_candidates_gives_the_oracles_permutation(M):
    # diagonal entries far apart compared with the coupling: no near ties at any step
    rng = np.random.default_rng(77)
    n = 64
    g = rng.standard_normal((n, n))
    a = 1e-3 * (g + g.T)
    a[np.arange(n), np.arange(n)] = rng.permutation(1.5 ** np.arange(n)) * rng.choice([-1.0, 1.0], n)
    ad = dev(a)
    d = torch.zeros(n, dtype=torch.float64, device="cuda")
    dinv = torch.zeros_like(d)
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    flags = torch.full((2 + 1024,), -1, dtype=torch.int64, device="cuda")
    M.mdet_step_panel_factor_pivoted(ad, n, d, dinv, perm, flags)
    torch.cuda.synchronize()
    o = oracle.ldlt_pivoted(a)
    assert np.array_equal(perm.cpu().numpy(), o.perm)
    assert np.max(np.abs(d.cpu().numpy() - o.diag) / np.abs(o.diag)) <= 1e-12


def test_ties_go_to_the_first_candidate(M):
    # exact ties: a diagonal matrix with repeated magnitudes -> stable order on both sides
    dv = np.array([1.0, -2.0, 2.0, 0.5, -2.0, 1.0, 3.0, 3.0] * 8)
    a = np.diag(dv)
    perm = torch.full((64,), -1, dtype=torch.int32, device="cuda")
    diag = torch.empty(64, dtype=torch.float64, device="cuda")
    res = M.mdet_logdet_device(dev(a), block_size=64, flags=M.FLAG_PIVOT, diag=diag, perm=perm)
    o = oracle.ldlt_pivoted(a)
    assert np.array_equal(perm.cpu().numpy(), o.perm) and np.array_equal(diag.cpu().numpy(), o.diag)
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= 1e-14


# ---------------------------------------------------------------------------
# whole path
# ---------------------------------------------------------------------------
def run_device(M, a, bs, flags=0, **kw):
    n = a.shape[0]
    ad = dev(a)
    diag = torch.empty(n, dtype=ad.dtype, device="cuda")
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    res = M.mdet_logdet_device(ad, block_size=bs, flags=M.FLAG_PIVOT | flags, diag=diag, perm=perm, **kw)
    return res, perm.cpu().numpy().astype(np.int64), diag.cpu().numpy().astype(np.float64), ad


@pytest.mark.parametrize("n,bs", [(1, 64), (63, 64), (64, 64), (65, 64), (512, 128), (1000, 256), (777, 64),
                                  (1536, 512), (2048, 1024), (1300, 192)])
def test_indefinite_matrix_that_needs_pivoting(M, n, bs):
    a = indefinite(n + bs, n)
    res, perm, d, _ = run_device(M, a, bs)
    check_against_oracle(a, perm, d, res)
    if n > 1:
        # without pivoting the zero at the top of the diagonal ends the call
        plain = M.mdet_logdet_device(dev(a), block_size=bs)
        assert plain.status == M.Status.ESINGULAR and plain.bad_pivot_index == 0


@pytest.mark.parametrize("cfg,n,bs", [(1, 512, 128), (2, 1536, 256), (3, 1280, 128), (4, 1100, 192)])
def test_paper_workloads_with_pivoting(M, cfg, n, bs):
    # the positive-definite workloads: pivoting changes the order, not the determinant
    w = W.scaled_down(W.config(cfg), n, bs)
    a = w.dense()
    res, perm, d, _ = run_device(M, a, bs)
    check_against_oracle(a, perm, d, res)
    plain = oracle.ldlt_logdet(a)
    assert rel(res.logabsdet, plain.logabsdet) <= TOL["f64"] and np.all(d > 0)


def test_fp32(M):
    a = indefinite(5, 1024, np.float32)
    res, perm, d, _ = run_device(M, a, 256)
    check_against_oracle(a, perm, d, res, dtype="f32")


def test_fp32_storage_with_fp64_arithmetic(M):
    a = indefinite(6, 768, np.float32)
    n = a.shape[0]
    diag = torch.empty(n, dtype=torch.float64, device="cuda")
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    res = M.mdet_logdet_device(dev(a), block_size=128, flags=M.FLAG_PIVOT | M.FLAG_COMPUTE_F64, diag=diag,
                               perm=perm)
    check_against_oracle(a, perm.cpu().numpy().astype(np.int64), diag.cpu().numpy(), res)


def test_stored_factor_and_permutation_reconstruct_the_matrix(M):
    # overwrite = 1: A = M D M^T with M = the stored factor, rows of each diagonal
    # 64 x 64 block scattered by perm
    n, bs = 600, 128
    a = indefinite(11, n)
    res, perm, d, ad = run_device(M, a, bs, overwrite=True)
    s = np.tril(ad.cpu().numpy(), -1) + np.eye(n)
    m = s.copy()
    for g0 in range(0, n, GROUP):
        g1 = min(n, g0 + GROUP)
        m[perm[g0:g1], g0:g1] = s[g0:g1, g0:g1]
    rec = m @ np.diag(d) @ m.T
    assert np.max(np.abs(rec - a)) <= 1e-11 * np.max(np.abs(m)) ** 2 * np.max(np.abs(d))
    # the usual form: rows of the columns before each group permuted too
    L = s.copy()
    for g0 in range(0, n, GROUP):
        g1 = min(n, g0 + GROUP)
        L[g0:g1, :g0] = s[perm[g0:g1], :g0]
    rec2 = L @ np.diag(d) @ L.T
    assert np.max(np.abs(rec2 - a[perm][:, perm])) <= 1e-11 * np.max(np.abs(L)) ** 2 * np.max(np.abs(d))
    # the diagonal of the stored matrix holds D
    assert np.array_equal(np.diag(ad.cpu().numpy()), d)


def test_same_bits_on_one_stream_and_with_the_scaled_copy(M):
    a = indefinite(21, 1536)
    r0, p0, d0, _ = run_device(M, a, 256)
    r1, p1, d1, _ = run_device(M, a, 256, flags=M.FLAG_NO_LOOKAHEAD)
    r2, p2, d2, _ = run_device(M, a, 256, flags=M.FLAG_SCALED_COPY)
    assert r0.logabsdet == r1.logabsdet == r2.logabsdet
    assert np.array_equal(p0, p1) and np.array_equal(p0, p2)
    assert np.array_equal(d0, d1) and np.array_equal(d0, d2)
    assert r0.kernel_launches > M.mdet_logdet_device(dev(a + 9 * np.eye(1536)), block_size=256).kernel_launches


def test_input_is_preserved_without_overwrite(M):
    a = indefinite(31, 500)
    ad = dev(a)
    res = M.mdet_logdet_device(ad, block_size=128, flags=M.FLAG_PIVOT)
    assert res.status == 0 and np.array_equal(ad.cpu().numpy(), a)
    # perm is optional
    o = oracle.ldlt_pivoted(a)
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= TOL["f64"]


@pytest.mark.parametrize("n,bs", [(1024, 128), (1100, 192)])
def test_host_paths_in_core_and_streamed(M, n, bs):
    a = indefinite(n, n)
    pk = M.pack_lower_block_columns(torch.from_numpy(a), bs, pin=True)
    diag = torch.empty(n, dtype=torch.float64)
    perm = torch.full((n,), -1, dtype=torch.int32)
    res = M.mdet_logdet_host(pk.clone(), n, bs, flags=M.FLAG_PIVOT, diag=diag, perm=perm)
    assert not res.out_of_core
    check_against_oracle(a, perm.numpy().astype(np.int64), diag.numpy(), res)
    # streamed under the smallest budget the planner accepts: the same bits
    lo, hi = 0, 1 << 40
    while hi - lo > 4096:
        mid = (lo + hi) // 2
        try:
            M.mdet_plan(n, "f64", bs, mid, flags=M.FLAG_FORCE_OUT_OF_CORE | M.FLAG_PIVOT)
            hi = mid
        except M.MemdetError:
            lo = mid
    diag2 = torch.empty(n, dtype=torch.float64)
    perm2 = torch.full((n,), -1, dtype=torch.int32)
    res2 = M.mdet_logdet_host(pk.clone(), n, bs, mem_budget=hi, flags=M.FLAG_PIVOT | M.FLAG_FORCE_OUT_OF_CORE,
                              diag=diag2, perm=perm2)
    assert res2.out_of_core and res2.num_superpanels > 1 and res2.dev_bytes_high_water <= hi
    assert res2.logabsdet == res.logabsdet and torch.equal(perm, perm2) and torch.equal(diag, diag2)


def test_block_provider_with_pivoting(M):
    import ctypes
    n, bs = 900, 128
    a = indefinite(41, n)

    def provider(bi, bj, rows, cols, dst, ld):
        buf = (ctypes.c_double * (rows * ld)).from_address(dst)
        view = np.frombuffer(buf, dtype=np.float64).reshape(rows, ld)
        view[:, :cols] = a[bi * bs:bi * bs + rows, bj * bs:bj * bs + cols]
        return 0

    diag = torch.empty(n, dtype=torch.float64)
    perm = torch.full((n,), -1, dtype=torch.int32)
    res = M.mdet_logdet_provider(provider, n, "f64", bs, flags=M.FLAG_PIVOT, diag=diag, perm=perm)
    check_against_oracle(a, perm.numpy().astype(np.int64), diag.numpy(), res)
    ref, p_ref, d_ref, _ = run_device(M, a, bs)
    assert res.logabsdet == ref.logabsdet and np.array_equal(perm.numpy(), p_ref)


def test_no_usable_pivot_is_reported_as_singular(M):
    # [[0, 1], [1, 0]] inside a larger matrix: determinant -1, but every candidate on the
    # diagonal is zero when its turn comes (a 2 x 2 pivot would be needed)
    n = 130
    a = np.eye(n) * 2.0
    a[128:, 128:] = [[0.0, 1.0], [1.0, 0.0]]
    res = M.mdet_logdet_device(dev(a), block_size=64, flags=M.FLAG_PIVOT)
    o = oracle.ldlt_pivoted(a)
    assert o.status == 1 and o.bad_pivot_index == 128
    assert res.status == M.Status.ESINGULAR and res.bad_pivot_index == 128
    assert res.sign == 0 and res.logabsdet == -math.inf


def test_non_finite_input_is_reported(M):
    a = indefinite(3, 200)
    a[70, 70] = np.nan
    res = M.mdet_logdet_device(dev(a), block_size=64, flags=M.FLAG_PIVOT)
    assert res.status == M.Status.ENONFINITE and res.bad_pivot_index == 64   # taken first in its group


def test_bad_arguments(M):
    a = dev(np.eye(128))
    with pytest.raises(M.MemdetError) as e:
        M.mdet_logdet_device(a, block_size=64, flags=M.FLAG_PIVOT | M.FLAG_ASSUME_SPD)
    assert e.value.status == M.Status.EINVAL
    with pytest.raises(ValueError):
        M.mdet_logdet_device(a, block_size=64, flags=M.FLAG_PIVOT,
                             perm=torch.zeros(128, dtype=torch.int64, device="cuda"))
    # the workspace grows by the permutation
    plain, _ = M.mdet_workspace_query(4096, "f64", 512, for_device_input=True)
    piv, _ = M.mdet_workspace_query(4096, "f64", 512, flags=M.FLAG_PIVOT, for_device_input=True)
    assert piv == plain + 4096 * 4
