"""GPU parity of pivoting over the whole diagonal block (MDET_FLAG_PIVOT_BLOCK: P A P^T = L D L^T
with the pivot of every step taken from the diagonal of the current Schur complement anywhere
inside the block column's own b x b diagonal block; Sec. 2.2: pivoting within each block, none
between blocks) against oracle.ldlt_pivoted called with group = b.

As for the 64-column form, the pivot is an argmax over values the two sides round differently,
so the tests compare what is unique (log|det|, sign, inertia; the pivots under the GPU's own
order; the permutation where the candidates are well separated or exactly tied) and check that
the rest is valid (perm keeps every block; every pivot taken was the largest candidate up to
rounding).
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import workloads as W

pytestmark = pytest.mark.gpu
TOL = {"f64": 1e-10, "f32": 1e-4}


def rel(a, b):
    return abs(a - b) / max(1.0, abs(b))


@pytest.fixture(scope="module")
def M():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_04424_amd as m
    m.load()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def indefinite(seed, n, dtype=np.float64):
    """Symmetric, indefinite, well conditioned, with zeros planted on the diagonal so that the
    factorisation without pivoting stops at once."""
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((n, n))
    a = (g + g.T) / math.sqrt(n)
    a[np.arange(n), np.arange(n)] = rng.uniform(4.0, 8.0, n) * rng.choice([-1.0, 1.0], n)
    if n > 1:
        a[0, 0] = 0.0
    if n > 70:
        a[64, 64] = 0.0
    return a.astype(dtype)


def block_of(bs):
    return (bs + 63) // 64 * 64


def run_device(M, a, bs, flags=0, **kw):
    n = a.shape[0]
    ad = dev(a)
    diag = torch.empty(n, dtype=torch.float64 if (flags & M.FLAG_COMPUTE_F64) else ad.dtype, device="cuda")
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    res = M.mdet_logdet_device(ad, block_size=bs, flags=M.FLAG_PIVOT_BLOCK | flags, diag=diag, perm=perm, **kw)
    return res, perm.cpu().numpy().astype(np.int64), diag.cpu().numpy().astype(np.float64), ad


def check_against_oracle(a, perm, d, res, bs, dtype="f64", want_equal_perm=False):
    n, b = a.shape[0], block_of(bs)
    a64 = a.astype(np.float64)
    assert sorted(perm.tolist()) == list(range(n))
    assert np.array_equal(perm // b, np.arange(n) // b)           # no pivoting between blocks
    o = oracle.ldlt_pivoted(a64, group=b)
    assert o.status == 0 and res.status == 0
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= TOL[dtype]
    assert res.negative_pivots == o.negative_pivots
    # the GPU's order handed to the oracle, which then swaps nothing: every pivot taken was the
    # largest candidate of its block up to rounding, and the pivots are the oracle's
    replay = oracle.ldlt_pivoted(a64[perm][:, perm], group=b, choose=False)
    eps = 1e-9 if dtype == "f64" else 1e-3
    assert replay.status == 0 and np.min(replay.slack) >= 1.0 - eps
    assert np.max(np.abs(d - replay.diag) / np.abs(replay.diag)) <= eps
    if want_equal_perm:
        assert np.array_equal(perm, o.perm)
    return o


@pytest.mark.parametrize("n,bs", [(1, 64), (63, 64), (65, 128), (130, 128), (512, 256), (1000, 256), (777, 320),
                                  (1536, 512), (2048, 1024), (1300, 192), (900, 1024)])
def test_indefinite_matrix_pivoted_over_the_whole_diagonal_block(M, n, bs):
    a = indefinite(n + bs, n)
    res, perm, d, _ = run_device(M, a, bs)
    check_against_oracle(a, perm, d, res, bs)
    if n > 64 and bs > 64:
        # the pivots really come from beyond a group of 64: the first pivot is the largest
        # diagonal entry of the first block, wherever it stands
        b = min(block_of(bs), n)
        assert perm[0] == int(np.argmax(np.abs(np.diag(a)[:b])))


def test_separated_candidates_give_the_oracles_permutation(M):
    # diagonal entries far apart compared with the coupling: no near ties at any step
    rng = np.random.default_rng(78)
    n, bs = 768, 256
    g = rng.standard_normal((n, n))
    a = 1e-4 * (g + g.T)
    a[np.arange(n), np.arange(n)] = rng.permutation(1.03 ** np.arange(n)) * rng.choice([-1.0, 1.0], n)
    res, perm, d, _ = run_device(M, a, bs)
    o = check_against_oracle(a, perm, d, res, bs, want_equal_perm=True)
    assert np.max(np.abs(d - o.diag) / np.abs(o.diag)) <= 1e-11


def test_exact_ties_go_to_the_candidate_that_came_first(M):
    dv = np.array([1.0, -2.0, 2.0, 0.5, -2.0, 1.0, 3.0, 3.0] * 40)         # n = 320, one block of 320
    a = np.diag(dv)
    res, perm, d, _ = run_device(M, a, 320)
    o = oracle.ldlt_pivoted(a, group=320)
    assert np.array_equal(perm, o.perm) and np.array_equal(d, o.diag)
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= 1e-14


@pytest.mark.parametrize("cfg,n,bs", [(1, 512, 128), (2, 1536, 256), (3, 1280, 256), (4, 1100, 192)])
def test_paper_workloads(M, cfg, n, bs):
    # positive-definite workloads: the order changes, the determinant does not
    w = W.scaled_down(W.config(cfg), n, bs)
    a = w.dense()
    res, perm, d, _ = run_device(M, a, bs)
    check_against_oracle(a, perm, d, res, bs)
    plain = oracle.ldlt_logdet(a)
    assert rel(res.logabsdet, plain.logabsdet) <= TOL["f64"] and np.all(d > 0)


def test_fp32_and_fp32_storage_with_fp64_arithmetic(M):
    a = indefinite(5, 1024, np.float32)
    res, perm, d, _ = run_device(M, a, 256)
    check_against_oracle(a, perm, d, res, 256, dtype="f32")
    res, perm, d, _ = run_device(M, a, 256, flags=M.FLAG_COMPUTE_F64)
    check_against_oracle(a, perm, d, res, 256)


def test_stored_factor_and_permutation_reconstruct_the_matrix(M):
    # overwrite = 1: each diagonal block holds L and D of that block in pivot order; the rows
    # left of a block keep the input order
    n, bs = 700, 256
    a = indefinite(12, n)
    res, perm, d, ad = run_device(M, a, bs, overwrite=True)
    s = np.tril(ad.cpu().numpy(), -1) + np.eye(n)
    L = s.copy()
    for g0 in range(0, n, bs):
        g1 = min(n, g0 + bs)
        L[g0:g1, :g0] = s[perm[g0:g1], :g0]
    rec = L @ np.diag(d) @ L.T
    assert np.max(np.abs(rec - a[perm][:, perm])) <= 1e-11 * np.max(np.abs(L)) ** 2 * np.max(np.abs(d))
    assert np.array_equal(np.diag(ad.cpu().numpy()), d)
    # every multiplier inside a block is bounded by 1 in magnitude on positive-definite input
    w = W.scaled_down(W.config(1), 600, 256).dense()
    res, perm, d, ad = run_device(M, w, 256, overwrite=True)
    s = np.tril(ad.cpu().numpy(), -1)
    for g0 in range(0, 600, 256):
        g1 = min(600, g0 + 256)
        assert np.max(np.abs(s[g0:g1, g0:g1])) <= 1.0 + 1e-12


def test_same_bits_on_one_stream_and_input_preserved(M):
    a = indefinite(22, 1536)
    r0, p0, d0, _ = run_device(M, a, 512)
    r1, p1, d1, _ = run_device(M, a, 512, flags=M.FLAG_NO_LOOKAHEAD)
    assert r0.logabsdet == r1.logabsdet and np.array_equal(p0, p1) and np.array_equal(d0, d1)
    ad = dev(a)
    res = M.mdet_logdet_device(ad, block_size=512, flags=M.FLAG_PIVOT_BLOCK)
    assert res.status == 0 and res.logabsdet == r0.logabsdet and np.array_equal(ad.cpu().numpy(), a)


@pytest.mark.parametrize("n,bs", [(1024, 128), (1100, 192)])
def test_host_paths_in_core_and_streamed(M, n, bs):
    a = indefinite(n, n)
    F = M.FLAG_PIVOT_BLOCK
    ref, pref, dref, _ = run_device(M, a, bs)
    pk = M.pack_lower_block_columns(torch.from_numpy(a), bs, pin=True)
    diag = torch.empty(n, dtype=torch.float64)
    perm = torch.full((n,), -1, dtype=torch.int32)
    res = M.mdet_logdet_host(pk.clone(), n, bs, flags=F, diag=diag, perm=perm)
    assert not res.out_of_core
    check_against_oracle(a, perm.numpy().astype(np.int64), diag.numpy(), res, bs)
    assert res.logabsdet == ref.logabsdet and np.array_equal(perm.numpy(), pref)
    lo, hi = 0, 1 << 40
    while hi - lo > 4096:
        mid = (lo + hi) // 2
        try:
            M.mdet_plan(n, "f64", bs, mid, flags=M.FLAG_FORCE_OUT_OF_CORE | F)
            hi = mid
        except M.MemdetError:
            lo = mid
    diag2 = torch.empty(n, dtype=torch.float64)
    perm2 = torch.full((n,), -1, dtype=torch.int32)
    res2 = M.mdet_logdet_host(pk.clone(), n, bs, mem_budget=hi, flags=F | M.FLAG_FORCE_OUT_OF_CORE, diag=diag2,
                              perm=perm2)
    assert res2.out_of_core and res2.num_superpanels > 1 and res2.dev_bytes_high_water <= hi
    assert res2.logabsdet == res.logabsdet and torch.equal(perm, perm2) and torch.equal(diag, diag2)


def test_no_usable_pivot_and_non_finite_input(M):
    # [[0, 1], [1, 0]] at the end of a block: every candidate left on the block's diagonal is
    # zero when its turn comes (a 2 x 2 pivot would be needed)
    n = 130
    a = np.eye(n) * 2.0
    a[128:, 128:] = [[0.0, 1.0], [1.0, 0.0]]
    res = M.mdet_logdet_device(dev(a), block_size=128, flags=M.FLAG_PIVOT_BLOCK)
    o = oracle.ldlt_pivoted(a, group=128)
    assert o.status == 1 and o.bad_pivot_index == 128
    assert res.status == M.Status.ESINGULAR and res.bad_pivot_index == 128 and res.sign == 0
    b = indefinite(3, 300)
    b[170, 170] = np.nan
    res = M.mdet_logdet_device(dev(b), block_size=256, flags=M.FLAG_PIVOT_BLOCK)
    assert res.status == M.Status.ENONFINITE and res.bad_pivot_index == 0      # a NaN is taken first in its block


def test_bad_arguments_and_workspace(M):
    a = dev(np.eye(128))
    for extra in (M.FLAG_PIVOT, M.FLAG_ASSUME_SPD, M.FLAG_GENERAL):
        with pytest.raises(M.MemdetError) as e:
            M.mdet_logdet_device(a, block_size=64, flags=M.FLAG_PIVOT_BLOCK | extra)
        assert e.value.status == M.Status.EINVAL
    plain, _ = M.mdet_workspace_query(4096, "f64", 512, for_device_input=True)
    piv, _ = M.mdet_workspace_query(4096, "f64", 512, flags=M.FLAG_PIVOT_BLOCK, for_device_input=True)
    assert piv >= plain + (2 * 512 * 512 + (4096 - 512) * 512) * 8
