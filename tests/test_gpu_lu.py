"""GPU parity of the form for general matrices (MDET_FLAG_GENERAL: P A = L D U with the
pivot of every column taken among the rows of its group of 64 consecutive rows; Sec. 2.2,
Eq. 1 and Alg. 1: M = P L U for generic matrices, pivoting inside a block, none between
blocks) against oracle.lu_logdet.

What is compared.  The pivot is an argmax over floating-point values that the two sides
round differently, so where two candidates are within rounding of each other either
choice is right.  Every test checks what is unique and that the rest is valid:
* perm is a permutation that maps each group of 64 onto itself;
* the oracle, given the rows in the GPU's order and told to choose nothing (groups of one
  row), reproduces the GPU's pivots;
* log|det| and sign against the oracle's own run: 1e-10 relative in fp64, 1e-4 in fp32;
and on matrices whose candidates are well separated the permutations and the factors
themselves must be equal.
"""
import math
import os

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


def shuffled_dominant(seed, n, dtype=np.float64):
    """A general matrix that needs its rows exchanged and says clearly which: entries of
    magnitude 4 .. 8 with random signs on the diagonal plus unsymmetric noise of norm about
    1.4, then the rows shuffled inside every group of 64.  The diagonal of the result is
    mostly noise, some of it set to exactly zero."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((n, n)) / math.sqrt(2.0 * n)
    a[np.arange(n), np.arange(n)] = rng.uniform(4.0, 8.0, n) * rng.choice([-1.0, 1.0], n)
    rows = np.concatenate([g0 + rng.permutation(min(GROUP, n - g0)) for g0 in range(0, n, GROUP)])
    a = a[rows]
    if n > 1 and rows[0] != 0:
        a[0, 0] = 0.0
    return np.ascontiguousarray(a.astype(dtype))


def gaussian(seed, n, dtype=np.float64):
    """No structure at all: independent standard normal entries."""
    return np.random.default_rng(seed).standard_normal((n, n)).astype(dtype)


def run_device(M, a, bs, flags=0, overwrite=False):
    n = a.shape[0]
    ad = dev(a)
    diag = torch.empty(n, dtype=ad.dtype, device="cuda")
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    res = M.mdet_logdet_device(ad, block_size=bs, flags=M.FLAG_GENERAL | flags, diag=diag, perm=perm,
                               overwrite=overwrite)
    return res, perm.cpu().numpy().astype(np.int64), diag.cpu().numpy().astype(np.float64), ad


def check_against_oracle(a, perm, d, res, dtype="f64", want_equal_perm=False, pivots=True):
    n = a.shape[0]
    a64 = a.astype(np.float64)
    assert sorted(perm.tolist()) == list(range(n))
    assert np.array_equal(perm // GROUP, np.arange(n) // GROUP)
    o = oracle.lu_logdet(a64)
    assert o.status == 0 and res.status == 0
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= TOL[dtype]
    assert res.negative_pivots == int(np.sum(d < 0))
    # the rows in the GPU's order, eliminated with no choice left
    replay = oracle.lu_logdet(a64[perm], group=1)
    eps = 1e-8 if dtype == "f64" else 2e-3
    assert replay.status == 0
    if pivots:
        assert np.max(np.abs(d - replay.diag) / np.abs(replay.diag)) <= eps
    if want_equal_perm:
        assert np.array_equal(perm, o.perm)
    return o


def stored_factors(s, perm):
    """(L, U) of A[perm] = L diag(d) U from the array the library returns with
    overwrite = 1: rows of every group gathered for the columns left of the group."""
    n = s.shape[0]
    L = np.tril(s, -1) + np.eye(n)
    for g0 in range(0, n, GROUP):
        g1 = min(n, g0 + GROUP)
        L[g0:g1, :g0] = np.tril(s, -1)[perm[g0:g1], :g0]
    U = np.triu(s, 1) + np.eye(n)
    return L, U


# ---------------------------------------------------------------------------
# one block column through the single-step entry point
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("m,w", [(64, 64), (40, 40), (1, 1), (200, 64), (333, 128), (1000, 256), (100, 100)])
def test_block_column_factor_of_a_general_matrix(M, dtype, m, w):
    npdt = np.float64 if dtype == "f64" else np.float32
    a = shuffled_dominant(m * 7 + w, m, npdt)
    ld = (m + 3) // 4 * 4
    both = torch.zeros((2, m, ld), dtype=dev(a).dtype, device="cuda")
    lower, upper_t = both[0, :, :m], both[1, :, :m]
    lower.copy_(dev(a))
    upper_t.copy_(dev(np.ascontiguousarray(a.T)))
    d = torch.zeros(w, dtype=lower.dtype, device="cuda")
    dinv = torch.zeros_like(d)
    perm = torch.full((w,), -1, dtype=torch.int32, device="cuda")
    flags = torch.zeros(4 + 2048, dtype=torch.int64, device="cuda")
    flags[:2] = -1
    M.mdet_step_panel_factor_general(lower, upper_t, w, d, dinv, perm, flags)
    torch.cuda.synchronize()
    assert int(flags[0].item()) == -1
    pw = perm.cpu().numpy().astype(np.int64)
    o = oracle.lu_logdet(a.astype(np.float64), want_LU=True)
    assert o.status == 0 and np.array_equal(pw, o.perm[:w])
    # sign of the row order of these w rows
    assert (-1) ** int(flags[2].item()) == round(np.linalg.det(np.eye(w)[pw]))
    tol = 1e-11 if dtype == "f64" else 2e-4
    dd = d.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(dd - o.diag[:w]) / np.abs(o.diag[:w])) < tol
    assert np.max(np.abs(dinv.cpu().numpy().astype(np.float64) * o.diag[:w] - 1)) < tol
    # L: the stored rows of a group are in input order for the columns left of the group
    got = lower.cpu().numpy().astype(np.float64)
    for g0 in range(GROUP, m, GROUP):
        g1 = min(m, g0 + GROUP)
        left = min(g0, w)
        got[g0:g1, :left] = got[o.perm[g0:g1], :left]
    i, j = np.indices((m, w))
    assert np.max(np.abs(got[:, :w] - o.LU[:, :w])[i > j], initial=0.0) < tol
    assert np.max(np.abs(np.diag(got)[:w] - o.diag[:w]) / np.abs(o.diag[:w])) < tol
    # U^T: columns of the matrix are not exchanged; U = D U~
    gq = upper_t.cpu().numpy().astype(np.float64)
    want_ut = (o.LU[:w, :] / o.diag[:w, None]).T                     # (m, w): U~[j][i] at [i][j]
    assert np.max(np.abs(gq[:, :w] - want_ut)[i > j], initial=0.0) < tol


@pytest.mark.parametrize("n,bs", [(1, 64), (2, 64), (63, 64), (64, 64), (65, 64), (130, 64), (512, 128),
                                  (1000, 256), (777, 64), (1536, 512), (2048, 1024), (1300, 192)])
def test_shuffled_rows_are_found_again(M, n, bs):
    a = shuffled_dominant(n + bs, n)
    res, perm, d, _ = run_device(M, a, bs)
    check_against_oracle(a, perm, d, res, want_equal_perm=True)
    # every pivot is one of the large entries
    assert np.min(np.abs(d)) > 2.0


@pytest.mark.parametrize("n,bs", [(64, 64), (200, 64), (640, 128), (1100, 192), (2048, 512)])
def test_unstructured_matrix(M, n, bs):
    a = gaussian(n * 3 + bs, n)
    res, perm, d, _ = run_device(M, a, bs)
    check_against_oracle(a, perm, d, res)
    sg, lad = np.linalg.slogdet(a)
    assert res.sign == sg and rel(res.logabsdet, lad) <= 1e-9


def test_transpose_has_the_same_determinant(M):
    a = gaussian(77, 900)
    r0, _, _, _ = run_device(M, a, 128)
    r1, _, _, _ = run_device(M, np.ascontiguousarray(a.T), 128)
    assert r0.sign == r1.sign and rel(r0.logabsdet, r1.logabsdet) <= 1e-10


def test_stored_factors_reconstruct_the_matrix_and_match_the_oracle(M):
    n, bs = 600, 128
    a = shuffled_dominant(11, n)
    res, perm, d, ad = run_device(M, a, bs, overwrite=True)
    s = ad.cpu().numpy()
    L, U = stored_factors(s, perm)
    rec = L @ np.diag(d) @ U
    assert np.max(np.abs(rec - a[perm])) <= 1e-12 * np.max(np.abs(L)) * np.max(np.abs(d)) * np.max(np.abs(U)) * n
    assert np.array_equal(np.diag(s), d)
    o = oracle.lu_logdet(a, want_LU=True)
    assert np.array_equal(o.perm, perm)
    assert np.max(np.abs(np.tril(o.LU, -1) - np.tril(L, -1))) <= 1e-12
    assert np.max(np.abs(np.triu(o.LU) - np.diag(d) @ U)) <= 1e-11
    assert np.max(np.abs(o.diag - d) / np.abs(d)) <= 1e-12


def test_symmetric_positive_definite_input_agrees_with_the_symmetric_path(M):
    w = W.scaled_down(W.config(2), 1536, 256)
    a = w.dense()
    res, perm, d, _ = run_device(M, a, 256)
    check_against_oracle(a, perm, d, res)
    plain = oracle.ldlt_logdet(a)
    sym = M.mdet_logdet_device(dev(a), block_size=256)
    assert res.sign == 1 and rel(res.logabsdet, plain.logabsdet) <= TOL["f64"]
    assert rel(res.logabsdet, sym.logabsdet) <= TOL["f64"]
    # about twice the arithmetic of the symmetric form
    assert 1.7 <= res.flops / sym.flops <= 2.3


def test_permutation_matrices_give_the_sign_of_the_permutation(M):
    rng = np.random.default_rng(4)
    n = 200
    for trial in range(6):
        rows = np.concatenate([g0 + rng.permutation(min(GROUP, n - g0)) for g0 in range(0, n, GROUP)])
        a = np.eye(n)[rows]
        res, perm, d, _ = run_device(M, a, 64)
        o = oracle.lu_logdet(a)
        assert res.status == 0 and res.logabsdet == 0.0 and np.all(d == 1.0)
        assert res.sign == o.sign == round(np.linalg.det(a))
        assert np.array_equal(perm, o.perm)


def test_ties_go_to_the_row_that_came_first_in_the_input(M):
    # step 0 takes row 5; at step 1 rows 0 and 3 tie.  Had rows 0 and 5 changed places,
    # "the first" by position would be row 3: the rule goes by the rows of the input.
    n = 8
    a = np.zeros((n, n))
    a[5, 0] = 4.0
    a[0, 1], a[3, 1] = 2.0, -2.0
    for r, c in [(1, 2), (2, 3), (3, 4), (4, 5), (6, 6), (7, 7)]:
        a[r, c] = 1.0
    res, perm, d, _ = run_device(M, a, 64)
    o = oracle.lu_logdet(a)
    assert perm.tolist() == [5, 0, 1, 2, 3, 4, 6, 7] and np.array_equal(perm, o.perm)
    assert res.sign == o.sign == round(np.sign(np.linalg.det(a))) and rel(res.logabsdet, math.log(8.0)) <= 1e-14
    # and a chain of ties with no exchange at all
    n = 64
    a = np.zeros((n, n))
    for j in range(n):
        a[j, j] = 2.0
        if j + 1 < n:
            a[j + 1, j] = -2.0
    res, perm, d, _ = run_device(M, a, 64)
    assert perm.tolist() == list(range(n)) and res.sign == 1 and rel(res.logabsdet, n * math.log(2.0)) <= 1e-14


def test_fp32(M):
    a = shuffled_dominant(5, 1024, np.float32)
    res, perm, d, _ = run_device(M, a, 256)
    check_against_oracle(a, perm, d, res, dtype="f32", want_equal_perm=True)
    g = gaussian(6, 700, np.float32)
    res, perm, d, _ = run_device(M, g, 128)
    # with no exchanges between groups the entries grow along the elimination of an
    # unstructured matrix, and single pivots late in the order are determined to a few
    # digits only in fp32 (their product is not affected: the errors cancel in it)
    check_against_oracle(g, perm, d, res, dtype="f32", pivots=False)


def test_same_bits_on_one_stream(M):
    a = gaussian(21, 1536)
    r0, p0, d0, _ = run_device(M, a, 256)
    r1, p1, d1, _ = run_device(M, a, 256, flags=M.FLAG_NO_LOOKAHEAD)
    r2, p2, d2, _ = run_device(M, a, 256)
    assert r0.logabsdet == r1.logabsdet == r2.logabsdet and r0.sign == r1.sign == r2.sign
    assert np.array_equal(p0, p1) and np.array_equal(d0, d1) and np.array_equal(d0, d2)


def test_input_is_preserved_without_overwrite_and_strided_input_works(M):
    a = gaussian(31, 500)
    ad = dev(a)
    res = M.mdet_logdet_device(ad, block_size=128, flags=M.FLAG_GENERAL)
    o = oracle.lu_logdet(a)
    assert res.status == 0 and np.array_equal(ad.cpu().numpy(), a)
    assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= TOL["f64"]
    # a view with a leading dimension of its own, worked on in place
    big = torch.full((500, 512), float("nan"), dtype=torch.float64, device="cuda")
    view = big[:, :500]
    view.copy_(dev(a))
    r2 = M.mdet_logdet_device(view, block_size=128, flags=M.FLAG_GENERAL, overwrite=True)
    assert r2.logabsdet == res.logabsdet and r2.sign == res.sign
    assert bool(torch.isnan(big[:, 500:]).all())


def test_singular_and_non_finite_input(M):
    # a column of zeros stays a column of zeros: nothing to take when its turn comes
    for col in (5, 70, 199):
        a = shuffled_dominant(3, 200)
        a[:, col] = 0.0
        o = oracle.lu_logdet(a)
        res = M.mdet_logdet_device(dev(a), block_size=64, flags=M.FLAG_GENERAL)
        assert o.status == 1 and o.bad_pivot_index == col
        assert res.status == M.Status.ESINGULAR and res.bad_pivot_index == col
        assert res.sign == 0 and res.logabsdet == -math.inf
    c = gaussian(10, 150)
    c[70, 3] = np.nan
    rc = M.mdet_logdet_device(dev(c), block_size=64, flags=M.FLAG_GENERAL)
    assert rc.status == M.Status.ENONFINITE


def test_bad_arguments_and_workspace(M):
    a = dev(np.eye(128))
    for extra in (M.FLAG_PIVOT, M.FLAG_ASSUME_SPD):
        with pytest.raises(M.MemdetError) as e:
            M.mdet_logdet_device(a, block_size=64, flags=M.FLAG_GENERAL | extra)
        assert e.value.status == M.Status.EINVAL
    with pytest.raises(M.MemdetError) as e:
        M.mdet_logdet_device(dev(np.eye(128, dtype=np.float32)), block_size=64,
                             flags=M.FLAG_GENERAL | M.FLAG_COMPUTE_F64)
    assert e.value.status == M.Status.EINVAL
    # the workspace grows by the transposed upper triangle and the permutation
    plain, _ = M.mdet_workspace_query(4096, "f64", 512, for_device_input=True)
    gen, _ = M.mdet_workspace_query(4096, "f64", 512, flags=M.FLAG_GENERAL, for_device_input=True)
    assert gen == plain + 4096 * 4096 * 8 + 4096 * 4
    # a budget that has no room for it
    with pytest.raises(M.MemdetError) as e:
        M.mdet_logdet_device(dev(np.eye(1024)), block_size=128, flags=M.FLAG_GENERAL, mem_budget=12 << 20)
    assert e.value.status == M.Status.EBUDGET


@pytest.mark.parametrize("n", [8192, 32768])
def test_benchmark_size_against_a_product_of_known_factors(M, n):
    # the sizes bench.py --general times: A = (rows shuffled inside groups of 64) of L0 U0 with
    # a unit lower L0 of small entries and an upper U0 with a known diagonal:
    # log|det A| = sum log|diag U0| up to the conditioning of the product
    g = torch.Generator(device="cuda").manual_seed(5)
    L0 = torch.tril(torch.randn((n, n), generator=g, device="cuda", dtype=torch.float64), -1) / (2.0 * math.sqrt(n))
    L0 += torch.eye(n, device="cuda", dtype=torch.float64)
    U0 = torch.triu(torch.randn((n, n), generator=g, device="cuda", dtype=torch.float64), 1) / (2.0 * math.sqrt(n))
    du = (torch.rand(n, generator=g, device="cuda", dtype=torch.float64) * 4.0 + 4.0)
    du = du * (torch.randint(0, 2, (n,), generator=g, device="cuda").to(torch.float64) * 2.0 - 1.0)
    U0 += torch.diag(du)
    a = L0 @ U0
    rng = np.random.default_rng(6)
    rows = np.concatenate([g0 + rng.permutation(GROUP) for g0 in range(0, n, GROUP)])
    a = a[torch.from_numpy(rows).cuda()].contiguous()
    want = float(torch.sum(torch.log(torch.abs(du))).item())
    sg_perm = round(np.linalg.det(np.eye(GROUP)[rows[:GROUP]]))
    for g0 in range(GROUP, n, GROUP):
        sg_perm *= round(np.linalg.det(np.eye(GROUP)[rows[g0:g0 + GROUP] - g0]))
    want_sign = sg_perm * int(torch.prod(torch.sign(du)).item())
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    res = M.mdet_logdet_device(a, flags=M.FLAG_GENERAL, perm=perm)
    assert res.status == 0 and res.sign == want_sign
    assert rel(res.logabsdet, want) <= 1e-10
    p = perm.cpu().numpy().astype(np.int64)
    assert sorted(p.tolist()) == list(range(n)) and np.array_equal(p // GROUP, np.arange(n) // GROUP)
    # sampled outputs the oracle can compute: the first group's pivots depend on the first
    # 64 rows alone (up to the rows' order), so the oracle on the leading 64 x 64 block gives them
    diag = torch.empty(n, dtype=torch.float64, device="cuda")
    M.mdet_logdet_device(a, flags=M.FLAG_GENERAL, diag=diag)
    o = oracle.lu_logdet(a[:GROUP, :GROUP].cpu().numpy())
    assert np.max(np.abs(diag[:GROUP].cpu().numpy() - o.diag) / np.abs(o.diag)) <= 1e-10
    assert np.array_equal(p[:GROUP], o.perm)


def test_empty_matrix_unaligned_views_and_two_callers(M):
    import threading
    r = M.mdet_logdet_device(torch.empty((0, 0), dtype=torch.float64, device="cuda"), flags=M.FLAG_GENERAL)
    assert r.status == 0 and r.logabsdet == 0.0 and r.sign == 1
    # views whose rows are not 16-byte aligned are factored in a copy even with overwrite = 1;
    # block sizes are rounded up to multiples of 64
    for n, bs, dt in [(130, 100, np.float64), (500, 0, np.float32), (257, 64, np.float32)]:
        a = gaussian(n + bs, n, dt)
        big = torch.zeros((n, n + 6), dtype=dev(a).dtype, device="cuda")
        v = big[:, :n]
        v.copy_(dev(a))
        r0 = M.mdet_logdet_device(v, block_size=bs, flags=M.FLAG_GENERAL)
        assert np.array_equal(v.cpu().numpy(), a)
        r1 = M.mdet_logdet_device(v, block_size=bs, flags=M.FLAG_GENERAL, overwrite=True)
        o = oracle.lu_logdet(a.astype(np.float64))
        assert r0.status == r1.status == 0 and r0.logabsdet == r1.logabsdet and r0.sign == r1.sign == o.sign
        assert rel(r0.logabsdet, o.logabsdet) <= TOL["f64" if dt is np.float64 else "f32"]
    # two host threads on one device: calls are serialised inside the library
    a = gaussian(15, 1500)
    ad = dev(a)
    o = oracle.lu_logdet(a)
    out = [None, None]

    def work(i):
        for _ in range(4):
            out[i] = M.mdet_logdet_device(ad, block_size=256, flags=M.FLAG_GENERAL)
    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert out[0].logabsdet == out[1].logabsdet and out[0].sign == out[1].sign == o.sign
    assert rel(out[0].logabsdet, o.logabsdet) <= TOL["f64"]


# ---------------------------------------------------------------------------
# the memory-constrained generic case (Alg. 1): the matrix in host memory or a file, under a budget
# ---------------------------------------------------------------------------
def min_budget_general(M, n, dtype, bs):
    lo, hi = 0, 1 << 40
    while hi - lo > 4096:
        mid = (lo + hi) // 2
        try:
            M.mdet_plan(n, dtype, bs, mid, flags=M.FLAG_GENERAL | M.FLAG_FORCE_OUT_OF_CORE)
            hi = mid
        except M.MemdetError:
            lo = mid
    return hi


@pytest.mark.parametrize("kind,n,bs,dtype", [("dominant", 1024, 128, "f64"), ("dominant", 1100, 192, "f64"),
                                             ("gaussian", 1280, 256, "f64"), ("dominant", 777, 64, "f64"),
                                             ("dominant", 1500, 256, "f32")])
def test_general_matrix_from_host_memory_in_core_and_streamed(M, kind, n, bs, dtype):
    npdt = np.float64 if dtype == "f64" else np.float32
    a = (shuffled_dominant(n + bs, n, npdt) if kind == "dominant" else gaussian(n + bs, n, npdt))
    o = oracle.lu_logdet(a.astype(np.float64) if dtype == "f64" else a)
    ref, pref, dref, _ = run_device(M, a, bs)
    assert ref.sign == o.sign and rel(ref.logabsdet, o.logabsdet) <= TOL[dtype]
    G = M.FLAG_GENERAL
    h = M.pack_general_block_columns(torch.from_numpy(a), bs, pin=True)
    keep = h.clone()
    tdt = torch.float64 if dtype == "f64" else torch.float32
    d = torch.empty(n, dtype=tdt)
    perm = torch.full((n,), -1, dtype=torch.int32)
    r0 = M.mdet_logdet_host(h.clone(), n, bs, flags=G, diag=d, perm=perm)
    assert not r0.out_of_core and r0.status == 0
    # the same arithmetic as the resident device run: same bits, same row order
    assert r0.logabsdet == ref.logabsdet and r0.sign == ref.sign
    assert np.array_equal(d.numpy().astype(np.float64), dref) and np.array_equal(perm.numpy().astype(np.int64), pref)
    assert r0.bytes_h2d == M.mdet_plan(n, dtype, bs, flags=G).stream_bytes_h2d == h.numel() * h.element_size()
    lo = min_budget_general(M, n, dtype, bs)
    full = M.mdet_plan(n, dtype, bs, flags=G).dev_bytes_needed
    groups = set()
    for budget in (lo, (lo + full) // 2, int(lo * 1.3)):
        plan = M.mdet_plan(n, dtype, bs, budget, overwrite=False, flags=G | M.FLAG_FORCE_OUT_OF_CORE)
        assert plan.host_bytes_needed == h.numel() * h.element_size()
        d2 = torch.empty(n, dtype=tdt)
        p2 = torch.full((n,), -1, dtype=torch.int32)
        res = M.mdet_logdet_host(h, n, bs, mem_budget=budget, overwrite=False, flags=G | M.FLAG_FORCE_OUT_OF_CORE,
                                 diag=d2, perm=p2)
        assert res.out_of_core and res.status == 0 and res.dev_bytes_high_water <= budget
        assert res.logabsdet == r0.logabsdet and res.sign == r0.sign
        assert torch.equal(d2, d) and torch.equal(p2, perm)
        assert (res.bytes_h2d, res.num_superpanels) == (plan.stream_bytes_h2d, plan.num_superpanels)
        assert res.flops == pytest.approx(2 * 2 * (n ** 3 - n) / 6, rel=1e-12)
        assert torch.equal(h, keep)                       # overwrite = 0: the input stays as it is
        groups.add(res.num_superpanels)
    assert max(groups) >= 3
    # in place: the layouts end up holding L, D and U^T of the streamed groups
    hw = h.clone()
    res = M.mdet_logdet_host(hw, n, bs, mem_budget=lo, flags=G | M.FLAG_FORCE_OUT_OF_CORE)
    assert res.logabsdet == r0.logabsdet and not torch.equal(hw, keep)
    first_diag = hw[:bs * bs].view(bs, bs).diagonal() if n >= bs else None
    if first_diag is not None:
        assert np.array_equal(first_diag.numpy(), d.numpy()[:bs])          # D on the diagonal of the first layout


@pytest.mark.parametrize("n,bs,store", [(1100, 192, "f64"), (777, 64, "f64"), (1280, 256, "f32"), (130, 64, "f64")])
def test_general_matrix_through_the_block_provider(M, n, bs, store):
    # every block of the matrix, of both triangles, is asked for once; the result is that of the same
    # matrix handed over in host memory, bit for bit, resident and streamed
    import ctypes
    name = store
    npdt = np.float64 if name == "f64" else np.float32
    a = shuffled_dominant(n + 3, n, npdt)
    stored = torch.from_numpy(a)
    G = M.FLAG_GENERAL
    h = M.pack_general_block_columns(stored, bs)
    ddt = stored.dtype
    d0 = torch.empty(n, dtype=ddt)
    p0 = torch.full((n,), -1, dtype=torch.int32)
    ref = M.mdet_logdet_host(h.clone(), n, bs, flags=G, diag=d0, perm=p0)
    o = oracle.lu_logdet(a)
    assert ref.sign == o.sign and rel(ref.logabsdet, o.logabsdet) <= TOL[name]
    esize = stored.element_size()
    raw = stored.contiguous().view(torch.uint8).numpy().reshape(n, n * esize)
    calls = []

    def provider(bi, bj, rows, cols, dst, ld):
        calls.append((bi, bj))
        buf = (ctypes.c_uint8 * (rows * ld * esize)).from_address(dst)
        view = np.frombuffer(buf, dtype=np.uint8).reshape(rows, ld * esize)
        view[:, :cols * esize] = raw[bi * bs:bi * bs + rows, bj * bs * esize:(bj * bs + cols) * esize]
        return 0

    T = (n + bs - 1) // bs
    lo = min_budget_general(M, n, name, bs)
    for budget in (0, lo, int(lo * 1.4)):
        calls.clear()
        d1 = torch.empty(n, dtype=ddt)
        p1 = torch.full((n,), -1, dtype=torch.int32)
        fl = G | (M.FLAG_FORCE_OUT_OF_CORE if budget else 0)
        res = M.mdet_logdet_provider(provider, n, name, bs, mem_budget=budget, flags=fl, diag=d1, perm=p1)
        assert res.status == 0 and res.out_of_core == bool(budget)
        assert sorted(calls) == [(i, j) for i in range(T) for j in range(T)]          # each block exactly once
        assert res.logabsdet == ref.logabsdet and res.sign == ref.sign
        assert torch.equal(d1, d0) and torch.equal(p1, p0)
        if budget:
            assert res.dev_bytes_high_water <= budget
    bad = M.mdet_logdet_provider(lambda bi, bj, *rest: 7 if bj > bi else 0, n, name, bs, flags=G, raise_on_error=False)
    assert bad.status == M.Status.EPROVIDER


def test_general_matrix_in_a_file_and_error_paths(M, tmp_path):
    n, bs = 1100, 192
    a = shuffled_dominant(33, n)
    o = oracle.lu_logdet(a)
    G = M.FLAG_GENERAL | M.FLAG_FORCE_OUT_OF_CORE
    h = M.pack_general_block_columns(torch.from_numpy(a), bs)
    path, spath = str(tmp_path / "m.bin"), str(tmp_path / "s.bin")
    h.numpy().tofile(path)
    lo = min_budget_general(M, n, "f64", bs)
    ref = M.mdet_logdet_host(h.clone(), n, bs, mem_budget=lo, flags=G)
    perm = torch.full((n,), -1, dtype=torch.int32)
    res = M.mdet_logdet_file(path, n, "f64", bs, mem_budget=lo, overwrite=False, scratch_path=spath, flags=G, perm=perm)
    assert res.out_of_core and res.logabsdet == ref.logabsdet and res.sign == ref.sign == o.sign
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"] and np.array_equal(perm.numpy(), o.perm)
    assert np.array_equal(np.fromfile(path, dtype=np.float64), h.numpy())
    # a file that holds one triangle only is too short
    short = str(tmp_path / "short.bin")
    h.numpy()[: h.numel() // 2].tofile(short)
    bad = M.mdet_logdet_file(short, n, "f64", bs, flags=M.FLAG_GENERAL, raise_on_error=False)
    assert bad.status == M.Status.EIO
    # a zero column: singular at the oracle's index, also when it is met in a streamed group
    z = a.copy()
    z[:, 900] = 0.0
    oz = oracle.lu_logdet(z)
    rz = M.mdet_logdet_host(M.pack_general_block_columns(torch.from_numpy(z), bs), n, bs, mem_budget=lo, flags=G)
    assert rz.status == M.Status.ESINGULAR and rz.sign == 0 == oz.sign and rz.bad_pivot_index == 900
    # budget below two block columns' worth
    with pytest.raises(M.MemdetError) as e:
        M.mdet_logdet_host(h, n, bs, mem_budget=lo - 8192, flags=M.FLAG_GENERAL)
    assert e.value.status == M.Status.EBUDGET
