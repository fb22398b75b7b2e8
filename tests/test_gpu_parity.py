"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Bars (the benchmark spec): relative error of logdet <= 1e-10 in fp64, <= 1e-4 in fp32,
sign and singular/negative-pivot reporting exact.  Inputs are seeded and formed
on the CPU so both sides read the same bits.
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
    m.load()          # fails loudly if the HIP library is not built
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ---------------------------------------------------------------------------
# single steps
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("M_,N_,K_,lower", [
    (128, 128, 64, False), (256, 128, 128, False), (300, 200, 64, False),
    (1000, 517, 192, False), (64, 64, 64, True), (384, 384, 128, True),
    (777, 333, 64, True), (1, 1, 64, False), (129, 1, 64, True), (2050, 1030, 256, True),
    (2300, 2300, 64, True), (1100, 1500, 64, False),
])
def test_schur_update_against_definition(M, dtype, M_, N_, K_, lower):
    rng = np.random.default_rng(M_ * 7 + N_)
    npdt = np.float64 if dtype == "f64" else np.float32
    a = rng.standard_normal((M_, K_)).astype(npdt)
    b = rng.standard_normal((N_, K_)).astype(npdt)
    d = rng.uniform(0.5, 2.0, K_).astype(npdt) * rng.choice([-1, 1], K_).astype(npdt)
    c = rng.standard_normal((M_, N_)).astype(npdt)
    # definition, in float64 on the same bits
    ref = c.astype(np.float64) - (a.astype(np.float64) * d.astype(np.float64)) @ b.astype(np.float64).T
    cd = dev(c)
    M.mdet_step_schur_update(cd, dev(a), dev(b), dev(d), lower=lower)
    torch.cuda.synchronize()
    got = cd.cpu().numpy().astype(np.float64)
    tol = (1e-13 if dtype == "f64" else 1e-4) * math.sqrt(K_)
    if lower:
        i, j = np.indices((M_, N_))
        low = j <= i
        assert np.max(np.abs(got - ref)[low]) < tol * 10
        # entries above the diagonal are left untouched
        assert np.array_equal(got[~low], c.astype(np.float64)[~low])
    else:
        assert np.max(np.abs(got - ref)) < tol * 10


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("m,w", [(64, 64), (200, 64), (40, 40), (512, 256), (1000, 232), (130, 130)])
def test_panel_factor_matches_oracle_factor(M, dtype, m, w):
    """Block column of an SPD matrix: pivots and every entry of L vs the oracle."""
    wl = W.scaled_down(W.config(1), m)
    wl.dtype = dtype
    a = wl.dense()
    r = oracle.ldlt_logdet(a, want_diag=True, want_L=True)
    # rows must stay 16-byte aligned for the step entry point: pad the leading dimension
    ad = torch.zeros((m, (m + 3) // 4 * 4), dtype=dev(a).dtype, device="cuda")[:, :m]
    ad.copy_(dev(a))
    d = torch.zeros(w, dtype=ad.dtype, device="cuda")
    dinv = torch.zeros_like(d)
    flags = torch.full((2 + 1024,), -1, dtype=torch.int64, device="cuda")
    M.mdet_step_panel_factor(ad, w, d, dinv, flags)
    torch.cuda.synchronize()
    got = ad.cpu().numpy().astype(np.float64)
    tol = 1e-11 if dtype == "f64" else 2e-3
    dd = d.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(dd - r.diag[:w]) / np.abs(r.diag[:w])) < tol
    assert np.max(np.abs(dinv.cpu().numpy().astype(np.float64) * r.diag[:w] - 1)) < tol
    i, j = np.indices((m, w))
    strict = i > j
    assert np.max(np.abs(got[:, :w] - r.L[:, :w])[strict]) < tol
    assert int(flags[0].item()) == -1


# ---------------------------------------------------------------------------
# whole path, device entry point
# ---------------------------------------------------------------------------
def run_device(M, a, bs, **kw):
    ad = dev(a)
    diag = torch.empty(a.shape[0], dtype=ad.dtype, device="cuda")
    res = M.mdet_logdet_device(ad, block_size=bs, diag=diag, **kw)
    return res, diag.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("name,wl", [
    ("cfg1", lambda: W.config(1)),
    ("kms512", lambda: W.kms(512, 0.5, block_size=128)),
    ("cfg2_1536", lambda: W.scaled_down(W.config(2), 1536, 256)),
    ("cfg3_1280", lambda: W.scaled_down(W.config(3), 1280, 192)),
    ("cfg4_1100", lambda: W.scaled_down(W.config(4), 1100, 256)),
    ("cfg5_1024", lambda: W.scaled_down(W.config(5), 1024, 128)),
])
def test_logdet_device_fp64_matches_oracle(M, name, wl):
    w = wl()
    a = w.dense()
    o = oracle.ldlt_logdet(a, want_diag=True)
    res, diag = run_device(M, a, w.block_size)
    assert res.status == 0 and res.sign == o.sign
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]
    assert res.negative_pivots == o.negative_pivots
    # leading principal minors (App. D): running sums of log|d|
    cum = np.cumsum(np.log(np.abs(diag)))
    assert np.max(np.abs(cum - o.cum_logabs) / np.maximum(1, np.abs(o.cum_logabs))) <= TOL["f64"]
    cf = w.closed_form_logdet()
    if cf is not None:
        assert rel(res.logabsdet, cf) <= TOL["f64"]


@pytest.mark.parametrize("name,wl", [
    ("cfg1", lambda: W.config(1)),
    ("kms512", lambda: W.kms(512, 0.5, block_size=128)),
    ("cfg1_2000", lambda: W.scaled_down(W.config(1), 2000, 256)),
])
def test_logdet_device_fp32_matches_oracle_on_same_bits(M, name, wl):
    w = wl()
    w.dtype = "f32"
    a = w.dense()
    assert a.dtype == np.float32
    o = oracle.ldlt_logdet(a)            # oracle reads the fp32 bits exactly
    res, _ = run_device(M, a, w.block_size)
    assert res.status == 0 and res.sign == o.sign
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f32"]


@pytest.mark.parametrize("name,wl", [
    ("cfg1", lambda: W.config(1)),
    ("cfg3_1280", lambda: W.scaled_down(W.config(3), 1280, 192)),
    ("cfg2_1000", lambda: W.scaled_down(W.config(2), 1000, 128)),
])
def test_fp32_storage_with_fp64_arithmetic(M, name, wl):
    """App. C, data-precision pipeline, stage 3: the matrix may be stored in fp32, the
    log-determinant is computed in 64 bit.  Against the oracle on the same fp32 bits the
    fp64 bar applies, also on the ill-conditioned inputs pure fp32 arithmetic cannot do."""
    w = wl()
    w.dtype = "f32"
    a = w.dense()
    o = oracle.ldlt_logdet(a, want_diag=True)
    ad = dev(a)
    before = ad.clone()
    diag = torch.empty(w.n, dtype=torch.float64, device="cuda")
    res = M.mdet_logdet_device(ad, block_size=w.block_size, flags=M.FLAG_COMPUTE_F64, diag=diag,
                               overwrite=True)
    assert res.status == 0 and res.sign == o.sign and res.negative_pivots == o.negative_pivots
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]
    assert torch.equal(ad, before)                      # the fp32 input is never written
    # same bits as the fp64 path on the widened matrix
    r64, d64 = run_device(M, a.astype(np.float64), w.block_size)
    assert r64.logabsdet == res.logabsdet and np.array_equal(d64, diag.cpu().numpy())
    # workspace accounting: the fp64 copy is part of it
    dev_bytes, _ = M.mdet_workspace_query(w.n, "f32", w.block_size, for_device_input=True,
                                          flags=M.FLAG_COMPUTE_F64)
    assert dev_bytes >= w.n * w.n * 8
    # the host entry point in the same mode: the fp32 bits cross the link, the same arithmetic
    packed = M.pack_lower_block_columns(torch.from_numpy(a), w.block_size)
    hres = M.mdet_logdet_host(packed, w.n, w.block_size, flags=M.FLAG_COMPUTE_F64)
    assert hres.logabsdet == res.logabsdet and hres.sign == res.sign


@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 65, 127, 129, 257, 777, 1001])
def test_ragged_and_tiny_orders(M, n):
    if n == 0:
        a = torch.empty((0, 0), dtype=torch.float64, device="cuda")
        res = M.mdet_logdet_device(a, block_size=64)
        assert (res.status, res.sign, res.logabsdet) == (0, 1, 0.0)
        return
    a = W.scaled_down(W.config(1), n).dense()
    o = oracle.ldlt_logdet(a)
    for bs in (64, 128, 320):
        res, _ = run_device(M, a, bs)
        assert res.sign == o.sign and rel(res.logabsdet, o.logabsdet) <= TOL["f64"], (n, bs)


def test_odd_leading_dimension_and_preserved_input(M):
    n = 333
    a = W.scaled_down(W.config(1), n).dense()
    view = torch.zeros((n, 339), dtype=torch.float64, device="cuda")[:, :n]
    view.copy_(torch.from_numpy(a))
    before = view.clone()
    o = oracle.ldlt_logdet(a)
    res = M.mdet_logdet_device(view, block_size=128, overwrite=False)
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]
    assert torch.equal(view, before)
    res = M.mdet_logdet_device(view, block_size=128, overwrite=True)   # misaligned ld: works on a copy
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]


def test_upper_triangle_is_never_read(M):
    n = 300
    a = W.scaled_down(W.config(1), n).dense()
    o = oracle.ldlt_logdet(a)
    b = np.tril(a) + np.triu(np.full((n, n), np.nan), 1)
    res, _ = run_device(M, b, 128)
    assert res.status == 0 and rel(res.logabsdet, o.logabsdet) <= TOL["f64"]


def test_block_size_invariance_and_lookahead_bit_identity(M):
    w = W.scaled_down(W.config(2), 2048, 256)
    a = w.dense()
    o = oracle.ldlt_logdet(a)
    vals = []
    for bs in (64, 128, 256, 512, 1024, 2048):
        res, _ = run_device(M, a, bs)
        assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]
        vals.append(res.logabsdet)
    assert max(vals) - min(vals) <= 1e-10 * abs(o.logabsdet)
    r1, d1 = run_device(M, a, 256)
    r2, d2 = run_device(M, a, 256, flags=M.FLAG_NO_LOOKAHEAD)
    assert r1.logabsdet == r2.logabsdet and np.array_equal(d1, d2)


def test_bulk_update_in_rounds_beside_the_panel_chain(M):
    """Large enough that the bulk of the trailing update is issued as several launches
    that leave part of the device to the next block column's factorisation: same bits
    as the single-stream run, and the KMS closed form (Sec. 4.1-style check)."""
    w = W.kms(4608, 0.7, block_size=256)
    a = torch.from_numpy(w.dense()).cuda()
    r1 = M.mdet_logdet_device(a.clone(), block_size=256, overwrite=True)
    r2 = M.mdet_logdet_device(a.clone(), block_size=256, overwrite=True, flags=M.FLAG_NO_LOOKAHEAD)
    r3 = M.mdet_logdet_device(a.clone(), block_size=512, overwrite=True)
    assert r1.status == 0 and r1.sign == 1
    assert r1.kernel_launches > r2.kernel_launches       # the rounds are extra launches
    assert r1.logabsdet == r2.logabsdet
    exact = w.closed_form_logdet()
    assert rel(r1.logabsdet, exact) <= TOL["f64"] and rel(r3.logabsdet, exact) <= TOL["f64"]


def test_flop_counter_is_tiling_independent(M):
    n = 1000
    a = W.scaled_down(W.config(1), n).dense()
    for bs in (64, 192, 512, 1024):
        res, _ = run_device(M, a, bs)
        assert res.flops == pytest.approx(2 * (n ** 3 - n) / 6, rel=1e-12)
    # leading term of App. E.1's total m^3/6 - m^2/4 + m/12
    assert M.mdet_paper_fma_count(n) == pytest.approx((n ** 3 - n) / 6, rel=2.0 / n)


def test_indefinite_matrix_sign_and_negative_count(M):
    rng = np.random.default_rng(42)
    n = 500
    g = rng.standard_normal((n, n))
    a = g + g.T + np.diag(rng.choice([-40.0, 40.0], n))     # strongly indefinite, safe minors
    o = oracle.ldlt_logdet(a)
    res, _ = run_device(M, a, 128)
    assert o.negative_pivots > 50
    assert (res.sign, res.negative_pivots) == (o.sign, o.negative_pivots)
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]


def test_scaling_identity_on_gpu(M):
    n = 600
    a = W.scaled_down(W.config(1), n).dense()
    base, _ = run_device(M, a, 128)
    for c in (1e-30, 1e25):
        res, _ = run_device(M, c * a, 128)
        assert rel(res.logabsdet, n * math.log(c) + base.logabsdet) <= TOL["f64"]


def test_singular_and_nonfinite_inputs_are_reported(M):
    # Sec. 2.1 example: the stored Gram matrix [[1,1],[1,1]] is exactly singular
    a = np.array([[1.0, 1.0], [1.0, 1.0]])
    res = M.mdet_logdet_device(dev(a), block_size=64)
    assert res.status == M.Status.ESINGULAR and res.sign == 0
    assert res.logabsdet == -math.inf and res.bad_pivot_index == 1
    n = 200
    a = W.scaled_down(W.config(1), n).dense()
    a[150, 150] = np.nan
    res = M.mdet_logdet_device(dev(a), block_size=64)
    assert res.status == M.Status.ENONFINITE and res.bad_pivot_index == 150
    # a zero block later in the matrix: singular at its first column
    a = np.eye(300)
    a[170:, 170:] = 0.0
    res = M.mdet_logdet_device(dev(a), block_size=128)
    assert res.status == M.Status.ESINGULAR and res.bad_pivot_index == 170


def test_budget_is_enforced_for_device_copy(M):
    n = 512
    a = dev(W.config(1).dense())
    with pytest.raises(M.MemdetError) as ei:
        M.mdet_logdet_device(a, block_size=128, overwrite=False, mem_budget=1 << 20)
    assert ei.value.status == M.Status.EBUDGET
    res = M.mdet_logdet_device(a, block_size=128, overwrite=True, mem_budget=1 << 20)
    assert res.status == 0 and res.dev_bytes_high_water <= (1 << 20)


@pytest.mark.parametrize("cfg,n,bs,dtype", [(1, 512, 128, "f64"), (2, 1536, 256, "f64"), (3, 2304, 512, "f64"),
                                            (5, 1100, 192, "f64"), (1, 1000, 64, "f32"), (3, 4608, 1024, "f64")])
def test_scaled_copy_gives_the_same_bits(M, cfg, n, bs, dtype):
    # MDET_FLAG_SCALED_COPY: the updates read W = L D from a second array instead of scaling
    # L on the fly; every product and every sum is the same
    w = W.scaled_down(W.config(cfg, dtype), n, bs)
    a = w.dense().astype(np.float64 if dtype == "f64" else np.float32)
    ref = M.mdet_logdet_device(dev(a), block_size=bs)
    diag = torch.empty(n, dtype=torch.float64 if dtype == "f64" else torch.float32, device="cuda")
    res = M.mdet_logdet_device(dev(a), block_size=bs, flags=M.FLAG_SCALED_COPY, diag=diag)
    assert res.status == 0 and res.logabsdet == ref.logabsdet and res.sign == ref.sign
    plain = M.mdet_plan(n, dtype, bs, overwrite=False, for_device_input=True)
    extra = M.mdet_plan(n, dtype, bs, overwrite=False, for_device_input=True, flags=M.FLAG_SCALED_COPY)
    beta = 8 if dtype == "f64" else 4
    rounded_bs = (bs + 63) // 64 * 64
    assert extra.dev_bytes_needed - plain.dev_bytes_needed == 2 * ((n * rounded_bs * beta + 255) // 256 * 256)
    assert res.dev_bytes_high_water == extra.dev_bytes_needed
    # host entry point, everything resident
    h = M.pack_lower_block_columns(torch.from_numpy(a), bs, pin=True)
    hres = M.mdet_logdet_host(h, n, bs, flags=M.FLAG_SCALED_COPY)
    assert hres.logabsdet == ref.logabsdet
    # a budget that has no room for the copies: the flag is ignored, not an error
    tight = M.mdet_logdet_device(dev(a), block_size=bs, flags=M.FLAG_SCALED_COPY,
                                 mem_budget=plain.dev_bytes_needed + 4096)
    assert tight.logabsdet == ref.logabsdet and tight.dev_bytes_high_water == plain.dev_bytes_needed


def test_scaled_copy_is_taken_unasked_for_a_large_uncapped_call_and_dropped_if_memory_is_short(M):
    # no budget and n >= 24576: the plan holds the two arrays of MDET_FLAG_SCALED_COPY by
    # itself; a caller's workspace that has no room for them is not an error; same bits
    n, bs, rho = 24576, 1024, 0.5
    plain_ws, _ = M.mdet_workspace_query(n, "f64", bs, mem_budget=1 << 50, for_device_input=True)
    auto_ws, _ = M.mdet_workspace_query(n, "f64", bs, for_device_input=True)
    assert auto_ws == plain_ws + 2 * n * bs * 8
    idx = torch.arange(n, device="cuda", dtype=torch.float64)
    a = (idx[:, None] - idx[None, :]).abs_()
    a = torch.pow(torch.tensor(rho, dtype=torch.float64, device="cuda"), a, out=a)
    r_auto = M.mdet_logdet_device(a.clone(), block_size=bs, overwrite=True)
    assert r_auto.status == 0 and r_auto.dev_bytes_high_water == auto_ws
    ws = torch.empty(plain_ws, dtype=torch.uint8, device="cuda")
    r_short = M.mdet_logdet_device(a.clone(), block_size=bs, overwrite=True, workspace=ws)
    assert r_short.status == 0 and r_short.dev_bytes_high_water == plain_ws
    assert r_short.logabsdet == r_auto.logabsdet
    closed = (n - 1) * math.log(1 - rho * rho)          # KMS matrix
    assert abs(r_auto.logabsdet - closed) <= 1e-10 * abs(closed)


@pytest.mark.parametrize("store", ["float16", "bfloat16"])
@pytest.mark.parametrize("n,bs", [(600, 128), (1030, 256)])
def test_sixteen_bit_storage_with_fp64_arithmetic(M, store, n, bs):
    # App. C (data-precision pipeline): whatever format the matrix is stored in, the
    # log-determinant is computed in 64 bit.  The library widens the stored bits exactly.
    rng = np.random.default_rng(n)
    g = rng.standard_normal((n, 2 * n))
    a = g @ g.T / (2 * n) + np.eye(n)
    stored = torch.from_numpy(a).to(getattr(torch, store))
    exact = stored.to(torch.float64).numpy()              # the same bits, widened exactly
    o = oracle.ldlt_logdet(exact, want_diag=True)
    diag = torch.empty(n, dtype=torch.float64, device="cuda")
    keep = stored.clone()
    dstored = stored.cuda()
    res = M.mdet_logdet_device(dstored, block_size=bs, flags=M.FLAG_COMPUTE_F64, diag=diag)
    assert res.status == 0 and res.sign == o.sign and res.negative_pivots == o.negative_pivots
    assert rel(res.logabsdet, o.logabsdet) <= TOL["f64"]
    assert np.max(np.abs(diag.cpu().numpy() - o.diag) / np.abs(o.diag)) <= 1e-9
    assert torch.equal(dstored.cpu().view(torch.int16), keep.view(torch.int16))   # input untouched
    # the 16-bit types are storage formats only
    with pytest.raises(M.MemdetError) as e:
        M.mdet_logdet_device(dstored, block_size=bs)
    assert e.value.status == M.Status.EINVAL


def test_concurrent_calls_from_two_threads(M):
    # the header allows concurrent calls with distinct workspaces: two threads, each with
    # its own matrix (device path) or host array (host path, streamed), several calls each;
    # every result must be the bits of the same call made alone
    import threading
    mats = [W.scaled_down(W.config(c), 1200 + 64 * c, 128).dense() for c in (1, 2, 3, 4)]
    alone = [M.mdet_logdet_device(dev(a), block_size=128).logabsdet for a in mats]
    packs = [M.pack_lower_block_columns(torch.from_numpy(a), 128, pin=True) for a in mats]
    budget = 4 * 1500 * 128 * 8
    out, errs = {}, []

    def work(tid):
        try:
            torch.cuda.set_device(0)
            for rep in range(3):
                for i in range(tid, len(mats), 2):
                    r1 = M.mdet_logdet_device(dev(mats[i]), block_size=128)
                    r2 = M.mdet_logdet_host(packs[i].clone(), mats[i].shape[0], 128, mem_budget=budget,
                                            flags=M.FLAG_FORCE_OUT_OF_CORE)
                    out[(tid, rep, i)] = (r1.logabsdet, r2.logabsdet, r1.status, r2.status)
        except Exception as e:           # surfaced below
            errs.append(e)

    ts = [threading.Thread(target=work, args=(t,)) for t in (0, 1)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert not errs and len(out) == 12
    for (tid, rep, i), (l1, l2, s1, s2) in out.items():
        assert s1 == 0 and s2 == 0 and l1 == alone[i] and l2 == alone[i]

