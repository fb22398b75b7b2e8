"""GPU parity for matrices stored narrower than the arithmetic on the host, provider and file
entry points (App. C, data-precision pipeline: stored in 16 / 32 bits, computed in 64): the
stored bits cross the host link as they are and are widened exactly on the device; the oracle
reads the same bits widened on the CPU.  fp64 bars throughout."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import workloads as W

pytestmark = pytest.mark.gpu
TOL = 1e-10
STORE = {"f32": (torch.float32, 4), "f16": (torch.float16, 2), "bf16": (torch.bfloat16, 2)}


def rel(a, b):
    return abs(a - b) / max(1.0, abs(b))


@pytest.fixture(scope="module")
def M():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_04424_amd as m
    m.load()
    return m


def stored_matrix(n, store, cfg=1):
    """A configuration's matrix rounded to the storage type (well conditioned enough that the
    rounded matrix is still far from singular), and the same bits widened to float64."""
    if store == "f32":
        a = W.scaled_down(W.config(cfg), n).dense()
    else:
        rng = np.random.default_rng(n)
        g = rng.standard_normal((n, 2 * n))
        a = g @ g.T / (2 * n) + np.eye(n)
    st = torch.from_numpy(a).to(STORE[store][0])
    return st, st.to(torch.float64).numpy()


def min_budget(M, n, dtype, bs, flags):
    lo, hi = 0, 1 << 40
    while hi - lo > 4096:
        mid = (lo + hi) // 2
        try:
            M.mdet_plan(n, dtype, bs, mid, flags=flags)
            hi = mid
        except M.MemdetError:
            lo = mid
    return hi


@pytest.mark.parametrize("store", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("n,bs", [(1024, 128), (1100, 192), (777, 64)])
def test_narrow_storage_on_the_host_path_in_core_and_streamed(M, store, n, bs):
    st, exact = stored_matrix(n, store)
    o = oracle.ldlt_logdet(exact, want_diag=True)
    F = M.FLAG_COMPUTE_F64
    # the device entry point in the same mode is the reference for "same arithmetic"
    ddev = torch.empty(n, dtype=torch.float64, device="cuda")
    ref = M.mdet_logdet_device(st.cuda(), block_size=bs, flags=F, diag=ddev)
    h = M.pack_lower_block_columns(st, bs, pin=True)
    keep = h.clone()
    d = torch.empty(n, dtype=torch.float64)
    r0 = M.mdet_logdet_host(h, n, bs, flags=F, diag=d)
    assert not r0.out_of_core and r0.status == 0 and r0.sign == o.sign
    assert rel(r0.logabsdet, o.logabsdet) <= TOL
    assert np.max(np.abs(d.numpy() - o.diag) / np.abs(o.diag)) <= 1e-9
    assert r0.logabsdet == ref.logabsdet and torch.equal(d, ddev.cpu())
    plan0 = M.mdet_plan(n, store, bs, flags=F)
    assert r0.bytes_h2d == plan0.stream_bytes_h2d == plan0.host_matrix_bytes // 8 * STORE[store][1]
    # streamed: three budgets, several groups; the originals still cross in the stored width
    FO = F | M.FLAG_FORCE_OUT_OF_CORE
    lo = min_budget(M, n, store, bs, FO)
    full = plan0.dev_bytes_needed
    groups = set()
    for budget in (lo, (lo + full) // 2, int(lo * 1.3)):
        plan = M.mdet_plan(n, store, bs, budget, flags=FO)
        scratch = torch.empty(plan.host_bytes_needed // 8, dtype=torch.float64, pin_memory=True)
        d2 = torch.empty(n, dtype=torch.float64)
        res = M.mdet_logdet_host(h, n, bs, mem_budget=budget, flags=FO, diag=d2, host_scratch=scratch)
        assert res.out_of_core and res.status == 0 and res.dev_bytes_high_water <= budget
        assert res.logabsdet == r0.logabsdet and res.sign == r0.sign and torch.equal(d2, d)
        assert (res.bytes_h2d, res.num_superpanels) == (plan.stream_bytes_h2d, plan.num_superpanels)
        groups.add(res.num_superpanels)
        assert torch.equal(h.view(torch.uint8), keep.view(torch.uint8))     # the stored matrix is never written
    assert max(groups) >= 3
    # scratch of the library's own, ordinary (pageable) source memory
    hp = M.pack_lower_block_columns(st, bs, pin=False)
    res = M.mdet_logdet_host(hp, n, bs, mem_budget=lo, flags=FO)
    assert res.out_of_core and res.logabsdet == r0.logabsdet
    # a scratch area that is too small is refused
    small = torch.empty(16, dtype=torch.float64, pin_memory=True)
    bad = M.mdet_logdet_host(h, n, bs, mem_budget=lo, flags=FO, host_scratch=small, raise_on_error=False)
    assert bad.status == M.Status.ENOMEM_HOST


def test_narrow_storage_ill_conditioned_input_meets_the_fp64_bar(M):
    # the NTK-shaped configuration scaled down, stored in fp32: pure fp32 arithmetic cannot do
    # it (Sec. 2.1), fp64 arithmetic on the same bits can, also streamed
    n, bs = 1280, 128
    w = W.scaled_down(W.config(3), n, bs)
    w.dtype = "f32"
    a = w.dense()
    o = oracle.ldlt_logdet(a)
    FO = M.FLAG_COMPUTE_F64 | M.FLAG_FORCE_OUT_OF_CORE
    lo = min_budget(M, n, "f32", bs, FO)
    res = M.mdet_logdet_host(M.pack_lower_block_columns(torch.from_numpy(a), bs, pin=True), n, bs,
                             mem_budget=lo, flags=FO)
    assert res.out_of_core and res.num_superpanels >= 3
    assert res.sign == o.sign == 1 and res.negative_pivots == 0 and rel(res.logabsdet, o.logabsdet) <= TOL


@pytest.mark.parametrize("store", ["f32", "bf16"])
def test_narrow_storage_in_a_file(M, tmp_path, store):
    n, bs = 1500, 192
    st, exact = stored_matrix(n, store)
    o = oracle.ldlt_logdet(exact)
    h = M.pack_lower_block_columns(st, bs, pin=False)
    path, spath = str(tmp_path / "m.bin"), str(tmp_path / "s.bin")
    raw = h.view(torch.uint8).numpy()
    raw.tofile(path)
    FO = M.FLAG_COMPUTE_F64 | M.FLAG_FORCE_OUT_OF_CORE
    lo = min_budget(M, n, store, bs, FO)
    ref = M.mdet_logdet_host(h, n, bs, mem_budget=lo, flags=FO)
    d = torch.empty(n, dtype=torch.float64)
    res = M.mdet_logdet_file(path, n, store, bs, mem_budget=lo, overwrite=True, scratch_path=spath, flags=FO, diag=d)
    assert res.out_of_core and res.logabsdet == ref.logabsdet and rel(res.logabsdet, o.logabsdet) <= TOL
    assert res.bytes_h2d == ref.bytes_h2d and res.bytes_d2h == ref.bytes_d2h
    assert np.array_equal(np.fromfile(path, dtype=np.uint8), raw)          # never written, whatever overwrite says
    # streams and has nowhere to put fp64 factors
    bad = M.mdet_logdet_file(path, n, store, bs, mem_budget=lo, overwrite=True, flags=FO, raise_on_error=False)
    assert bad.status == M.Status.EINVAL
    # everything resident: no scratch needed
    res = M.mdet_logdet_file(path, n, store, bs, flags=M.FLAG_COMPUTE_F64)
    assert not res.out_of_core and res.logabsdet == ref.logabsdet
    # a file of the fp64 layout's length in fp32 elements is long enough, half of it is not
    open(str(tmp_path / "short.bin"), "wb").write(raw[: raw.size // 2].tobytes())
    bad = M.mdet_logdet_file(str(tmp_path / "short.bin"), n, store, bs, flags=M.FLAG_COMPUTE_F64,
                             raise_on_error=False)
    assert bad.status == M.Status.EIO


@pytest.mark.parametrize("store", ["f64", "f32"])
def test_provider_fetches_each_block_once_when_needed(M, store):
    n, bs = 1000, 128
    w = W.scaled_down(W.config(4), n, bs)
    a = w.dense()
    if store == "f32":
        a = a.astype(np.float32)
    exact = a.astype(np.float64)
    o = oracle.ldlt_logdet(exact)
    ctype = ctypes.c_double if store == "f64" else ctypes.c_float
    calls = []

    def provider(bi, bj, rows, cols, dst, ld):
        calls.append((bi, bj))
        buf = (ctype * (rows * ld)).from_address(dst)
        view = np.frombuffer(buf, dtype=a.dtype).reshape(rows, ld)
        view[:, :cols] = a[bi * bs:bi * bs + rows, bj * bs:bj * bs + cols]
        return 0

    T = (n + bs - 1) // bs
    flags = M.FLAG_COMPUTE_F64 if store == "f32" else 0
    lo = min_budget(M, n, store, bs, flags | M.FLAG_FORCE_OUT_OF_CORE)
    href = M.mdet_logdet_host(M.pack_lower_block_columns(torch.from_numpy(a), bs, pin=True), n, bs, flags=flags)
    for budget, fl in ((0, flags), (lo, flags | M.FLAG_FORCE_OUT_OF_CORE), (lo * 2, flags | M.FLAG_FORCE_OUT_OF_CORE)):
        calls.clear()
        res = M.mdet_logdet_provider(provider, n, store, bs, mem_budget=budget, flags=fl)
        assert sorted(calls) == sorted((i, j) for j in range(T) for i in range(j, T))     # each exactly once
        assert res.status == 0 and res.out_of_core == bool(budget)
        assert res.logabsdet == href.logabsdet and rel(res.logabsdet, o.logabsdet) <= TOL
        assert res.bytes_h2d >= href.bytes_h2d
    # a provider that fails part-way through a streamed run
    count = [0]

    def flaky(bi, bj, rows, cols, dst, ld):
        count[0] += 1
        return 0 if count[0] < 12 else 3
    bad = M.mdet_logdet_provider(flaky, n, store, bs, mem_budget=lo, flags=flags | M.FLAG_FORCE_OUT_OF_CORE,
                                 raise_on_error=False)
    assert bad.status == M.Status.EPROVIDER


def test_profile_covers_both_trailing_update_kernels_and_calibration_kernels_run(M):
    # MDET_FLAG_PROFILE: launches, summed durations and flops per kernel, and the union of the
    # launches' intervals, which can only be shorter than the sum
    n, bs = 8192, 1024
    w = W.scaled_down(W.config(2), n, bs)
    f = w.factor_torch("cuda")
    a = w.block_torch(f, 0, n, 0, n, device="cuda")
    res = M.mdet_logdet_device(a, block_size=bs, overwrite=True, flags=M.FLAG_PROFILE)
    assert res.trailing_update_launches > 0 and res.trailing_update64_launches > 0
    total = res.t_trailing_update + res.t_trailing_update64
    assert 0 < res.t_trailing_update_busy <= total * (1 + 1e-6) + 1e-5
    assert res.t_trailing_update_busy <= res.t_total
    # together the two kernels do all the Schur updates by whole block columns: block column k
    # updates the lower triangle of order m_k = n - (k + 1) b with K = b
    T = n // bs
    got = res.trailing_update_flops + res.trailing_update64_flops
    assert got == pytest.approx(2 * sum(bs * (n - (k + 1) * bs) * (n - (k + 1) * bs + 1) / 2 for k in range(T - 1)),
                                rel=1e-9)
    # the measuring sticks: a copy that copies, a register-only loop that reports its flops
    src = torch.arange(1 << 20, dtype=torch.float64, device="cuda")
    dst = torch.zeros_like(src)
    M.mdet_step_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    out = torch.empty(65536, dtype=torch.float64, device="cuda")
    for nacc in (4, 16):
        flop = M.mdet_step_mfma_peak("f64", 256, 10, out, accumulators=nacc)
        torch.cuda.synchronize()
        assert flop == 256 * 4 * 10 * 16 * 2048
