"""Full-size checks of the benchmark configurations 3, 4 and 5, in the launch configuration
bench.py times (minutes of GPU time, up to ~150 GiB of host memory).  Each test is skipped
only on a probed fact: not enough available host memory or free device memory for its matrix.

No full-size long-double oracle run is feasible for these orders (hours to days of CPU time),
so each result is pinned by what is: the oracle on a leading principal block (the partial sums
of log|d_j| are the log-determinants of the leading blocks, Sec. 2.1), the low-rank-plus-shift
determinant identity evaluated with the oracle on the small p x p problem, the KMS closed
form, and agreement between block sizes, budgets, and in-core and streamed runs (App. E.3).
"""
import math
import time

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import workloads as W

pytestmark = [pytest.mark.gpu, pytest.mark.full]

GIB = 1 << 30


def rel(a, b):
    return abs(a - b) / max(1.0, abs(b))


def host_available_gib():
    for line in open("/proc/meminfo"):
        if line.startswith("MemAvailable:"):
            return int(line.split()[1]) / (1 << 20)
    return 0.0


def need(host_gib=0.0, device_gib=0.0):
    """Skip on a probed shortage of memory, and say which."""
    have = host_available_gib()
    if have < host_gib:
        pytest.skip(f"host MemAvailable {have:.0f} GiB < {host_gib:.0f} GiB needed for this configuration's matrix")
    free, _ = torch.cuda.mem_get_info()
    if free / GIB < device_gib:
        pytest.skip(f"free device memory {free / GIB:.0f} GiB < {device_gib:.0f} GiB needed")


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import bench
    import paper_2503_04424_amd as M
    M.load()
    return M, bench


@pytest.fixture
def say(capsys):
    """Progress lines that reach the terminal while the test runs (these tests take a while)."""
    t0 = time.perf_counter()

    def _say(msg):
        with capsys.disabled():
            print(f"\n  [full-size {time.perf_counter() - t0:6.1f}s] {msg}", end="", flush=True)
    return _say


def sylvester_rhs(w):
    """(n-p) log(shift) + logdet(F^T F / p + shift I_p), the p x p part by the oracle."""
    f = w.factor()
    small = f.T @ f / w.p + w.shift * np.eye(w.p)
    o = oracle.ldlt_logdet(small)
    assert o.sign == 1
    return (w.n - w.p) * math.log(w.shift) + o.logabsdet


def test_config3_fp64_in_core_against_low_rank_identity(env, say):
    M, bench = env
    need(host_gib=8, device_gib=30)
    w = W.config(3)
    a = bench.form_matrix_device(w, torch)
    keep = a.clone()
    diag = torch.empty(w.n, dtype=a.dtype, device="cuda")
    lead = a[:4096, :4096].cpu().numpy()
    res = M.mdet_logdet_device(a, block_size=w.block_size, overwrite=True, diag=diag)
    say(f"cfg3 fp64: logdet={res.logabsdet:.10f} t={res.t_total:.3f}s; oracle on the p x p problem ...")
    rhs = sylvester_rhs(w)
    say(f"identity={rhs:.10f} rel={rel(res.logabsdet, rhs):.2e}")
    assert res.sign == 1 and res.negative_pivots == 0
    assert rel(res.logabsdet, rhs) <= 1e-10
    o = oracle.ldlt_logdet(lead)
    part = float(torch.log(diag[:4096].abs()).sum().item())
    assert rel(part, o.logabsdet) <= 1e-10
    # the result does not depend on the blocking (App. E.3: 1e-12 ... 1e-16 across n_b)
    for bs in (1024, 4096):
        a.copy_(keep)
        r2 = M.mdet_logdet_device(a, block_size=bs, overwrite=True)
        say(f"block size {bs}: rel diff {rel(r2.logabsdet, res.logabsdet):.2e}")
        assert r2.sign == 1 and rel(r2.logabsdet, res.logabsdet) <= 1e-12


def test_config3_fp32_storage_fp64_arithmetic(env, say):
    """Configuration 3 stored in fp32, computed in fp64 (App. C: whatever the storage precision,
    the log-determinant is computed in 64 bits): sign +1, no negative pivot, the fp64 bar against
    the oracle on the same fp32 bits (leading block), invariant to the block size."""
    M, bench = env
    need(host_gib=8, device_gib=30)
    w = W.config(3, "f32")
    a = bench.form_matrix_device(w, torch)
    diag = torch.empty(w.n, dtype=torch.float64, device="cuda")
    res = M.mdet_logdet_device(a, block_size=w.block_size, flags=M.FLAG_COMPUTE_F64, diag=diag)
    say(f"cfg3 fp32 storage / fp64 arithmetic: logdet={res.logabsdet:.8f} sign={res.sign} "
        f"negative_pivots={res.negative_pivots} t={res.t_total:.3f}s")
    assert res.status == 0 and res.sign == 1 and res.negative_pivots == 0
    m = 6144
    o = oracle.ldlt_logdet(a[:m, :m].cpu().numpy())         # the same fp32 bits, widened exactly
    part = float(torch.log(diag[:m].abs()).sum().item())
    say(f"leading {m} block vs oracle: {rel(part, o.logabsdet):.2e}")
    assert o.sign == 1 and rel(part, o.logabsdet) <= 1e-10
    r2 = M.mdet_logdet_device(a, block_size=4096, flags=M.FLAG_COMPUTE_F64)
    assert rel(r2.logabsdet, res.logabsdet) <= 1e-12
    # the stored matrix streamed from host memory in fp32 under a budget, widened on the device
    h = M.pack_lower_block_columns(a, w.block_size, pin=True)
    r3 = M.mdet_logdet_host(h, w.n, w.block_size, mem_budget=3 * GIB, flags=M.FLAG_COMPUTE_F64, overwrite=False)
    say(f"streamed in fp32 under 3 GiB: {r3.num_superpanels} groups, h2d {r3.bytes_h2d / 1e9:.1f} GB, "
        f"rel diff {rel(r3.logabsdet, res.logabsdet):.2e}")
    assert r3.out_of_core and r3.dev_bytes_high_water <= 3 * GIB
    assert r3.sign == 1 and rel(r3.logabsdet, res.logabsdet) <= 1e-13


def test_config3_pure_fp32_arithmetic_is_a_recorded_miss(env, say):
    """cond(K) ~ 3e4 / 1e-8 exceeds 1/eps32: Sec. 2.1's warning applies to arithmetic in the
    storage precision.  The run must complete and stay within 1e-3 of the value of the same
    fp32 bits; the 1e-4 bar is expected to be missed and the test records that as xfail."""
    M, bench = env
    need(host_gib=8, device_gib=30)
    w = W.config(3, "f32")
    a = bench.form_matrix_device(w, torch)
    ref = M.mdet_logdet_device(a, block_size=w.block_size, flags=M.FLAG_COMPUTE_F64)
    res = M.mdet_logdet_device(a, block_size=w.block_size, overwrite=True)
    err = rel(res.logabsdet, ref.logabsdet)
    say(f"cfg3 pure fp32: logdet={res.logabsdet:.6f} sign={res.sign} negative_pivots={res.negative_pivots} "
        f"vs fp64 arithmetic on the same bits {ref.logabsdet:.6f}: rel={err:.2e} t={res.t_total:.3f}s")
    assert res.status in (M.Status.OK, M.Status.ESINGULAR, M.Status.ENONFINITE)
    assert err <= 1e-3
    if err > 1e-4 or res.sign != 1:
        pytest.xfail(f"pure fp32 arithmetic on configuration 3: rel {err:.1e}, sign {res.sign}, "
                     f"{res.negative_pivots} negative pivot(s); cond(K) > 1/eps32 (Sec. 2.1)")


def test_config4_streamed_equals_in_core_and_oracle_on_leading_block(env, say):
    M, bench = env
    need(host_gib=85, device_gib=170)
    w = W.config(4)
    say("forming cfg4 in host memory ...")
    h = bench.form_matrix_host_packed(w, torch, M)
    diag = torch.empty(w.n, dtype=h.dtype, pin_memory=True)
    say("streamed run under 16 GiB ...")
    r_ooc = M.mdet_logdet_host(h, w.n, w.block_size, mem_budget=w.mem_budget, overwrite=True, diag=diag)
    del h
    say(f"streamed logdet={r_ooc.logabsdet:.12f} ({r_ooc.t_total:.2f}s, {r_ooc.num_superpanels} groups, "
        f"h2d {r_ooc.bytes_h2d / 1e9:.1f} GB)")
    assert r_ooc.out_of_core and r_ooc.dev_bytes_high_water <= w.mem_budget
    f = w.factor_torch("cuda")
    lead = w.block_torch(f, 0, 4096, 0, 4096, device="cuda").cpu().numpy()
    o = oracle.ldlt_logdet(lead)
    part = float(np.sum(np.log(np.abs(diag[:4096].numpy()))))
    assert rel(part, o.logabsdet) <= 1e-10
    del f, lead
    torch.cuda.empty_cache()
    say("forming cfg4 in HBM ...")
    a = bench.form_matrix_device(w, torch)
    torch.cuda.synchronize()
    diag_in = torch.empty(w.n, dtype=a.dtype, device="cuda")
    r_in = M.mdet_logdet_device(a, block_size=w.block_size, overwrite=True, diag=diag_in)
    say(f"in-core logdet={r_in.logabsdet:.12f} ({r_in.t_total:.2f}s); streamed / in-core time "
        f"{r_ooc.t_total / r_in.t_total:.2f}")
    assert rel(r_ooc.logabsdet, r_in.logabsdet) <= 1e-12
    # every pivot, not only their product: the two schedules do the same arithmetic
    assert torch.equal(diag_in.cpu(), diag)


def test_config5_streamed_against_low_rank_identity(env, say):
    M, bench = env
    need(host_gib=165, device_gib=36)
    w = W.config(5)
    say("forming cfg5 in host memory ...")
    h = bench.form_matrix_host_packed(w, torch, M)
    say("streamed run under 32 GiB ...")
    res = M.mdet_logdet_host(h, w.n, w.block_size, mem_budget=w.mem_budget, overwrite=True)
    del h
    say(f"cfg5: logdet={res.logabsdet:.8f} t={res.t_total:.2f}s groups={res.num_superpanels} "
        f"h2d={res.bytes_h2d / 1e9:.1f} GB planned device bytes={res.dev_bytes_high_water / 2**30:.2f} GiB; "
        "oracle on the p x p problem ...")
    rhs = sylvester_rhs(w)
    say(f"identity={rhs:.8f} rel={rel(res.logabsdet, rhs):.2e}")
    assert res.out_of_core and res.dev_bytes_high_water <= w.mem_budget
    assert res.sign == 1 and rel(res.logabsdet, rhs) <= 1e-10


def test_kms_at_config5_size_against_closed_form(env, say):
    M, bench = env
    need(host_gib=165, device_gib=36)
    c5 = W.config(5)
    k = W.kms(c5.n, 0.9, block_size=c5.block_size, mem_budget=c5.mem_budget)
    say(f"forming KMS rho=0.9 n={k.n} in host memory ...")
    h = bench.form_matrix_host_packed(k, torch, M)
    say("streamed run under 32 GiB ...")
    diag = torch.empty(k.n, dtype=h.dtype, pin_memory=True)
    res = M.mdet_logdet_host(h, k.n, k.block_size, mem_budget=k.mem_budget, overwrite=True, diag=diag)
    cf = k.closed_form_logdet()
    say(f"kms: logdet={res.logabsdet:.8f} closed form={cf:.8f} rel={rel(res.logabsdet, cf):.2e} t={res.t_total:.2f}s")
    assert res.out_of_core and rel(res.logabsdet, cf) <= 1e-10
    # every pivot has a closed form too: d_0 = 1, d_j = 1 - rho^2
    d = diag.numpy()
    assert abs(d[0] - 1.0) <= 1e-14 and np.max(np.abs(d[1:] - (1.0 - 0.81))) <= 1e-12
