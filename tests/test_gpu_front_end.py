"""The front end with the call shape of the paper's software appendix (memdet(M, max_mem, assume,
triangle, ...)): it only chooses entry point and flags, so it is checked against the oracle and numpy
on small matrices of every form, resident and streamed."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle


def rel(a, b):
    return abs(a - b) / max(1.0, abs(b))


def test_sizes_are_read_as_written():
    from paper_2503_04424_amd.api import parse_bytes
    assert parse_bytes("32GB") == 32 * 10 ** 9 and parse_bytes("16GiB") == 16 * 2 ** 30
    assert parse_bytes(" 1.5 MB ") == 1500000 and parse_bytes(4096) == 4096
    assert parse_bytes(None) == 0 and parse_bytes(float("inf")) == 0
    with pytest.raises(ValueError):
        parse_bytes("12 parsecs")


def test_arguments_are_checked_before_anything_runs():
    from paper_2503_04424_amd.api import memdet, FitLogdet
    with pytest.raises(ValueError):
        memdet(np.zeros((3, 4)))
    with pytest.raises(ValueError):
        memdet(np.eye(4), assume="lower")
    with pytest.raises(ValueError):
        memdet(np.eye(4), assume="sym", triangle="x")
    with pytest.raises(ValueError):
        memdet(np.eye(4), assume="gen", pivot="leaf")
    with pytest.raises(ValueError):
        memdet(np.eye(4), assume="sym", mixed_precision="float16")
    with pytest.raises(ValueError):
        FitLogdet(q=2).eval([10.0])


@pytest.fixture(scope="module")
def M():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_04424_amd as m
    m.load()
    return m


def spd_matrix(seed, n):
    g = np.random.default_rng(seed)
    x = g.standard_normal((n, n // 2 + 3))
    return x @ x.T / x.shape[1] + np.diag(0.5 + g.random(n))


@pytest.mark.gpu
def test_symmetric_forms_resident_and_streamed(M):
    n = 900
    a = spd_matrix(1, n)
    o = oracle.ldlt_logdet(a, want_diag=True)
    # resident on the device, lower triangle
    ld, sign, diag, perm = M.memdet(torch.from_numpy(a).cuda(), assume="sym", block_size=128)
    assert sign == o.sign == 1 and rel(ld, o.logabsdet) <= 1e-10
    assert np.allclose(diag, o.diag, rtol=1e-9) and np.array_equal(perm, np.arange(n))
    # only the upper triangle filled, the rest poisoned
    up = np.triu(a) + np.tril(np.full((n, n), np.nan), -1)
    ld_u, sign_u, diag_u, _ = M.memdet(torch.from_numpy(up).cuda(), assume="sym", triangle="u", block_size=128)
    assert ld_u == ld and sign_u == 1 and np.array_equal(diag_u, diag)
    # from host memory under a cap that forces streaming, with the information record
    lo = None
    for cap in range(1 << 20, 64 << 20, 1 << 19):
        try:
            if M.mdet_plan(n, "f64", 128, cap).out_of_core:
                lo = cap
                break
        except M.MemdetError:
            continue
    assert lo is not None
    ld_h, sign_h, diag_h, _, info = M.memdet(a, max_mem=f"{lo / 1e6:.3f}MB", assume="sym", block_size=128,
                                             return_info=True)
    assert info["out_of_core"] and info["dev_bytes_high_water"] <= lo
    assert ld_h == ld and sign_h == 1 and np.array_equal(diag_h, diag)
    # Cholesky form, and fp64 arithmetic on fp32 storage
    ld_c, sign_c, _, _ = M.memdet(torch.from_numpy(a).cuda(), assume="spd", block_size=128)
    assert sign_c == 1 and rel(ld_c, o.logabsdet) <= 1e-10
    a32 = a.astype(np.float32)
    o32 = oracle.ldlt_logdet(a32.astype(np.float64))
    ld_m, sign_m, diag_m, _ = M.memdet(a32, assume="sym", mixed_precision="float64", block_size=128)
    assert diag_m.dtype == np.float64 and sign_m == 1 and rel(ld_m, o32.logabsdet) <= 1e-10


@pytest.mark.gpu
def test_pivoted_and_general_forms(M):
    n = 640
    g = np.random.default_rng(3)
    x = g.standard_normal((n, n))
    s = (x + x.T) / 40.0 + np.diag(g.uniform(2, 4, n) * g.choice([-1.0, 1.0], n))
    s[0, 0] = 0.0                                              # needs the exchange
    sign_ref, ld_ref = np.linalg.slogdet(s)
    for pivot in ("leaf", "block"):
        ld, sign, diag, perm = M.memdet(torch.from_numpy(s).cuda(), assume="sym", pivot=pivot, block_size=128)
        assert sign == int(sign_ref) and rel(ld, ld_ref) <= 1e-10
        assert sorted(perm.tolist()) == list(range(n)) and perm[0] != 0
        assert rel(np.sum(np.log(np.abs(diag))), ld_ref) <= 1e-10
    a = x / 25.0 + np.diag(g.uniform(2, 4, n))
    sign_ref, ld_ref = np.linalg.slogdet(a)
    for src in (torch.from_numpy(a).cuda(), a):                 # resident, and from host memory
        ld, sign, diag, perm = M.memdet(src, assume="gen", block_size=128)
        assert sign == int(sign_ref) and rel(ld, ld_ref) <= 1e-10 and sorted(perm.tolist()) == list(range(n))
    with pytest.raises(ValueError):
        M.memdet(a, assume="gen", pivot="leaf")
    with pytest.raises(ValueError):
        M.memdet(a, assume="lower")


@pytest.mark.gpu
def test_fit_and_extrapolate_in_the_shape_of_the_appendix(M):
    # the ratio law exact (Assumption 1 of Sec. 3.2): ell_n - ell_{n-1} = log C - nu log n; fitted on
    # n = 1 .. 2000 (Eq. 7 is written relative to L_{n0}; it reproduces the law exactly for n0 = 1), the
    # curve gives ell at n = 20000; and the pivots of a factorisation feed it
    import math
    ell_1, Cc, nu = -0.8, 5.0, 1.7
    k = np.arange(2, 20001, dtype=np.float64)
    ell = np.concatenate([[ell_1], ell_1 + np.cumsum(np.log(Cc) - nu * np.log(k))])     # ell[n - 1]
    n = np.arange(1, 20001)
    mask = (n >= 1) & (n <= 2000)
    f = M.FitLogdet(q=0).fit(n[mask], ell[mask])
    got = f.eval(np.array([5000.0, 20000.0]))
    assert np.max(np.abs(got - ell[[4999, 19999]]) / np.abs(ell[[4999, 19999]])) <= 1e-9
    assert abs(f.parameters[1] - nu) <= 1e-9
    with pytest.raises(ValueError):
        M.FitLogdet(q=1).fit(np.array([1, 2, 4, 5, 6]), np.zeros(5))
    a = spd_matrix(5, 1200)
    ld, sign, diag, perm = M.memdet(torch.from_numpy(a).cuda(), assume="sym", block_size=128)
    cum = np.cumsum(np.log(np.abs(diag)))[3::4]                 # every 4th: orders 1 .. 300 of 4 x 4 blocks
    nn = np.arange(1, cum.size + 1)
    fit = M.FitLogdet(q=1).fit(nn[20:200], cum[20:200])
    from oracle import flodance_oracle as F
    want = F.fit(np.cumsum(np.log(np.abs(diag))), 4, 21, 200, 1)         # the same samples: d = 4, n = 21 .. 200
    ref = want.eval(np.array([300.0]))[0] * 300.0
    assert abs(fit.eval(np.array([300.0]))[0] - ref) <= 1e-7 * abs(ref)

