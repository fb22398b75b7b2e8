"""Seeded random sweep over orders, block sizes, entry points, budgets and flags:
every case against the long-double oracle on the same bits (fp64 bar), and the three
entry points against each other to the last bit."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def rel(a, b):
    return abs(a - b) / max(1.0, abs(b))


@pytest.fixture(scope="module")
def M():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2503_04424_amd as m
    m.load()
    return m


def _min_budget(M, n, bs):
    lo, hi = 0, 1 << 40
    while hi - lo > 4096:
        mid = (lo + hi) // 2
        try:
            M.mdet_plan(n, "f64", bs, mid, flags=M.FLAG_FORCE_OUT_OF_CORE)
            hi = mid
        except M.MemdetError:
            lo = mid
    return hi


CASES = []
_rng = np.random.default_rng(20250304)
for _case in range(36):
    CASES.append((int(_rng.integers(1, 900)), int(_rng.choice([64, 128, 192, 256, 320])),
                  int(_rng.integers(1, 6)), bool(_rng.integers(0, 2)), float(_rng.uniform(1.0, 3.0)),
                  int(_rng.integers(0, 1 << 30))))


@pytest.mark.parametrize("n,bs,cfg,lookahead,budget_factor,seed", CASES)
def test_random_case(M, n, bs, cfg, lookahead, budget_factor, seed):
    w = W.scaled_down(W.config(cfg), n, bs)
    w.seed = seed
    a = w.dense()
    if cfg % 2 == 0 and n > 1:
        # symmetric quasi-definite now and then: [[A11, A12], [A21, -A22]] has an LDL^T
        # without pivoting, n - m negative pivots and a sign to get right
        m = int(np.random.default_rng(seed).integers(1, n))
        a = a.copy()
        a[m:, m:] *= -1.0
    o = oracle.ldlt_logdet(a, want_diag=True)
    if o.status != 0 or np.min(np.abs(o.diag)) < 1e-9 * np.max(np.abs(o.diag)):
        pytest.skip("pivot too small for an unpivoted factorisation to be meaningful")
    flags = 0 if lookahead else M.FLAG_NO_LOOKAHEAD
    dev = M.mdet_logdet_device(torch.from_numpy(a).cuda(), block_size=bs, flags=flags)
    assert dev.status == 0 and dev.sign == o.sign and dev.negative_pivots == o.negative_pivots
    assert rel(dev.logabsdet, o.logabsdet) <= 1e-10
    h = M.pack_lower_block_columns(torch.from_numpy(a), bs, pin=bool(seed & 1))
    host = M.mdet_logdet_host(h.clone(), n, bs, flags=flags)
    assert host.logabsdet == dev.logabsdet and host.sign == dev.sign
    budget = int(_min_budget(M, n, bs) * budget_factor)
    ooc = M.mdet_logdet_host(h, n, bs, mem_budget=budget, flags=flags | M.FLAG_FORCE_OUT_OF_CORE)
    assert ooc.out_of_core and ooc.dev_bytes_high_water <= budget
    assert ooc.logabsdet == dev.logabsdet and ooc.sign == dev.sign
