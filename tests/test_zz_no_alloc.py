"""The allocation-free entry point against mdet_logdet_device: same path, same bits, two calls
in a row on the library's fixed scratch array, the second smaller than the first."""
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


def test_noalloc_entry_point_matches_the_allocating_one_on_two_calls_in_a_row(M):
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    stream = torch.cuda.Stream()
    for n, bs, cfg in ((1500, 256, 1), (778, 128, 2)):         # the second call is the smaller one
        w = W.scaled_down(W.config(cfg), n, bs)
        a = w.dense()
        o = oracle.ldlt_logdet(a, want_diag=True)
        ref_in = torch.from_numpy(a).cuda()
        dref = torch.empty(n, dtype=torch.float64, device="cuda")
        ref = M.mdet_logdet_device(ref_in, block_size=bs, overwrite=True, diag=dref)
        work = torch.from_numpy(a).cuda()
        d = torch.empty(n, dtype=torch.float64, device="cuda")
        out.fill_(-7.0)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            st = M.mdet_logdet_device_noalloc(work, out, block_size=bs, diag=d, stream=stream)
        assert st == M.Status.OK
        stream.synchronize()
        got = out.cpu().numpy()
        assert got[4] == M.Status.OK and got[3] == -1.0
        assert got[0] == ref.logabsdet and int(got[1]) == ref.sign and int(got[2]) == ref.negative_pivots
        assert torch.equal(d, dref) and torch.equal(work, ref_in)         # pivots and the stored factor
        assert int(got[1]) == o.sign and rel(got[0], o.logabsdet) <= 1e-10


def test_noalloc_entry_point_other_forms_and_error_reports(M):
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    # positive-definite form, fp32
    n, bs = 900, 128
    a = W.scaled_down(W.config(1), n, bs).dense().astype(np.float32)
    ref = M.mdet_logdet_device(torch.from_numpy(a).cuda(), block_size=bs, overwrite=True, flags=M.FLAG_ASSUME_SPD)
    assert M.mdet_logdet_device_noalloc(torch.from_numpy(a).cuda(), out, block_size=bs, flags=M.FLAG_ASSUME_SPD) == 0
    torch.cuda.synchronize()
    assert out[0].item() == ref.logabsdet and out[4].item() == 0
    # pivoting: the permutation comes back too
    rng = np.random.default_rng(5)
    g = rng.standard_normal((n, n))
    b = (g + g.T) / 30.0 + np.diag(rng.uniform(4, 8, n) * rng.choice([-1.0, 1.0], n))
    b[0, 0] = 0.0
    pref = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    ref = M.mdet_logdet_device(torch.from_numpy(b).cuda(), block_size=bs, overwrite=True, flags=M.FLAG_PIVOT, perm=pref)
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    assert M.mdet_logdet_device_noalloc(torch.from_numpy(b).cuda(), out, block_size=bs, flags=M.FLAG_PIVOT,
                                        perm=perm) == 0
    torch.cuda.synchronize()
    assert out[0].item() == ref.logabsdet and int(out[1].item()) == ref.sign and torch.equal(perm, pref)
    # a singular matrix: reported through out, as the synchronous entry point reports it
    s = np.eye(300)
    s[200:, 200:] = 0.0
    assert M.mdet_logdet_device_noalloc(torch.from_numpy(s).cuda(), out, block_size=64) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert got[4] == M.Status.ESINGULAR and got[3] == 200 and got[1] == 0 and got[0] == -np.inf
    # what it refuses: a copy (overwrite = 0 is not offered), other forms, sizes beyond the array
    S = M.Status
    assert M.mdet_logdet_device_noalloc(torch.eye(64, dtype=torch.float64, device="cuda"), out,
                                        flags=M.FLAG_GENERAL) == S.EINVAL
    assert M.mdet_logdet_device_noalloc(torch.eye(64, dtype=torch.float64, device="cuda"), out,
                                        flags=M.FLAG_PROFILE) == S.EINVAL
    v = torch.zeros((66, 67), dtype=torch.float64, device="cuda")[:, :66]          # rows not 16-byte aligned
    assert M.mdet_logdet_device_noalloc(v, out) == S.EINVAL
    import ctypes as C
    p = M.binding._params(400000, "f64", 4096, 0, True, 0, None)
    assert M.lib().mdet_logdet_device_noalloc(C.byref(p), C.c_void_p(out.data_ptr()), 400000,
                                              C.c_void_p(out.data_ptr()), None) == S.ENOMEM_DEVICE


def test_noalloc_entry_point_recorded_into_a_graph_and_replayed(M):
    # what the entry point is for: the whole path recorded once into a HIP graph (capture refuses
    # allocations and waits) and replayed on new matrices in the same buffers, with eager work and
    # synchronisation between the replays; every replay gives the bits of the allocating entry point
    n, bs = 1024, 128
    srcs = [torch.from_numpy(W.scaled_down(W.config(c), n, bs).dense()).cuda() for c in (1, 2, 4)]
    refs, drefs = [], []
    for src in srcs:
        dref = torch.empty(n, dtype=torch.float64, device="cuda")
        refs.append(M.mdet_logdet_device(src.clone(), block_size=bs, overwrite=True, diag=dref,
                                         flags=M.FLAG_NO_LOOKAHEAD))
        drefs.append(dref)
    work = srcs[0].clone()
    out = torch.zeros(5, dtype=torch.float64, device="cuda")
    d = torch.empty(n, dtype=torch.float64, device="cuda")
    # one call outside the capture: the scratch array's address is looked up on the first call
    assert M.mdet_logdet_device_noalloc(work, out, block_size=bs, diag=d) == M.Status.OK
    torch.cuda.synchronize()
    work.copy_(srcs[0])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    with torch.cuda.graph(g, stream=stream):
        st = M.mdet_logdet_device_noalloc(work, out, block_size=bs, diag=d, stream=stream)
    assert st == M.Status.OK
    for rep in range(2):
        for src, ref, dref in zip(srcs, refs, drefs):
            work.copy_(src)                    # eager work between the replays
            out.fill_(-7.0)
            d.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert got[4] == M.Status.OK and got[0] == ref.logabsdet and int(got[1]) == ref.sign
            assert torch.equal(d, dref)

