#!/usr/bin/env python3
"""Benchmark of the log-determinant hot path on one MI355X.

One "step" = one whole pass of the path (block-column factorisation, Schur
updates, log/sign reduction) over one synthetic matrix that is already resident
where the configuration puts it (HBM for the in-core configurations, pinned host
memory for the out-of-core ones) when the timed region starts.

Prints ONE JSON line.  `value` = (n^3/3) / seconds-per-step in TFLOP/s.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"f64": 78.6, "f32": 157.3}     # MI355X dense matrix-core peaks, TFLOP/s


def form_matrix_device(w, torch, rows_per_call=2048):
    f = w.factor_torch("cuda")
    n = w.n
    a = torch.empty((n, n), dtype=torch.float64 if w.dtype == "f64" else torch.float32, device="cuda")
    for r0 in range(0, n, rows_per_call):
        r1 = min(n, r0 + rows_per_call)
        a[r0:r1] = w.block_torch(f, r0, r1, 0, n, device="cuda")
    del f
    return a


PINNED_CAP = 60 << 30    # the test machines refuse to pin more than ~64 GiB of host memory


def form_matrix_host_packed(w, torch, M, out=None):
    """Packed lower block-column layout in host memory (pinned when it fits under the
    box's pinning cap, pageable otherwise), formed tile by tile on the GPU."""
    n, b = w.n, w.block_size
    T = (n + b - 1) // b
    total = M.mdet_host_layout_offset(n, b, T)
    dt = torch.float64 if w.dtype == "f64" else torch.float32
    if out is None:
        nbytes = total * (8 if w.dtype == "f64" else 4)
        out = torch.empty(total, dtype=dt, pin_memory=nbytes <= PINNED_CAP)
    f = w.factor_torch("cuda")
    for j in range(T):
        wj = min(b, n - j * b)
        off = M.mdet_host_layout_offset(n, b, j)
        col = out[off:off + (n - j * b) * wj].view(n - j * b, wj)
        for i in range(j, T):
            r0, r1 = i * b, min(n, (i + 1) * b)
            col[r0 - j * b:r1 - j * b].copy_(w.block_torch(f, r0, r1, j * b, j * b + wj, device="cuda"))
    torch.cuda.synchronize()
    return out


def measured_traffic(workload):
    """HBM-side bytes per launch of the trailing update kernel for this workload, from the
    committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE, scaled by what the same
    counters read for a plain copy), or None when no summary covers the workload."""
    path = os.path.join(ROOT, "profiles", "trailing_update_hbm_traffic_cfg2.txt")
    try:
        kv = {}
        for line in open(path):
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split(None, 1)
            kv[k] = v.strip()
        if kv.get("workload") == workload:
            return float(kv["traffic_bytes_per_dispatch"])
    except (OSError, KeyError, ValueError):
        pass
    return None


def kernel_report(reps=5):
    """Stand-alone rates of the path's kernels through the single-step entry points:
    the Schur update against the matrix-core peak, the leaf solve and the log/sign
    reduction against HBM bandwidth.  One JSON line."""
    import torch
    import paper_2503_04424_amd as M
    M.load()
    torch.cuda.set_device(0)
    HBM = 8000.0   # GB/s, published

    def timed(fn, prep=None):
        best = None
        for _ in range(reps):
            if prep:
                prep()
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best

    out = []
    for dt, name in ((torch.float64, "f64"), (torch.float32, "f32")):
        for K in (1024, 4096):
            Mr = 16384
            g = torch.Generator(device="cuda").manual_seed(7)
            a = torch.randn(Mr, K, dtype=dt, device="cuda", generator=g)
            d = torch.rand(K, dtype=dt, device="cuda", generator=g) + 0.5
            c = torch.zeros(Mr, Mr, dtype=dt, device="cuda")
            ms = timed(lambda: M.mdet_step_schur_update(c, a, a, d, lower=True))
            flop = 2.0 * K * (Mr * (Mr + 1) / 2)
            tf = flop / ms / 1e9
            out.append({"kernel": "trailing_update_kernel", "dtype": name,
                        "shape": f"M=N={Mr} K={K} lower", "ms": ms, "achieved": tf, "unit": "TFLOP/s",
                        "bound": "mfma", "peak": PEAK[name], "frac": tf / PEAK[name]})
            ms = timed(lambda: M.mdet_step_schur_update(c, a, a, None, lower=True))
            tf = flop / ms / 1e9
            out.append({"kernel": "trailing_update_kernel, positive-definite form (no diagonal scaling)",
                        "dtype": name, "shape": f"M=N={Mr} K={K} lower", "ms": ms, "achieved": tf,
                        "unit": "TFLOP/s", "bound": "mfma", "peak": PEAK[name], "frac": tf / PEAK[name]})
            del a, c, d
    # one 64-column leaf: factorisation of the 64 x 64 diagonal block + solve of the rows below
    for m in (32768, 131072):
        w = 64
        g = torch.Generator(device="cuda").manual_seed(11)
        src = torch.randn(m, w, dtype=torch.float64, device="cuda", generator=g) * 0.01
        src[:w] += torch.eye(w, dtype=torch.float64, device="cuda")
        src[:w] = (src[:w] + src[:w].T) / 2
        panel = torch.empty_like(src)
        dv = torch.zeros(w, dtype=torch.float64, device="cuda")
        di = torch.zeros_like(dv)
        flags = torch.zeros(16 + 8192, dtype=torch.uint8, device="cuda")
        flags[:16] = 255
        ms = timed(lambda: M.mdet_step_panel_factor(panel, w, dv, di, flags), prep=lambda: panel.copy_(src))
        gb = 2.0 * (m - w) * w * 8 / 1e9
        out.append({"kernel": "leaf_factor_kernel + leaf_solve_kernel", "dtype": "f64",
                    "shape": f"m={m} w={w}", "ms": ms, "bytes": gb * 1e9,
                    "note": "both launches timed together; the solve's own duration and GB/s are in the "
                            "rocprofv3 summary of this command", "bound": "hbm", "peak": HBM, "unit": "GB/s",
                    "achieved": gb / (ms * 1e-3), "frac": gb / (ms * 1e-3) / HBM})
    # the same leaf with pivoting: its own 64 x 64 factorisation kernel, then the solve
    for m in (32768,):
        w = 64
        g = torch.Generator(device="cuda").manual_seed(12)
        src = torch.randn(m, w, dtype=torch.float64, device="cuda", generator=g) * 0.01
        src[:w] += torch.diag(torch.linspace(1.0, 3.0, w, dtype=torch.float64, device="cuda"))
        src[:w] = (src[:w] + src[:w].T) / 2
        panel = torch.empty_like(src)
        dv = torch.zeros(w, dtype=torch.float64, device="cuda")
        di = torch.zeros_like(dv)
        pm = torch.zeros(w, dtype=torch.int32, device="cuda")
        flags = torch.zeros(16 + 8192, dtype=torch.uint8, device="cuda")
        flags[:16] = 255
        ms = timed(lambda: M.mdet_step_panel_factor_pivoted(panel, w, dv, di, pm, flags),
                   prep=lambda: panel.copy_(src))
        out.append({"kernel": "leaf_factor_pivoted_kernel + leaf_solve_kernel", "dtype": "f64",
                    "shape": f"m={m} w={w}", "ms": ms,
                    "note": "both launches timed together; each kernel's own duration is in the "
                            "rocprofv3 summary of this command (64 dependent pivot steps, latency-bound)"})
    # a leaf of a general matrix: P A = L D U of the 64 x 64 block, then the rows below it in
    # both triangles (one solve launch)
    for m in (32768,):
        w = 64
        g = torch.Generator(device="cuda").manual_seed(13)
        src = torch.randn(2, m, w, dtype=torch.float64, device="cuda", generator=g) * 0.01
        src[0, :w] += torch.diag(torch.linspace(1.0, 3.0, w, dtype=torch.float64, device="cuda"))[torch.randperm(
            w, generator=torch.Generator().manual_seed(13)).cuda()]
        panel = torch.empty_like(src)
        dv = torch.zeros(w, dtype=torch.float64, device="cuda")
        di = torch.zeros_like(dv)
        pm = torch.zeros(w, dtype=torch.int32, device="cuda")
        flags = torch.zeros(32 + 16384, dtype=torch.uint8, device="cuda")

        def prep():
            panel.copy_(src)
            flags.zero_()
            flags[:16] = 255
        ms = timed(lambda: M.mdet_step_panel_factor_general(panel[0], panel[1], w, dv, di, pm, flags), prep=prep)
        out.append({"kernel": "leaf_lu_kernel + leaf_solve_general_kernel", "dtype": "f64",
                    "shape": f"m={m} w={w} (both triangles)", "ms": ms,
                    "note": "both launches timed together; each kernel's own duration is in the "
                            "rocprofv3 summary of this command (64 dependent pivot steps, latency-bound)"})
    for n in (196608,):          # one workgroup per block column; here a single column
        dvec = torch.rand(n, dtype=torch.float64, device="cuda") + 0.5
        res = torch.zeros(8, dtype=torch.float64, device="cuda")
        ms = timed(lambda: M.mdet_step_logdet_reduce(dvec, res))
        gb = n * 8 / 1e9
        out.append({"kernel": "logdet_partial_kernel + logdet_combine_kernel", "dtype": "f64",
                    "shape": f"n={n}", "ms": ms, "bound": "hbm", "peak": HBM, "unit": "GB/s",
                    "achieved": gb / (ms * 1e-3), "frac": gb / (ms * 1e-3) / HBM})
    # principal-minor sequence and the FLODANCE regression (Sec. 3.2, Alg. 2) at the size of the
    # paper's experiments: 50 000 data points with d = 10 outputs, q = 10 correction terms
    n_s, dd, n0, q = 50000, 10, 100, 10
    piv = torch.rand(n_s * dd, dtype=torch.float64, device="cuda") + 0.5
    ell = torch.empty_like(piv)
    ws = torch.empty(M.mdet_sequence_workspace_query(n_s * dd, n_s - n0, q), dtype=torch.uint8, device="cuda")
    ms = timed(lambda: M.mdet_principal_logdets(piv, ell=ell, workspace=ws))
    gb = 3.0 * n_s * dd * 8 / 1e9          # pivots read twice, sequence written once
    out.append({"kernel": "seq_chunk_sums + seq_chunk_offsets + seq_running_sum", "dtype": "f64",
                "shape": f"n={n_s * dd}", "ms": ms, "bytes": gb * 1e9, "bound": "hbm", "peak": HBM,
                "unit": "GB/s", "achieved": gb / (ms * 1e-3), "frac": gb / (ms * 1e-3) / HBM})
    coef = torch.empty(q + 4, dtype=torch.float64, device="cuda")
    ms = timed(lambda: M.mdet_flodance_fit(ell, dd, n0, n_s, q, coef=coef, workspace=ws))
    out.append({"kernel": "flo_qr_kernel (3 levels)", "dtype": "f64",
                "shape": f"rows={n_s - n0} cols={q + 3}", "ms": ms,
                "note": "latency-bound: 13 dependent reflections per level, one block reduction each"})
    nv = torch.logspace(2, 6, 100000, dtype=torch.float64, device="cuda")
    ov = torch.empty_like(nv)
    ms = timed(lambda: M.mdet_flodance_eval(coef, q, nv, out=ov))
    out.append({"kernel": "flo_eval_kernel", "dtype": "f64", "shape": "count=100000", "ms": ms})
    print(json.dumps({"metric": "stand-alone kernel rates (single-step entry points)", "n_gpus": 1,
                      "data": "synthetic", "kernels": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (default 2)")
    ap.add_argument("--dtype", default=None, choices=["f64", "f32"])
    ap.add_argument("--block-size", type=int, default=0)
    ap.add_argument("--n", type=int, default=0, help="override the order (scaled-down stand-in)")
    ap.add_argument("--budget-gib", type=float, default=-1.0,
                    help="device budget in GiB; >0 puts the matrix in pinned host memory and streams it")
    ap.add_argument("--no-lookahead", action="store_true",
                    help="diagnostic: run every kernel on one stream, nothing overlapped")
    ap.add_argument("--compute-f64", action="store_true",
                    help="with --dtype f32 (in-core): fp32 storage, fp64 arithmetic")
    ap.add_argument("--scaled-copy", action="store_true",
                    help="in-core: MDET_FLAG_SCALED_COPY (2 n block_size elements more workspace)")
    ap.add_argument("--assume-spd", action="store_true",
                    help="the positive-definite (Cholesky) form of the method instead of LDL^T")
    ap.add_argument("--file-dir", default="",
                    help="out-of-core configurations: write the matrix to a file in this directory "
                         "and run mdet_logdet_file on it (factors go to a scratch file beside it)")
    ap.add_argument("--general", action="store_true",
                    help="MDET_FLAG_GENERAL: the configuration's matrix with its rows shuffled inside groups of 64, "
                         "factored as a general matrix (P A = L D U; in-core configurations; counts 2n^3/3)")
    ap.add_argument("--pivot", action="store_true",
                    help="MDET_FLAG_PIVOT: pivoting on the diagonal inside each group of 64 columns")
    ap.add_argument("--kernels", action="store_true",
                    help="instead of the path: stand-alone rates of its kernels (one JSON line)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=0, help="order of the oracle's sample block")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.kernels:
        kernel_report()
        return

    import numpy as np
    import torch
    import workloads as W
    import paper_2503_04424_amd as M
    M.load()
    torch.cuda.set_device(0)

    w = W.config(args.config, args.dtype)
    if args.dtype and w.dtype != args.dtype:
        print(f"bench.py: configuration {args.config} is defined in {w.dtype} only "
              "(configuration 3 has an f32 variant)", file=sys.stderr)
        sys.exit(2)
    if args.n:
        w = W.scaled_down(w, args.n, args.block_size or None)
    if args.block_size:
        w.block_size = args.block_size
    if args.budget_gib >= 0:
        w.mem_budget = int(args.budget_gib * (1 << 30))
    n, bs = w.n, w.block_size
    out_of_core = w.mem_budget > 0

    steps, warmup = args.steps, args.warmup
    xflags = M.FLAG_NO_LOOKAHEAD if args.no_lookahead else 0
    widen = bool(args.compute_f64) and w.dtype == "f32" and not out_of_core
    if args.compute_f64 and not widen:
        print("bench.py: --compute-f64 goes with --dtype f32 and an in-core configuration", file=sys.stderr)
        sys.exit(2)
    if widen:
        xflags |= M.FLAG_COMPUTE_F64
    if args.assume_spd:
        xflags |= M.FLAG_ASSUME_SPD
    if args.scaled_copy:
        xflags |= M.FLAG_SCALED_COPY
    if args.pivot:
        xflags |= M.FLAG_PIVOT
    if args.general:
        if out_of_core or widen or args.assume_spd or args.pivot or args.scaled_copy:
            print("bench.py: --general goes with an in-core configuration and no other form", file=sys.stderr)
            sys.exit(2)
        xflags |= M.FLAG_GENERAL
    results = []
    if not out_of_core:
        a = form_matrix_device(w, torch)
        if args.general:
            rng = np.random.default_rng(w.seed)
            rows = np.concatenate([g0 + rng.permutation(min(64, n - g0)) for g0 in range(0, n, 64)])
            a = a[torch.from_numpy(rows).cuda()].contiguous()
        torch.cuda.synchronize()
        free, _ = torch.cuda.mem_get_info()
        per = a.numel() * a.element_size()
        diag = torch.empty(n, dtype=torch.float64 if widen else a.dtype, device="cuda")
        if widen:
            # the library factors an fp64 copy in its own workspace; the input stays as it is
            ncopies = 1 << 30
            copies = {0: a}

            def refill():
                pass
        elif free * 0.8 >= per:
            ncopies = max(1, min(steps + warmup + 1, int(free * 0.8 // per)))
            copies = [a.clone() for _ in range(ncopies)]       # the path overwrites its input

            def refill():
                for c in copies:
                    c.copy_(a)
                torch.cuda.synchronize()
        else:
            # no room for a second copy: factor the matrix in place and form it again
            # (untimed) before the next pass
            ncopies = 1
            copies = [a]
            a = None

            def refill():
                copies[0] = None
                copies[0] = form_matrix_device(w, torch)
                torch.cuda.synchronize()

        def run(i, flags=0, want_diag=False):
            return M.mdet_logdet_device(copies[0 if widen else i % ncopies], block_size=bs, overwrite=True,
                                        flags=flags | (M.FLAG_COMPUTE_F64 if widen else 0) |
                                        (M.FLAG_GENERAL if args.general else 0),
                                        diag=diag if want_diag else None)
        done = 0
        for i in range(warmup):
            run(done); done += 1
        t_total = 0.0
        k = 0
        while k < steps:
            if done % ncopies == 0 and done:
                refill()
            batch = min(steps - k, ncopies - done % ncopies)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(batch):
                results.append(run(done, flags=M.FLAG_PROFILE | xflags, want_diag=True)); done += 1
            torch.cuda.synchronize()
            t_total += time.perf_counter() - t0
            k += batch
        final = results[-1]
        diag_host = diag.cpu().numpy().astype(np.float64)
    else:
        h = form_matrix_host_packed(w, torch, M)
        pinned = h.is_pinned()
        diag = torch.empty(n, dtype=h.dtype, pin_memory=True)
        # the run overwrites the host matrix with the factor, so it is formed afresh
        # (untimed) before every pass
        t_total = 0.0
        for i in range(warmup + steps):
            if i:
                form_matrix_host_packed(w, torch, M, out=h)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if args.file_dir:
                if i == 0:
                    os.makedirs(args.file_dir, exist_ok=True)
                    mpath = os.path.join(args.file_dir, "memdet_matrix.bin")
                    spath = os.path.join(args.file_dir, "memdet_scratch.bin")
                    h.numpy().tofile(mpath)          # untimed; the run leaves this file as it is
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                r = M.mdet_logdet_file(mpath, n, w.dtype, bs, mem_budget=w.mem_budget, overwrite=False,
                                       scratch_path=spath, flags=M.FLAG_PROFILE | xflags, diag=diag)
            else:
                r = M.mdet_logdet_host(h, n, bs, mem_budget=w.mem_budget, overwrite=True,
                                       flags=M.FLAG_PROFILE | xflags, diag=diag)
            torch.cuda.synchronize()
            if i >= warmup:
                t_total += time.perf_counter() - t0
                results.append(r)
        if args.file_dir:
            for f in (mpath, spath):
                if os.path.exists(f):
                    os.remove(f)
        final = results[-1]
        diag_host = diag.numpy().astype(np.float64)

    sec = t_total / steps
    flop = n ** 3 / 3.0 * (2.0 if args.general else 1.0)
    value = flop / sec / 1e12
    upd_t = sum(r.t_trailing_update for r in results)
    upd_f = sum(r.trailing_update_flops for r in results)
    upd_n = sum(r.trailing_update_launches for r in results)
    achieved = upd_f / upd_t / 1e12 if upd_t > 0 else None
    peak = PEAK["f64" if widen else w.dtype]
    line = {
        "metric": ("logdet throughput, (2n^3/3)/time-to-logdet" if args.general
                   else "logdet throughput, (n^3/3)/time-to-logdet"),
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64" if widen else w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n": n, "block_size": bs,
                   "placement": ("file (pread/pwrite through pinned chunks), streamed" if args.file_dir else
                                 ("pinned" if pinned else "pageable") + " host memory, streamed")
                   if out_of_core else "HBM, in-core",
                   "mem_budget_bytes": w.mem_budget, "seed": w.seed,
                   **({"storage": "f32, widened exactly; arithmetic f64"} if widen else {}),
                   **({"form": "positive definite (Cholesky), MDET_FLAG_ASSUME_SPD"} if args.assume_spd else {}),
                   **({"workspace": "MDET_FLAG_SCALED_COPY"} if args.scaled_copy else {}),
                   **({"pivoting": "inside groups of 64, MDET_FLAG_PIVOT"} if args.pivot else {}),
                   **({"form": "general matrix (rows shuffled inside groups of 64), P A = L D U, "
                               "MDET_FLAG_GENERAL; value counts 2n^3/3"} if args.general else {})},
        "time_to_logdet_s": sec, "frac_of_matrix_peak": value / peak,
        "logabsdet": final.logabsdet, "sign": final.sign, "negative_pivots": final.negative_pivots,
        "kernel_launches_per_step": final.kernel_launches,
        "roofline": {
            "kernel": ("trailing_update_kernel (Schur update A_ij -= L_ik L_jk^T on MFMA)" if args.assume_spd
                       else "trailing_update_general_kernel (Schur update A_ij -= L_ik D_k U_kj of both triangles "
                            "in one launch, on MFMA)" if args.general
                       else "trailing_update_kernel (Schur update A_ij -= L_ik D_k L_jk^T on MFMA)"),
            "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
            "frac": (achieved / peak) if achieved else None,
            "traffic": measured_traffic(w.name) if not (args.n or args.block_size or args.general) else None,
            "launches_timed": upd_n,
            "avg_launch_ms": (upd_t / upd_n * 1e3) if upd_n else None,
            "flop_per_launch_avg": (upd_f / upd_n) if upd_n else None,
        },
    }
    if out_of_core:
        line["host_link"] = {"bytes_h2d": final.bytes_h2d, "bytes_d2h": final.bytes_d2h,
                             "GBps_avg_h2d": final.bytes_h2d / sec / 1e9,
                             "seconds_busy_h2d": final.t_h2d, "seconds_busy_d2h": final.t_d2h,
                             "GBps_while_copying_h2d": (final.bytes_h2d / final.t_h2d / 1e9) if final.t_h2d else None,
                             "GBps_while_copying_d2h": (final.bytes_d2h / final.t_d2h / 1e9) if final.t_d2h else None,
                             "dev_bytes_high_water": final.dev_bytes_high_water,
                             "superpanels": final.num_superpanels}
    cf = w.closed_form_logdet()
    if cf is not None:
        line["closed_form_rel_err"] = abs(final.logabsdet - cf) / abs(cf)

    if not args.no_cpu_baseline:
        import oracle
        m = args.cpu_sample or min(n, 6144)
        if out_of_core:
            f = w.factor_torch("cuda")
            sample = w.block_torch(f, 0, m, 0, m, device="cuda").cpu().numpy()
        else:
            sample = (w.block_torch(w.factor_torch("cuda"), 0, m, 0, m, device="cuda").cpu().numpy()
                      if a is None else a[:m, :m].cpu().numpy())
        t0 = time.perf_counter()
        if args.assume_spd:
            oc = oracle.cholesky_logdet(sample)
            o_logabsdet, o_name = oc.logdet, "Cholesky"
        else:
            o_logabsdet, o_name = oracle.ldlt_logdet(sample).logabsdet, "LDL^T"
        t_cpu = time.perf_counter() - t0
        gpu_partial = float(np.sum(np.log(np.abs(diag_host[:m]))))
        line["cpu_baseline"] = {
            "value": (m ** 3 / 3.0) / t_cpu / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": t_cpu,
            "sample": f"leading principal {m}x{m} block of the same matrix (long-double unblocked {o_name})",
        }
        line["parity_vs_oracle_rel_err"] = abs(gpu_partial - o_logabsdet) / max(1.0, abs(o_logabsdet))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
