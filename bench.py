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
    box's pinning cap, pageable otherwise), formed tile by tile on the GPU.  Tiles bound
    for pageable memory pass through two pinned buffers, so that the device-to-host copy
    runs at the link's rate and the host-side copy overlaps the next tile's formation."""
    n, b = w.n, w.block_size
    T = (n + b - 1) // b
    total = M.mdet_host_layout_offset(n, b, T)
    dt = torch.float64 if w.dtype == "f64" else torch.float32
    if out is None:
        nbytes = total * (8 if w.dtype == "f64" else 4)
        out = torch.empty(total, dtype=dt, pin_memory=nbytes <= PINNED_CAP)
    f = w.factor_torch("cuda")
    bounce = None if out.is_pinned() else [torch.empty(b * b, dtype=dt, pin_memory=True) for _ in range(2)]
    events = [torch.cuda.Event(), torch.cuda.Event()]
    pending = None          # (destination view, bounce index, elements)
    t = 0

    def drain():
        nonlocal pending
        if pending is not None:
            dst, q, cnt = pending
            events[q].synchronize()
            dst.view(-1).copy_(bounce[q][:cnt])
            pending = None
    for j in range(T):
        wj = min(b, n - j * b)
        off = M.mdet_host_layout_offset(n, b, j)
        col = out[off:off + (n - j * b) * wj].view(n - j * b, wj)
        for i in range(j, T):
            r0, r1 = i * b, min(n, (i + 1) * b)
            tile = w.block_torch(f, r0, r1, j * b, j * b + wj, device="cuda")
            dst = col[r0 - j * b:r1 - j * b]
            if bounce is None:
                dst.copy_(tile)
                continue
            q = t & 1
            t += 1
            cnt = tile.numel()
            bounce[q][:cnt].copy_(tile.reshape(-1), non_blocking=True)
            events[q].record()
            drain()                       # the tile before this one, while this one is on its way
            pending = (dst, q, cnt)
    drain()
    torch.cuda.synchronize()
    return out


def measured_traffic(workload):
    """HBM-side bytes per launch of the trailing update kernel for this workload, from the
    committed rocprofv3 --pmc summary that names it (FETCH_SIZE and WRITE_SIZE, scaled by what
    the same counters read for a plain copy), or None when no summary covers the workload."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "trailing_update_hbm_traffic_*.txt"))):
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
            if K == 4096:
                # all 128 x 128 blocks of a square C: 16384 blocks = 32 full rounds of the device's 512
                # workgroup slots (the lower-triangular launch above has 8256 = 16.1, a nearly empty last one)
                ms = timed(lambda: M.mdet_step_schur_update(c, a, a, None, lower=False))
                tf = 2.0 * K * Mr * Mr / ms / 1e9
                out.append({"kernel": "trailing_update_kernel, positive-definite form (no diagonal scaling)",
                            "dtype": name, "shape": f"M=N={Mr} K={K} full", "ms": ms, "achieved": tf,
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
        out.append({"kernel": "logdet_partial_kernel + logdet_combine_kernel", "dtype": "f64",
                    "shape": f"n={n} as ONE block column", "ms": ms, "bytes": n * 8,
                    "note": "latency-bound, not a bandwidth kernel: one workgroup reduces one block column's pivots "
                            "(n logs by 256 threads) and one thread adds the columns' terms in order; in the path a "
                            "block column has 1024 ... 8192 pivots and the two launches take under 10 us together"})
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


def mfma_peak_report(reps=3):
    """The matrix pipe's measured ceiling: register-only loops of 16 x 16 x 4 products
    (mdet_step_mfma_peak), one and two workgroups per compute unit, in launches of about
    2, 20 and 200 ms (the clock the chip sustains depends on how long the pipe stays full).
    One JSON line."""
    import torch
    import paper_2503_04424_amd as M
    M.load()
    torch.cuda.set_device(0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    rows = []
    for dt, name in ((torch.float64, "f64"), (torch.float32, "f32")):
        out = torch.empty(65536, dtype=dt, device="cuda")
        for nacc, per_cu, scale in ((4, 1, 1), (4, 1, 10), (4, 2, 10), (16, 1, 1), (16, 1, 10), (16, 2, 10),
                                    (16, 1, 100)):
            wgs = cus * per_cu
            # one f64 product occupies a SIMD's matrix pipe for 64 clocks, one f32 product for 32
            iters = (4000 if name == "f64" else 8000) * scale // per_cu
            M.mdet_step_mfma_peak(name, wgs, 200, out, accumulators=nacc)
            best = None
            for _ in range(reps):
                torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                flop = M.mdet_step_mfma_peak(name, wgs, iters, out, accumulators=nacc)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            tf = flop / best / 1e9
            rows.append({"kernel": f"mfma_peak_{name}_kernel<{nacc}>", "dtype": name, "accumulators": nacc,
                         "workgroups": wgs, "wavefronts_per_simd": per_cu, "ms": round(best, 3),
                         "achieved": round(tf, 2), "unit": "TFLOP/s", "published_peak": PEAK[name],
                         "frac_of_published": round(tf / PEAK[name], 4)})
    print(json.dumps({"metric": "matrix-core ceiling, register-only 16x16x4 products", "n_gpus": 1,
                      "compute_units": cus, "rows": rows}))


def copy_calibration(gib=4.0, reps=3):
    """A plain copy of a known size by the library's copy_kernel (mdet_step_copy): run under
    `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` it gives the factor between what
    those counters report and bytes actually moved.  One JSON line."""
    import torch
    import paper_2503_04424_amd as M
    M.load()
    torch.cuda.set_device(0)
    nbytes = int(gib * (1 << 30)) // 16 * 16
    src = torch.ones(nbytes // 8, dtype=torch.float64, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        M.mdet_step_copy(dst, src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    print(json.dumps({"metric": "copy calibration (copy_kernel)", "bytes_read": nbytes, "bytes_written": nbytes,
                      "kib_read": nbytes / 1024, "dispatches": reps, "ms": best,
                      "GBps_read_plus_write": 2 * nbytes / best / 1e6}))


def pmc_summary(directory):
    """Per-kernel averages of the counters in the rocprofv3 --pmc CSV files under `directory`
    (KiB per dispatch for FETCH_SIZE / WRITE_SIZE).  Plain text, for profiles/."""
    import collections
    import csv
    import glob
    paths = sorted(glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True))
    if not paths:
        print(f"bench.py: no *counter_collection.csv under {directory}", file=sys.stderr)
        sys.exit(2)
    for path in paths:
        agg = collections.defaultdict(lambda: collections.defaultdict(float))
        seen = collections.defaultdict(set)
        for r in csv.DictReader(open(path)):
            name = r["Kernel_Name"]
            if "mdet::" not in name:
                continue
            k = name.split("mdet::")[1].split("(")[0].split("<")[0]
            agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
            seen[k].add(r["Dispatch_Id"])
        print(f"# {os.path.relpath(path, directory)}")
        print(f"{'kernel':44s} {'dispatches':>10s}  counter: average per dispatch")
        for k in sorted(agg):
            nd = len(seen[k])
            vals = "  ".join(f"{c}: {v / nd:.1f}" for c, v in sorted(agg[k].items()))
            print(f"{k:44s} {nd:10d}  {vals}")


def stats_summary(directory):
    """The library's kernels (and the runtime's copy kernels) from rocprofv3's kernel_stats CSV,
    and the copies from its memory-copy CSVs if there are any, under `directory`.  Plain text,
    for profiles/.  This rocprofv3 records no sizes for copies: bytes are in bench.py's own line."""
    import csv
    import glob
    for path in sorted(glob.glob(os.path.join(directory, "**", "*kernel_stats.csv"), recursive=True)):
        print(f"# {os.path.relpath(path, directory)}")
        print(f"{'kernel':58s} {'calls':>7s} {'total_ms':>11s} {'avg_us':>11s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}")
        other = 0.0
        for r in csv.DictReader(open(path)):
            name = r["Name"]
            if "mdet::" in name:
                short = name.split("mdet::")[1].split("(")[0]
            elif name.startswith("__amd_rocclr_"):
                short = name + " (runtime copy kernel)"
            else:
                other += float(r["TotalDurationNs"])
                continue
            print(f"{short[:58]:58s} {int(r['Calls']):7d} {float(r['TotalDurationNs']) / 1e6:11.3f} "
                  f"{float(r['AverageNs']) / 1e3:11.2f} {float(r['MinNs']) / 1e3:10.2f} "
                  f"{float(r['MaxNs']) / 1e3:10.2f} {float(r['Percentage']):6.2f}")
        print(f"{'(other kernels: input generation by torch)':58s} {'':7s} {other / 1e6:11.3f}")
    for path in sorted(glob.glob(os.path.join(directory, "**", "*memory_copy_stats.csv"), recursive=True)):
        print(f"# {os.path.relpath(path, directory)}")
        print(f"{'direction':30s} {'copies':>8s} {'busy_s':>9s} {'avg_us':>10s} {'min_us':>9s} {'max_us':>9s}")
        for r in csv.DictReader(open(path)):
            print(f"{r['Name']:30s} {int(r['Calls']):8d} {float(r['TotalDurationNs']) / 1e9:9.3f} "
                  f"{float(r['AverageNs']) / 1e3:10.2f} {float(r['MinNs']) / 1e3:9.2f} {float(r['MaxNs']) / 1e3:9.2f}")


def main():
    t_process = time.perf_counter()
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4,
                    help="benchmark configuration 1..5 (default 4: n=131072 streamed from host memory under a "
                         "16 GiB device budget, the configuration the metric is quoted on)")
    ap.add_argument("--dtype", default=None, choices=["f64", "f32"])
    ap.add_argument("--block-size", type=int, default=0)
    ap.add_argument("--n", type=int, default=0, help="override the order (scaled-down stand-in)")
    ap.add_argument("--budget-gib", type=float, default=-1.0,
                    help="device budget in GiB; >0 puts the matrix in host memory and streams it")
    ap.add_argument("--time-budget", type=float, default=450.0,
                    help="seconds of wall clock this process may take (0 = no limit): with passes of "
                         "many seconds the number of warm-up and timed passes is cut to fit, and the "
                         "line reports the numbers actually run")
    ap.add_argument("--no-incore", action="store_true",
                    help="streamed configurations: skip the pass over the same matrix resident in HBM")
    ap.add_argument("--no-lookahead", action="store_true",
                    help="diagnostic: run every kernel on one stream, nothing overlapped")
    ap.add_argument("--compute-f64", action="store_true",
                    help="with --dtype f32: fp32 storage, fp64 arithmetic")
    ap.add_argument("--scaled-copy", action="store_true",
                    help="in-core: MDET_FLAG_SCALED_COPY (2 n block_size elements more workspace)")
    ap.add_argument("--assume-spd", action="store_true",
                    help="the positive-definite (Cholesky) form of the method instead of LDL^T")
    ap.add_argument("--file-dir", default="",
                    help="out-of-core configurations: write the matrix to a file in this directory "
                         "and run mdet_logdet_file on it (factors go to a scratch file beside it)")
    ap.add_argument("--general", action="store_true",
                    help="MDET_FLAG_GENERAL: the configuration's matrix with its rows shuffled inside groups of 64, "
                         "factored as a general matrix (P A = L D U; counts 2n^3/3)")
    ap.add_argument("--pivot", action="store_true",
                    help="MDET_FLAG_PIVOT: pivoting on the diagonal inside each group of 64 columns")
    ap.add_argument("--pivot-block", action="store_true",
                    help="MDET_FLAG_PIVOT_BLOCK: pivoting on the diagonal over each whole diagonal block")
    ap.add_argument("--kernels", action="store_true",
                    help="instead of the path: stand-alone rates of its kernels (one JSON line)")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="instead of the path: the matrix pipe's measured ceiling (one JSON line)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the path: a plain copy of known size, for scaling the memory counters")
    ap.add_argument("--pmc-summary", default="", metavar="DIR",
                    help="no GPU work: per-kernel counter averages from rocprofv3 --pmc CSV output in DIR")
    ap.add_argument("--stats-summary", default="", metavar="DIR",
                    help="no GPU work: kernel and memory-copy statistics from rocprofv3 CSV output in DIR")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=0, help="order of the oracle's sample block")
    args = ap.parse_args()
    if args.pmc_summary:
        pmc_summary(args.pmc_summary)
        return
    if args.stats_summary:
        stats_summary(args.stats_summary)
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.kernels:
        kernel_report()
        return
    if args.mfma_peak:
        mfma_peak_report()
        return
    if args.copy_calibration:
        copy_calibration()
        return

    import numpy as np
    import torch
    import workloads as W
    import paper_2503_04424_amd as M
    M.load()
    torch.cuda.set_device(0)

    def log(msg):
        print(f"[bench {time.perf_counter() - t_process:7.1f}s] {msg}", file=sys.stderr, flush=True)

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
    budget_s = args.time_budget if args.time_budget > 0 else float("inf")

    def elapsed():
        return time.perf_counter() - t_process

    xflags = M.FLAG_NO_LOOKAHEAD if args.no_lookahead else 0
    widen = bool(args.compute_f64) and w.dtype == "f32"
    if args.compute_f64 and not widen:
        print("bench.py: --compute-f64 goes with --dtype f32", file=sys.stderr)
        sys.exit(2)
    if widen:
        xflags |= M.FLAG_COMPUTE_F64
    if args.assume_spd:
        xflags |= M.FLAG_ASSUME_SPD
    if args.scaled_copy:
        xflags |= M.FLAG_SCALED_COPY
    if args.pivot:
        xflags |= M.FLAG_PIVOT
    if args.pivot_block:
        xflags |= M.FLAG_PIVOT_BLOCK
    if args.general:
        if out_of_core or widen or args.assume_spd or args.pivot or args.pivot_block or args.scaled_copy:
            print("bench.py: --general goes with an in-core configuration and no other form", file=sys.stderr)
            sys.exit(2)
        xflags |= M.FLAG_GENERAL
    run_flags = M.FLAG_PROFILE | xflags
    requested = (steps, warmup)
    results = []
    pass_ms = []        # wall clock of every timed pass, ms
    incore = None
    a = None
    if not out_of_core:
        a = form_matrix_device(w, torch)
        if args.general:
            rng = np.random.default_rng(w.seed)
            rows = np.concatenate([g0 + rng.permutation(min(64, n - g0)) for g0 in range(0, n, 64)])
            a = a[torch.from_numpy(rows).cuda()].contiguous()
        torch.cuda.synchronize()
        # the workspace is the caller's (torch's), sized by the library's own query: nothing is
        # allocated or freed inside the timed region
        ws_bytes, _ = M.mdet_workspace_query(n, a.dtype, bs, 0, overwrite=not widen, flags=run_flags,
                                             for_device_input=True)
        ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
        free, _ = torch.cuda.mem_get_info()
        per = a.numel() * a.element_size()
        diag = torch.empty(n, dtype=torch.float64 if widen else a.dtype, device="cuda")
        if widen:
            # the library factors an fp64 copy in the workspace; the input stays as it is
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

        def run(i, want_diag=False):
            return M.mdet_logdet_device(copies[0 if widen else i % ncopies], block_size=bs, overwrite=not widen,
                                        flags=run_flags, workspace=ws, diag=diag if want_diag else None)
        done = 0
        for i in range(warmup):
            if done % ncopies == 0 and done:
                refill()
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
                results.append(run(done, want_diag=True)); done += 1
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            t_total += dt
            pass_ms.extend([dt / batch * 1e3] * batch)     # passes timed back to back share one clock reading
            k += batch
        final = results[-1]
        diag_host = diag.cpu().numpy().astype(np.float64)
    else:
        log(f"forming {w.name} in host memory")
        h = form_matrix_host_packed(w, torch, M)
        pinned = h.is_pinned()
        log(f"formed ({h.numel() * h.element_size() / 2**30:.1f} GiB, {'pinned' if pinned else 'pageable'})")
        diag = torch.empty(n, dtype=torch.float64 if widen else h.dtype, pin_memory=True)
        # overwrite = 0: the factored block columns go to a scratch area in host memory (the paper's
        # scratchpad, Sec. 2.2) and the matrix stays as it is, so no pass needs it formed again;
        # workspace and scratch are the caller's, sized by the library's own query
        # (a matrix too large for a second copy in host memory is factored in place and formed again,
        # untimed, before every pass)
        avail = 0
        for ln in open("/proc/meminfo"):
            if ln.startswith("MemAvailable:"):
                avail = int(ln.split()[1]) * 1024
        keep_input = h.numel() * h.element_size() < 0.45 * avail or widen
        ws_bytes, hs_bytes = M.mdet_workspace_query(n, h.dtype, bs, w.mem_budget, overwrite=not keep_input,
                                                    flags=run_flags)
        ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
        hs = None
        mpath = spath = None
        if args.file_dir:
            os.makedirs(args.file_dir, exist_ok=True)
            mpath = os.path.join(args.file_dir, "memdet_matrix.bin")
            spath = os.path.join(args.file_dir, "memdet_scratch.bin")
            h.numpy().tofile(mpath)          # untimed; the runs leave this file as it is
        elif hs_bytes:
            hs = torch.empty(hs_bytes, dtype=torch.uint8, pin_memory=pinned and hs_bytes <= PINNED_CAP // 2)

        passes_done = [0]

        def run_streamed():
            if not keep_input and passes_done[0]:
                form_matrix_host_packed(w, torch, M, out=h)
            passes_done[0] += 1
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if args.file_dir:
                r = M.mdet_logdet_file(mpath, n, w.dtype, bs, mem_budget=w.mem_budget, overwrite=False,
                                       scratch_path=spath, flags=run_flags, diag=diag, workspace=ws)
            else:
                r = M.mdet_logdet_host(h, n, bs, mem_budget=w.mem_budget, overwrite=not keep_input,
                                       flags=run_flags, diag=diag, workspace=ws, host_scratch=hs)
            torch.cuda.synchronize()
            return r, time.perf_counter() - t0

        # what still has to fit behind the timed passes: the resident pass and the oracle's sample
        tail_s = 0.0 if args.time_budget <= 0 else 25.0
        t_pass = None
        warm_done = 0
        for i in range(warmup):
            if t_pass is not None and elapsed() + (1 + min(steps, 2)) * t_pass + 3 * t_pass + tail_s > budget_s:
                break
            r, t_pass = run_streamed()
            warm_done += 1
            log(f"warm-up pass {i}: {t_pass:.3f} s")
        t_total = 0.0
        for i in range(steps):
            if i > 0 and elapsed() + t_pass + (0 if args.no_incore else 3 * t_pass) + tail_s > budget_s:
                break
            r, t_pass = run_streamed()
            t_total += t_pass
            pass_ms.append(t_pass * 1e3)
            results.append(r)
            log(f"timed pass {i}: {t_pass:.3f} s")
        if (len(results), warm_done) != (steps, warmup):
            log(f"time budget of {budget_s:.0f} s: {warm_done} of {warmup} warm-up and {len(results)} of {steps} "
                "timed passes run")
        steps, warmup = len(results), warm_done
        if args.file_dir:
            for f in (mpath, spath):
                if os.path.exists(f):
                    os.remove(f)
        final = results[-1]
        diag_host = diag.numpy().astype(np.float64)
        # ---- the same matrix resident in HBM, one pass (the in-core rate the streamed one is
        # compared with); skipped if the device cannot hold it
        dense_bytes = n * n * (8 if w.dtype == "f64" else 4)
        del ws, hs
        torch.cuda.empty_cache()
        free, _ = torch.cuda.mem_get_info()
        if not args.no_incore and not widen and free > dense_bytes * 1.15 + (4 << 30):
            log("forming the same matrix in HBM")
            ad = form_matrix_device(w, torch)
            wsb, _ = M.mdet_workspace_query(n, ad.dtype, bs, 0, overwrite=True, flags=run_flags, for_device_input=True)
            wsd = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ri = M.mdet_logdet_device(ad, block_size=bs, overwrite=True, flags=run_flags, workspace=wsd)
            torch.cuda.synchronize()
            ti = time.perf_counter() - t0
            log(f"resident pass: {ti:.3f} s")
            incore = {"time_to_logdet_s": ti, "value": n ** 3 / 3.0 / ti / 1e12, "unit": "TFLOP/s",
                      "passes": 1, "placement": "the same matrix, dense, resident in HBM (mdet_logdet_device)",
                      "logabsdet": ri.logabsdet, "sign": ri.sign,
                      "streamed_over_incore_time": (t_total / steps) / ti,
                      "rel_diff_logabsdet": abs(ri.logabsdet - final.logabsdet) / max(1.0, abs(final.logabsdet))}
            del ad, wsd
            torch.cuda.empty_cache()

    sec = t_total / steps
    flop = n ** 3 / 3.0 * (2.0 if args.general else 1.0)
    value = flop / sec / 1e12
    peak = PEAK["f64" if widen else w.dtype]
    # roofline of the trailing (Schur) update: every launch of its two kernels, bracketed by HIP
    # events on the stream it ran on; `achieved` = their flops / the time during which at least one
    # of them was running (launches on the two compute streams overlap: the plain sum of the
    # durations, which is what a profiler's per-kernel average gives, counts that time twice)
    f128 = sum(r.trailing_update_flops for r in results)
    t128 = sum(r.t_trailing_update for r in results)
    n128 = sum(r.trailing_update_launches for r in results)
    f64b = sum(r.trailing_update64_flops for r in results)
    t64b = sum(r.t_trailing_update64 for r in results)
    n64b = sum(r.trailing_update64_launches for r in results)
    busy = sum(r.t_trailing_update_busy for r in results)
    achieved = (f128 + f64b) / busy / 1e12 if busy > 0 else None
    traffic = measured_traffic(w.name) if not (args.n or args.block_size or args.general or xflags) else None
    line = {
        "metric": ("logdet throughput, (2n^3/3)/time-to-logdet" if args.general
                   else "logdet throughput, (n^3/3)/time-to-logdet"),
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": sec * 1e3, "ms_per_step_median": float(np.median(pass_ms)),
        "ms_per_step_min": float(np.min(pass_ms)), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64" if widen else w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n": n, "block_size": bs,
                   "placement": ("file (pread/pwrite through pinned chunks), streamed" if args.file_dir else
                                 ("pinned" if pinned else "pageable") + " host memory, streamed; factors " +
                                 ("to a host scratch area (overwrite = 0)" if keep_input else
                                  "over the matrix (overwrite = 1; formed again, untimed, before every pass)"))
                   if out_of_core else "HBM, in-core",
                   "mem_budget_bytes": w.mem_budget, "seed": w.seed,
                   **({"storage": "f32, widened exactly; arithmetic f64"} if widen else {}),
                   **({"form": "positive definite (Cholesky), MDET_FLAG_ASSUME_SPD"} if args.assume_spd else {}),
                   **({"workspace": "MDET_FLAG_SCALED_COPY"} if args.scaled_copy else {}),
                   **({"pivoting": "inside groups of 64, MDET_FLAG_PIVOT"} if args.pivot else {}),
                   **({"pivoting": "over each whole diagonal block, MDET_FLAG_PIVOT_BLOCK"} if args.pivot_block else {}),
                   **({"form": "general matrix (rows shuffled inside groups of 64), P A = L D U, "
                               "MDET_FLAG_GENERAL; value counts 2n^3/3"} if args.general else {})},
        "time_to_logdet_s": sec, "frac_of_matrix_peak": value / peak,
        "logabsdet": final.logabsdet, "sign": final.sign, "negative_pivots": final.negative_pivots,
        "kernel_launches_per_step": final.kernel_launches,
        "roofline": {
            "kernel": "trailing_update_kernel + trailing_update64_kernel (Schur update A_ij -= L_ik D_k L_jk^T "
                      "on MFMA; every launch of both)",
            "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
            "frac": (achieved / peak) if achieved else None,
            "traffic": traffic,
            "busy_s": busy, "flop": f128 + f64b, "share_of_path_flop": (f128 + f64b) / (flop * steps),
            "per_kernel": [
                {"kernel": "trailing_update_kernel", "launches": n128,
                 "flop_per_launch_avg": (f128 / n128) if n128 else None,
                 "avg_launch_ms": (t128 / n128 * 1e3) if n128 else None,
                 "flop_over_sum_of_durations": (f128 / t128 / 1e12) if t128 > 0 else None},
                {"kernel": "trailing_update64_kernel", "launches": n64b,
                 "flop_per_launch_avg": (f64b / n64b) if n64b else None,
                 "avg_launch_ms": (t64b / n64b * 1e3) if n64b else None,
                 "flop_over_sum_of_durations": (f64b / t64b / 1e12) if t64b > 0 else None}],
        },
    }
    if out_of_core:
        if requested != (steps, warmup):
            line["steps_requested"], line["warmup_requested"] = requested
            line["note"] = (f"passes of {sec:.1f} s: warm-up and timed passes cut to fit the "
                            f"{budget_s:.0f} s wall-clock budget of the whole run (--time-budget)")
        line["host_link"] = {"bytes_h2d": final.bytes_h2d, "bytes_d2h": final.bytes_d2h,
                             "GBps_avg_h2d": final.bytes_h2d / sec / 1e9,
                             "seconds_busy_h2d": final.t_h2d, "seconds_busy_d2h": final.t_d2h,
                             "GBps_while_copying_h2d": (final.bytes_h2d / final.t_h2d / 1e9) if final.t_h2d else None,
                             "GBps_while_copying_d2h": (final.bytes_d2h / final.t_d2h / 1e9) if final.t_d2h else None,
                             "dev_bytes_planned": final.dev_bytes_high_water,
                             "superpanels": final.num_superpanels}
        line["in_core"] = incore
    cf = w.closed_form_logdet()
    if cf is not None:
        line["closed_form_rel_err"] = abs(final.logabsdet - cf) / abs(cf)

    if not args.no_cpu_baseline:
        import oracle
        m = args.cpu_sample or min(n, 8192)      # configurations 1 and 2: the whole matrix
        if args.general:
            m = max(64, m // 64 * 64) if n >= 64 else n
        if a is None:
            f = w.factor_torch("cuda")
            sample = w.block_torch(f, 0, m, 0, m, device="cuda").cpu().numpy()
            del f
        else:
            sample = a[:m, :m].cpu().numpy()
        log(f"oracle on the leading {m} x {m} block")
        t0 = time.perf_counter()
        o_sign = None
        if args.general:
            # the leading block of the row-shuffled matrix, eliminated with the same rule
            og = oracle.lu_logdet(sample, group=64)
            o_logabsdet, o_name, o_sign = og.logabsdet, "Gaussian elimination, pivot inside groups of 64", og.sign
        elif args.assume_spd:
            oc = oracle.cholesky_logdet(sample)
            o_logabsdet, o_name = oc.logdet, "Cholesky"
        else:
            o_logabsdet, o_name = oracle.ldlt_logdet(sample).logabsdet, "LDL^T"
        t_cpu = time.perf_counter() - t0
        gpu_partial = float(np.sum(np.log(np.abs(diag_host[:m]))))
        cpu_flop = m ** 3 / 3.0 * (2.0 if args.general else 1.0)
        line["cpu_baseline"] = {
            "value": cpu_flop / t_cpu / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": t_cpu,
            "sample": f"leading principal {m}x{m} block of the same matrix (long-double unblocked {o_name})",
            "extrapolated_seconds_full_size": t_cpu * (n / m) ** 3,
            "extrapolation": "n^3 scaling of the sample's time; not measured",
        }
        line["parity_vs_oracle_rel_err"] = abs(gpu_partial - o_logabsdet) / max(1.0, abs(o_logabsdet))
        if args.general and n == m:
            line["parity_sign_equal"] = bool(o_sign == final.sign)
    line["wall_s_process"] = elapsed()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
