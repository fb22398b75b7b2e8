"""ctypes binding of include/memdet.h: same names, argument marshalling only.

The library must be built (``python paper_2503_04424_amd/build.py`` or
``__graft_entry__.build()``); loading fails loudly otherwise.  There is no CPU
fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass
from typing import Callable, Optional

from . import build as _build

MDET_F32, MDET_F64, MDET_F16, MDET_BF16 = 0, 1, 2, 3
FLAG_NO_LOOKAHEAD = 1
FLAG_FORCE_OUT_OF_CORE = 2
FLAG_PROFILE = 4
FLAG_COMPUTE_F64 = 8
FLAG_ASSUME_SPD = 16
FLAG_SCALED_COPY = 32
FLAG_PIVOT = 64
FLAG_GENERAL = 128
FLAG_PIVOT_BLOCK = 256


class Status:
    OK, EINVAL, EBUDGET, ENOMEM_DEVICE, ENOMEM_HOST, EHIP, ESINGULAR, ENONFINITE, EPROVIDER, ENOTPOSDEF, EIO = range(11)


class _Params(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("dtype", C.c_int32), ("n", C.c_int64),
        ("block_size", C.c_int64), ("mem_budget_bytes", C.c_uint64),
        ("overwrite", C.c_int32), ("reserved0", C.c_int32), ("flags", C.c_uint32),
        ("stream", C.c_void_p), ("dev_workspace", C.c_void_p),
        ("dev_workspace_bytes", C.c_uint64), ("host_scratch", C.c_void_p),
        ("host_scratch_bytes", C.c_uint64), ("perm", C.c_void_p),
    ]


class _Result(C.Structure):
    _fields_ = [
        ("logabsdet", C.c_double), ("sign", C.c_int32), ("hip_error", C.c_int32),
        ("bad_pivot_index", C.c_int64), ("negative_pivots", C.c_int64),
        ("block_size_used", C.c_int64), ("num_blocks", C.c_int64),
        ("out_of_core", C.c_int32), ("num_superpanels", C.c_int32),
        ("flops", C.c_double), ("t_total", C.c_double), ("bytes_h2d", C.c_uint64),
        ("bytes_d2h", C.c_uint64), ("dev_bytes_high_water", C.c_uint64),
        ("kernel_launches", C.c_uint64), ("trailing_update_launches", C.c_uint64),
        ("t_trailing_update", C.c_double), ("trailing_update_flops", C.c_double),
        ("t_h2d", C.c_double), ("t_d2h", C.c_double),
        ("trailing_update64_launches", C.c_uint64), ("t_trailing_update64", C.c_double),
        ("trailing_update64_flops", C.c_double), ("t_trailing_update_busy", C.c_double),
    ]


class _PlanInfo(C.Structure):
    _fields_ = [
        ("block_size_used", C.c_int64), ("num_blocks", C.c_int64),
        ("out_of_core", C.c_int32), ("num_superpanels", C.c_int32),
        ("dev_bytes_needed", C.c_uint64), ("host_bytes_needed", C.c_uint64),
        ("host_matrix_bytes", C.c_uint64), ("stream_bytes_h2d", C.c_uint64),
        ("stream_bytes_d2h", C.c_uint64), ("fma_decomp", C.c_double),
        ("fma_solve", C.c_double), ("fma_gemm", C.c_double), ("fma_syrk", C.c_double),
    ]


PROVIDER_CB = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                          C.c_void_p, C.c_int64)
PROVIDER_DEVICE_CB = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                 C.c_void_p, C.c_int64, C.c_void_p)

EXPORTS = [
    "mdet_plan", "mdet_workspace_query", "mdet_logdet_device", "mdet_logdet_host",
    "mdet_logdet_provider", "mdet_logdet_provider_device", "mdet_logdet_file", "mdet_host_layout_offset", "mdet_paper_block_rule",
    "mdet_paper_fma_count", "mdet_step_schur_update", "mdet_step_panel_factor",
    "mdet_step_panel_factor_pivoted",
    "mdet_step_panel_factor_general",
    "mdet_step_logdet_reduce", "mdet_strerror", "mdet_version",
    "mdet_sequence_workspace_query", "mdet_principal_logdets", "mdet_flodance_fit",
    "mdet_flodance_eval", "mdet_step_copy", "mdet_step_mfma_peak",
    "mdet_logdet_device_noalloc",
]

_lib = None


def lib_path() -> str:
    return _build.lib_path()


def load():
    """Loads libmemdet.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not built: run `python paper_2503_04424_amd/build.py`")
    L = C.CDLL(path)
    vp, i64, i32, u64 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64
    L.mdet_plan.argtypes = [C.POINTER(_Params), C.c_int, C.POINTER(_PlanInfo)]
    L.mdet_workspace_query.argtypes = [C.POINTER(_Params), C.c_int, C.POINTER(u64), C.POINTER(u64)]
    L.mdet_logdet_device.argtypes = [C.POINTER(_Params), vp, i64, C.POINTER(_Result), vp]
    L.mdet_logdet_host.argtypes = [C.POINTER(_Params), vp, C.POINTER(_Result), vp]
    L.mdet_logdet_provider.argtypes = [C.POINTER(_Params), PROVIDER_CB, vp, C.POINTER(_Result), vp]
    L.mdet_logdet_provider_device.argtypes = [C.POINTER(_Params), PROVIDER_DEVICE_CB, vp, C.POINTER(_Result), vp]
    L.mdet_logdet_file.argtypes = [C.POINTER(_Params), C.c_char_p, C.c_char_p, C.POINTER(_Result), vp]
    L.mdet_host_layout_offset.argtypes = [i64, i64, i64]
    L.mdet_host_layout_offset.restype = i64
    L.mdet_paper_block_rule.argtypes = [i64, i32, u64, C.POINTER(i64), C.POINTER(i64)]
    L.mdet_paper_fma_count.argtypes = [i64]
    L.mdet_paper_fma_count.restype = C.c_double
    L.mdet_step_schur_update.argtypes = [i32, vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, i32, vp]
    L.mdet_step_panel_factor.argtypes = [i32, vp, i64, i64, i64, vp, vp, i64, vp, vp]
    L.mdet_step_panel_factor_pivoted.argtypes = [i32, vp, i64, i64, i64, vp, vp, vp, i64, vp, vp]
    L.mdet_step_panel_factor_general.argtypes = [i32, vp, vp, i64, i64, i64, vp, vp, vp, i64, vp, vp]
    L.mdet_step_logdet_reduce.argtypes = [i32, vp, i64, vp, vp]
    L.mdet_sequence_workspace_query.argtypes = [i64, i64, i32, C.POINTER(u64)]
    L.mdet_principal_logdets.argtypes = [i32, vp, i64, vp, vp, u64, vp]
    L.mdet_flodance_fit.argtypes = [vp, i64, i64, i64, i64, i32, vp, vp, u64, vp]
    L.mdet_flodance_eval.argtypes = [vp, i32, vp, i64, vp, vp]
    L.mdet_logdet_device_noalloc.argtypes = [C.POINTER(_Params), vp, i64, vp, vp]
    L.mdet_step_copy.argtypes = [vp, vp, u64, vp]
    L.mdet_step_mfma_peak.argtypes = [i32, i32, i32, i32, vp, C.POINTER(C.c_double), vp]
    L.mdet_strerror.argtypes = [C.c_int]
    L.mdet_strerror.restype = C.c_char_p
    L.mdet_version.restype = C.c_char_p
    for name in EXPORTS:
        fn = getattr(L, name)      # raises if the library misses a declared symbol
        if name not in ("mdet_host_layout_offset", "mdet_paper_fma_count", "mdet_strerror", "mdet_version"):
            fn.restype = C.c_int
    _lib = L
    return L


def lib():
    return load()


class MemdetError(RuntimeError):
    def __init__(self, status: int, result=None):
        self.status = status
        self.result = result
        msg = load().mdet_strerror(status).decode()
        if result is not None and result.hip_error:
            msg += f" [hipError {result.hip_error}]"
        super().__init__(f"memdet status {status}: {msg}")


@dataclass
class LogdetResult:
    logabsdet: float
    sign: int
    status: int
    bad_pivot_index: int
    negative_pivots: int
    block_size_used: int
    num_blocks: int
    out_of_core: bool
    num_superpanels: int
    flops: float
    t_total: float
    bytes_h2d: int
    bytes_d2h: int
    dev_bytes_high_water: int
    kernel_launches: int
    hip_error: int = 0
    trailing_update_launches: int = 0
    t_trailing_update: float = 0.0
    trailing_update_flops: float = 0.0
    t_h2d: float = 0.0
    t_d2h: float = 0.0
    trailing_update64_launches: int = 0
    t_trailing_update64: float = 0.0
    trailing_update64_flops: float = 0.0
    t_trailing_update_busy: float = 0.0


@dataclass
class PlanInfo:
    block_size_used: int
    num_blocks: int
    out_of_core: bool
    num_superpanels: int
    dev_bytes_needed: int
    host_bytes_needed: int
    host_matrix_bytes: int
    stream_bytes_h2d: int
    stream_bytes_d2h: int
    fma_decomp: float
    fma_solve: float
    fma_gemm: float
    fma_syrk: float


def _dtype_code(dtype) -> int:
    if isinstance(dtype, int):
        if dtype in (MDET_F32, MDET_F64, MDET_F16, MDET_BF16):
            return dtype
        raise ValueError(f"unsupported dtype {dtype!r}")
    s = str(dtype)
    if s in ("f64", "float64", "torch.float64"):
        return MDET_F64
    if s in ("f32", "float32", "torch.float32"):
        return MDET_F32
    if s in ("f16", "float16", "torch.float16"):
        return MDET_F16
    if s in ("bf16", "bfloat16", "torch.bfloat16"):
        return MDET_BF16
    raise ValueError(f"unsupported dtype {dtype!r}")


def _params(n, dtype, block_size=0, mem_budget=0, overwrite=True, flags=0, stream=None,
            dev_workspace=None, dev_workspace_bytes=0, host_scratch=None, host_scratch_bytes=0,
            perm=None):
    p = _Params()
    p.struct_size = C.sizeof(_Params)
    p.dtype = _dtype_code(dtype)
    p.n = int(n)
    p.block_size = int(block_size)
    p.mem_budget_bytes = int(mem_budget)
    p.overwrite = 1 if overwrite else 0
    p.flags = int(flags)
    p.stream = stream
    p.dev_workspace = dev_workspace
    p.dev_workspace_bytes = int(dev_workspace_bytes)
    p.host_scratch = host_scratch
    p.host_scratch_bytes = int(host_scratch_bytes)
    p.perm = perm
    return p


def _result(status: int, r: _Result) -> LogdetResult:
    return LogdetResult(r.logabsdet, r.sign, status, r.bad_pivot_index, r.negative_pivots,
                        r.block_size_used, r.num_blocks, bool(r.out_of_core), r.num_superpanels,
                        r.flops, r.t_total, r.bytes_h2d, r.bytes_d2h, r.dev_bytes_high_water,
                        r.kernel_launches, r.hip_error, r.trailing_update_launches,
                        r.t_trailing_update, r.trailing_update_flops, r.t_h2d, r.t_d2h,
                        r.trailing_update64_launches, r.t_trailing_update64, r.trailing_update64_flops,
                        r.t_trailing_update_busy)


_SOFT = (Status.OK, Status.ESINGULAR, Status.ENONFINITE, Status.ENOTPOSDEF)


def mdet_strerror(status: int) -> str:
    return load().mdet_strerror(int(status)).decode()


def mdet_version() -> str:
    return load().mdet_version().decode()


def mdet_plan(n, dtype, block_size=0, mem_budget=0, overwrite=True, flags=0,
              for_device_input=False) -> PlanInfo:
    p = _params(n, dtype, block_size, mem_budget, overwrite, flags)
    info = _PlanInfo()
    st = load().mdet_plan(C.byref(p), 1 if for_device_input else 0, C.byref(info))
    if st != Status.OK:
        raise MemdetError(st)
    return PlanInfo(*[getattr(info, f[0]) for f in _PlanInfo._fields_][:2],
                    bool(info.out_of_core), info.num_superpanels, info.dev_bytes_needed,
                    info.host_bytes_needed, info.host_matrix_bytes, info.stream_bytes_h2d,
                    info.stream_bytes_d2h, info.fma_decomp, info.fma_solve, info.fma_gemm,
                    info.fma_syrk)


def mdet_workspace_query(n, dtype, block_size=0, mem_budget=0, overwrite=True, flags=0,
                         for_device_input=False):
    p = _params(n, dtype, block_size, mem_budget, overwrite, flags)
    d, h = C.c_uint64(0), C.c_uint64(0)
    st = load().mdet_workspace_query(C.byref(p), 1 if for_device_input else 0, C.byref(d), C.byref(h))
    if st != Status.OK:
        raise MemdetError(st)
    return d.value, h.value


def _stream_handle(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def _perm_ptr(perm, n, on_device):
    import torch
    if perm is None:
        return None
    if perm.dtype != torch.int32 or perm.numel() < n or perm.is_cuda != on_device or not perm.is_contiguous():
        raise ValueError("perm must be a contiguous int32 tensor of n elements, on the %s"
                         % ("GPU" if on_device else "host"))
    return perm.data_ptr()


def mdet_logdet_device(a, block_size=0, mem_budget=0, overwrite=False, flags=0, diag=None,
                       stream=None, workspace=None, raise_on_error=True, perm=None) -> LogdetResult:
    """log|det| and sign of the symmetric matrix whose lower triangle is in the
    2-D CUDA tensor ``a`` (float64 / float32, row-major, unit column stride).
    ``perm`` (int32 CUDA tensor, with FLAG_PIVOT or FLAG_GENERAL) receives the permutation.
    With FLAG_GENERAL ``a`` is a general matrix and all of it is read."""
    if a.dim() != 2 or a.shape[0] != a.shape[1] or not a.is_cuda or (a.numel() and a.stride(1) != 1):
        raise ValueError("square row-major CUDA tensor expected")
    n = a.shape[0]
    ld = a.stride(0) if n > 1 else max(n, 1)
    p = _params(n, a.dtype, block_size, mem_budget, overwrite, flags, _stream_handle(stream),
                workspace.data_ptr() if workspace is not None else None,
                workspace.numel() * workspace.element_size() if workspace is not None else 0,
                perm=_perm_ptr(perm, n, True))
    import torch
    diag_dtype = torch.float64 if (flags & FLAG_COMPUTE_F64) else a.dtype
    if diag is not None and (diag.dtype != diag_dtype or diag.numel() < n or not diag.is_cuda):
        raise ValueError("diag must be a CUDA tensor of n elements of the arithmetic's dtype")
    r = _Result()
    st = load().mdet_logdet_device(C.byref(p), C.c_void_p(a.data_ptr()), ld, C.byref(r),
                                   C.c_void_p(diag.data_ptr()) if diag is not None else None)
    if st not in _SOFT and raise_on_error:
        raise MemdetError(st, r)
    return _result(st, r)


def mdet_logdet_device_noalloc(a, out, block_size=0, flags=0, diag=None, stream=None, perm=None) -> int:
    """Queues the in-place factorisation of ``a`` on ``stream`` without allocating anything;
    ``out``: 5 float64 on the GPU (log|det|, sign, negative pivots, first bad pivot, status).
    Returns the status of the queueing itself."""
    if a.dim() != 2 or a.shape[0] != a.shape[1] or not a.is_cuda or (a.numel() and a.stride(1) != 1):
        raise ValueError("square row-major CUDA tensor expected")
    import torch
    if out.dtype != torch.float64 or out.numel() < 5 or not out.is_cuda:
        raise ValueError("out must be a CUDA tensor of 5 float64")
    n = a.shape[0]
    ld = a.stride(0) if n > 1 else max(n, 1)
    p = _params(n, a.dtype, block_size, 0, True, flags, _stream_handle(stream), perm=_perm_ptr(perm, n, True))
    return load().mdet_logdet_device_noalloc(C.byref(p), C.c_void_p(a.data_ptr()), ld, C.c_void_p(out.data_ptr()),
                                             C.c_void_p(diag.data_ptr()) if diag is not None else None)


def mdet_logdet_host(packed, n, block_size, mem_budget=0, overwrite=True, flags=0, diag=None,
                     stream=None, workspace=None, host_scratch=None, raise_on_error=True,
                     perm=None) -> LogdetResult:
    """``packed``: 1-D CPU tensor (ideally pinned) in the packed lower block-column layout."""
    if packed.is_cuda or packed.dim() != 1:
        raise ValueError("1-D host tensor expected")
    p = _params(n, packed.dtype, block_size, mem_budget, overwrite, flags, _stream_handle(stream),
                workspace.data_ptr() if workspace is not None else None,
                workspace.numel() * workspace.element_size() if workspace is not None else 0,
                host_scratch.data_ptr() if host_scratch is not None else None,
                host_scratch.numel() * host_scratch.element_size() if host_scratch is not None else 0,
                perm=_perm_ptr(perm, n, False))
    # the block size the library will use (0 = its own choice), for the size check only
    info = _PlanInfo()
    st = load().mdet_plan(C.byref(p), 0, C.byref(info))
    if st != Status.OK:
        if raise_on_error:
            raise MemdetError(st)
        return _result(st, _Result())
    b = info.block_size_used
    need = mdet_host_layout_offset(n, b, (n + b - 1) // b) if n > 0 else 0
    if flags & FLAG_GENERAL:
        need *= 2          # the layout of the matrix, then the layout of its transpose
    if packed.numel() < need:
        raise ValueError(f"packed layout needs {need} elements")
    import torch
    diag_dtype = torch.float64 if (flags & FLAG_COMPUTE_F64) else packed.dtype
    if diag is not None and (diag.dtype != diag_dtype or diag.numel() < n or diag.is_cuda):
        raise ValueError("diag must be a host tensor of n elements of the arithmetic's dtype")
    r = _Result()
    st = load().mdet_logdet_host(C.byref(p), C.c_void_p(packed.data_ptr()), C.byref(r),
                                 C.c_void_p(diag.data_ptr()) if diag is not None else None)
    if st not in _SOFT and raise_on_error:
        raise MemdetError(st, r)
    return _result(st, r)


def mdet_logdet_provider(provider: Callable, n, dtype, block_size, mem_budget=0, flags=0,
                         diag=None, stream=None, raise_on_error=True, perm=None) -> LogdetResult:
    """``provider(bi, bj, rows, cols, dst_ptr, ld) -> int`` fills one block (host memory)."""
    def _cb(user, bi, bj, rows, cols, dst, ld):
        try:
            return int(provider(bi, bj, rows, cols, dst, ld) or 0)
        except Exception:  # never let an exception cross the C boundary
            return -1
    cb = PROVIDER_CB(_cb)
    p = _params(n, dtype, block_size, mem_budget, True, flags, _stream_handle(stream),
                perm=_perm_ptr(perm, n, False))
    r = _Result()
    st = load().mdet_logdet_provider(C.byref(p), cb, None, C.byref(r),
                                     C.c_void_p(diag.data_ptr()) if diag is not None else None)
    if st not in _SOFT and raise_on_error:
        raise MemdetError(st, r)
    return _result(st, r)


def mdet_logdet_provider_device(provider: Callable, n, dtype, block_size, mem_budget=0, flags=0,
                                diag=None, stream=None, raise_on_error=True, perm=None) -> LogdetResult:
    """``provider(bi, bj, rows, cols, dst_device_ptr, ld, stream_handle) -> int`` queues on the stream
    it is handed the work that fills one block in device memory."""
    def _cb(user, bi, bj, rows, cols, dst, ld, st):
        try:
            return int(provider(bi, bj, rows, cols, dst, ld, st) or 0)
        except Exception:  # never let an exception cross the C boundary
            return -1
    cb = PROVIDER_DEVICE_CB(_cb)
    p = _params(n, dtype, block_size, mem_budget, True, flags, _stream_handle(stream),
                perm=_perm_ptr(perm, n, False))
    r = _Result()
    st = load().mdet_logdet_provider_device(C.byref(p), cb, None, C.byref(r),
                                            C.c_void_p(diag.data_ptr()) if diag is not None else None)
    if st not in _SOFT and raise_on_error:
        raise MemdetError(st, r)
    return _result(st, r)


def mdet_logdet_file(matrix_path, n, dtype, block_size, mem_budget=0, overwrite=True, flags=0, diag=None,
                     scratch_path=None, stream=None, workspace=None, raise_on_error=True,
                     perm=None) -> LogdetResult:
    """The matrix in a file holding the packed lower block-column layout (see mdet_logdet_host)."""
    p = _params(n, dtype, block_size, mem_budget, overwrite, flags, _stream_handle(stream),
                workspace.data_ptr() if workspace is not None else None,
                workspace.numel() * workspace.element_size() if workspace is not None else 0,
                perm=_perm_ptr(perm, n, False))
    if diag is not None and (diag.numel() < n or diag.is_cuda):
        raise ValueError("diag must be a host tensor of n elements of the matrix dtype")
    r = _Result()
    st = load().mdet_logdet_file(C.byref(p), os.fsencode(matrix_path),
                                 os.fsencode(scratch_path) if scratch_path is not None else None,
                                 C.byref(r), C.c_void_p(diag.data_ptr()) if diag is not None else None)
    if st not in _SOFT and raise_on_error:
        raise MemdetError(st, r)
    return _result(st, r)


def mdet_host_layout_offset(n, b, j) -> int:
    return load().mdet_host_layout_offset(int(n), int(b), int(j))


def mdet_paper_block_rule(m, beta, c):
    nb, b = C.c_int64(0), C.c_int64(0)
    st = load().mdet_paper_block_rule(int(m), int(beta), int(c), C.byref(nb), C.byref(b))
    if st != Status.OK:
        raise MemdetError(st)
    return nb.value, b.value


def mdet_paper_fma_count(m) -> float:
    return load().mdet_paper_fma_count(int(m))


def mdet_step_schur_update(c, a, b, d, lower=False, stream=None) -> None:
    """c[M,N] -= a[M,K] diag(d) b[N,K]^T on the GPU (asynchronous); d=None: c -= a b^T."""
    M, K = a.shape
    N = b.shape[0]
    st = load().mdet_step_schur_update(_dtype_code(c.dtype), c.data_ptr(), c.stride(0), a.data_ptr(),
                                       a.stride(0), b.data_ptr(), b.stride(0),
                                       d.data_ptr() if d is not None else None, M, N, K,
                                       1 if lower else 0, _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)


def mdet_step_panel_factor(panel, w, d, dinv, flags_buf, pivot_index0=0, stream=None) -> None:
    """In-place factorisation of a block column (m x >=w tensor view, first w columns)."""
    m = panel.shape[0]
    st = load().mdet_step_panel_factor(_dtype_code(panel.dtype), panel.data_ptr(), panel.stride(0), m,
                                       int(w), d.data_ptr(), dinv.data_ptr(), int(pivot_index0),
                                       flags_buf.data_ptr(), _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)


def mdet_step_panel_factor_pivoted(panel, w, d, dinv, perm, flags_buf, pivot_index0=0, stream=None) -> None:
    """As mdet_step_panel_factor with pivoting inside each 64-column leaf; perm: int32, w entries."""
    m = panel.shape[0]
    st = load().mdet_step_panel_factor_pivoted(_dtype_code(panel.dtype), panel.data_ptr(), panel.stride(0),
                                               m, int(w), d.data_ptr(), dinv.data_ptr(),
                                               _perm_ptr(perm, int(w), True), int(pivot_index0),
                                               flags_buf.data_ptr(), _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)


def mdet_step_panel_factor_general(lower, upper_t, w, d, dinv, perm, flags_buf, pivot_index0=0, stream=None) -> None:
    """One block column of a general matrix: ``lower`` (m x >= w, entries on and below the
    diagonal) and ``upper_t`` (same shape and row stride, the transposed entries above it);
    flags_buf: 32 + 16384 bytes, uint64 [0], [1] all-ones and [2] zero on entry."""
    m = lower.shape[0]
    if upper_t.shape[0] != m or upper_t.stride(0) != lower.stride(0) or upper_t.dtype != lower.dtype:
        raise ValueError("the two panels must have the same shape, row stride and dtype")
    st = load().mdet_step_panel_factor_general(_dtype_code(lower.dtype), lower.data_ptr(), upper_t.data_ptr(),
                                               lower.stride(0), m, int(w), d.data_ptr(), dinv.data_ptr(),
                                               _perm_ptr(perm, int(w), True), int(pivot_index0),
                                               flags_buf.data_ptr(), _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)


def mdet_step_logdet_reduce(d, out, stream=None) -> None:
    """out (>= 8 float64 on the GPU): [0]=sum log|d|, [1]=sign, [2]=negative count."""
    st = load().mdet_step_logdet_reduce(_dtype_code(d.dtype), d.data_ptr(), d.numel(), out.data_ptr(),
                                        _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)


def mdet_sequence_workspace_query(n=0, rows=0, q=0) -> int:
    """Device bytes of workspace for mdet_principal_logdets (n pivots) and
    mdet_flodance_fit (rows = n_s - n_0 samples, q correction terms)."""
    b = C.c_uint64(0)
    st = load().mdet_sequence_workspace_query(int(n), int(rows), int(q), C.byref(b))
    if st != Status.OK:
        raise MemdetError(st)
    return b.value


def _sequence_workspace(n, rows, q, like):
    import torch
    return torch.empty(max(256, mdet_sequence_workspace_query(n, rows, q)), dtype=torch.uint8,
                       device=like.device)


def mdet_principal_logdets(diag, ell=None, workspace=None, stream=None):
    """ell[k] = sum_{i<=k} log|diag[i]| on the GPU (asynchronous); returns ell (float64)."""
    import torch
    n = diag.numel()
    if ell is None:
        ell = torch.empty(n, dtype=torch.float64, device=diag.device)
    ws = workspace if workspace is not None else _sequence_workspace(n, 0, 0, diag)
    st = load().mdet_principal_logdets(_dtype_code(diag.dtype), diag.data_ptr(), n, ell.data_ptr(),
                                       ws.data_ptr(), ws.numel() * ws.element_size(),
                                       _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)
    return ell


def mdet_flodance_fit(ell, d, n0, ns, q, coef=None, workspace=None, stream=None):
    """The regression of Alg. 2 on the GPU (asynchronous); returns the q + 4 float64
    (c_0, nu_0 .. nu_q, L_{n0}, residual norm) as a device tensor."""
    import torch
    if coef is None:
        coef = torch.empty(max(int(q), 0) + 4, dtype=torch.float64, device=ell.device)
    ws = workspace if workspace is not None else _sequence_workspace(0, max(int(ns) - int(n0), 0),
                                                                     min(max(int(q), 0), 10), ell)
    st = load().mdet_flodance_fit(ell.data_ptr(), ell.numel(), int(d), int(n0), int(ns), int(q),
                                  coef.data_ptr(), ws.data_ptr(), ws.numel() * ws.element_size(),
                                  _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)
    return coef


def mdet_flodance_eval(coef, q, n_values, out=None, stream=None):
    """Lhat_n at every entry of n_values (float64 device tensor), on the GPU (asynchronous)."""
    import torch
    if out is None:
        out = torch.empty_like(n_values)
    st = load().mdet_flodance_eval(coef.data_ptr(), int(q), n_values.data_ptr(), n_values.numel(),
                                   out.data_ptr(), _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)
    return out


def mdet_step_copy(dst, src, stream=None) -> None:
    """dst <- src by the library's plain copy kernel (asynchronous); same byte size, a multiple of 16."""
    nb = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nb:
        raise ValueError("dst and src must have the same size in bytes")
    st = load().mdet_step_copy(dst.data_ptr(), src.data_ptr(), nb, _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)


def mdet_step_mfma_peak(dtype, workgroups, iters, out, accumulators=4, stream=None) -> float:
    """Queues the register-only matrix-core loop; returns the flops of the launch."""
    f = C.c_double(0.0)
    st = load().mdet_step_mfma_peak(_dtype_code(dtype), int(accumulators), int(workgroups), int(iters),
                                    out.data_ptr(), C.byref(f), _stream_handle(stream))
    if st != Status.OK:
        raise MemdetError(st)
    return f.value


def pack_general_block_columns(a, block_size: int, pin: bool = False):
    """Host layout of a general matrix for ``mdet_logdet_host`` with FLAG_GENERAL: the packed
    lower block-column layout of ``a`` followed by that of its transpose.  Layout marshalling only."""
    import torch
    n = a.shape[0]
    b = (int(block_size) + 63) // 64 * 64
    T = (n + b - 1) // b if n > 0 else 0
    total = mdet_host_layout_offset(n, b, T) if n > 0 else 0
    out = torch.empty(max(2 * total, 1), dtype=a.dtype, pin_memory=pin)
    pack_lower_block_columns(a, block_size, out=out[:max(total, 1)])
    pack_lower_block_columns(a.t(), block_size, out=out[total:] if total else out)
    return out


def pack_lower_block_columns(a, block_size: int, out=None, pin: bool = False):
    """Re-lays a dense 2-D tensor (CPU or CUDA) into the packed lower block-column
    host layout of ``mdet_logdet_host``.  Layout marshalling only."""
    import torch
    n = a.shape[0]
    b = (int(block_size) + 63) // 64 * 64
    T = (n + b - 1) // b if n > 0 else 0
    total = mdet_host_layout_offset(n, b, T) if n > 0 else 0
    if out is None:
        out = torch.empty(max(total, 1), dtype=a.dtype, pin_memory=pin)
    for j in range(T):
        w = min(b, n - j * b)
        off = mdet_host_layout_offset(n, b, j)
        rows = n - j * b
        out[off:off + rows * w].view(rows, w).copy_(a[j * b:, j * b:j * b + w])
    return out
