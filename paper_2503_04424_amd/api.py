"""A front end with the call shape of the paper's software appendix (``memdet(M, max_mem,
assume, triangle, overwrite, mixed_precision, ...)`` returning ``ld, sign, diag, perm[, info]``)
on top of the C ABI.  Argument marshalling only: it chooses the entry point and the flags,
lays a host matrix out in block columns, and turns the result struct into the tuple; every
step of the computation runs in the library.

Where the paper's call and this one differ:
  * ``M`` is a square CUDA tensor (resident: ``mdet_logdet_device``), or a CPU tensor / numpy
    array (``mdet_logdet_host`` on its packed block-column layout, streamed if it does not
    fit ``max_mem``).  Stores on disk go through ``mdet_logdet_file`` directly.
  * pivoting is off unless asked for (``pivot='leaf'`` or ``'block'``): ``perm`` is then the
    identity, and ``diag`` the pivots of the unpivoted factorisation (Sec. 2.2 pivots inside a
    block only; the determinant does not depend on it).
  * ``scratch_dir`` and ``parallel_io`` belong to the file entry point and are not taken here.
"""
import re

from . import binding as B

_UNITS = {"": 1, "B": 1, "KB": 10 ** 3, "MB": 10 ** 6, "GB": 10 ** 9, "TB": 10 ** 12,
          "KIB": 2 ** 10, "MIB": 2 ** 20, "GIB": 2 ** 30, "TIB": 2 ** 40}


def parse_bytes(max_mem) -> int:
    """``'32GB'``, ``'16GiB'``, a number of bytes, or None / inf for no limit (0)."""
    if max_mem is None:
        return 0
    if isinstance(max_mem, str):
        m = re.fullmatch(r"\s*([0-9]*\.?[0-9]+)\s*([A-Za-z]*)\s*", max_mem)
        if not m or m.group(2).upper() not in _UNITS:
            raise ValueError(f"cannot read a size from {max_mem!r}")
        return int(float(m.group(1)) * _UNITS[m.group(2).upper()])
    if max_mem == float("inf"):
        return 0
    return int(max_mem)


def memdet(M, max_mem=None, assume="gen", triangle=None, overwrite=False, mixed_precision=None,
           block_size=0, pivot=None, return_info=False, stream=None):
    """``ld, sign, diag, perm`` (and ``info`` with ``return_info``) of the square matrix ``M``.

    assume: 'gen' (P M = L D U), 'sym' (L D L^T) or 'spd' (Cholesky form).
    triangle: for 'sym' / 'spd', 'l' or None reads the lower triangle, 'u' the upper one.
    mixed_precision: 'float64' runs fp64 arithmetic on a matrix stored in fp32 / fp16 / bf16
    (App. C); None or the matrix's own type computes in that type.
    """
    import numpy as np
    import torch
    if isinstance(M, np.ndarray):
        M = torch.from_numpy(M)
    if M.dim() != 2 or M.shape[0] != M.shape[1]:
        raise ValueError("a square matrix is expected")
    n = M.shape[0]
    if assume not in ("gen", "sym", "spd"):
        raise ValueError("assume must be 'gen', 'sym' or 'spd'")
    if triangle not in (None, "l", "u"):
        raise ValueError("triangle must be None, 'l' or 'u'")
    flags = {"gen": B.FLAG_GENERAL, "sym": 0, "spd": B.FLAG_ASSUME_SPD}[assume]
    if pivot is not None:
        if assume != "sym" or pivot not in ("leaf", "block"):
            raise ValueError("pivot='leaf' or 'block' goes with assume='sym'")
        flags |= B.FLAG_PIVOT if pivot == "leaf" else B.FLAG_PIVOT_BLOCK
    wide = mixed_precision in ("float64", "f64", torch.float64)
    if mixed_precision not in (None, "float64", "f64", torch.float64, "float32", "f32", torch.float32):
        raise ValueError("mixed_precision must be None, 'float32' or 'float64'")
    if wide and M.dtype != torch.float64:
        flags |= B.FLAG_COMPUTE_F64
    elif not wide and mixed_precision is not None and M.dtype != torch.float32:
        raise ValueError("arithmetic narrower than the storage is not offered")
    if triangle == "u" and assume != "gen":
        M = M.t()                       # the upper triangle of M is the lower triangle of its transpose
    budget = parse_bytes(max_mem)
    arith = torch.float64 if (flags & B.FLAG_COMPUTE_F64) else M.dtype
    want_perm = bool(flags & (B.FLAG_PIVOT | B.FLAG_PIVOT_BLOCK | B.FLAG_GENERAL))
    if M.is_cuda:
        a = M if (M.stride(1) == 1 or n <= 1) else M.contiguous()
        if a is not M:
            overwrite = True            # the library may work in the copy just made
        diag = torch.empty(n, dtype=arith, device="cuda")
        perm = torch.full((n,), -1, dtype=torch.int32, device="cuda") if want_perm else None
        r = B.mdet_logdet_device(a, block_size=block_size, mem_budget=budget, overwrite=overwrite, flags=flags,
                                 diag=diag, perm=perm, stream=stream, raise_on_error=False)
        diag = diag.cpu()
        perm = perm.cpu() if want_perm else None
    else:
        bs = B.mdet_plan(n, M.dtype, block_size, budget, flags=flags).block_size_used if n > 0 else 64
        pack = B.pack_general_block_columns if assume == "gen" else B.pack_lower_block_columns
        packed = pack(M, bs)
        diag = torch.empty(n, dtype=arith)
        perm = torch.full((n,), -1, dtype=torch.int32) if want_perm else None
        r = B.mdet_logdet_host(packed, n, bs, mem_budget=budget, overwrite=True, flags=flags, diag=diag,
                               perm=perm, stream=stream, raise_on_error=False)
    if r.status not in (B.Status.OK, B.Status.ESINGULAR):
        raise B.MemdetError(r.status, r)
    perm_out = perm.numpy().astype("int64") if want_perm else np.arange(n, dtype="int64")
    out = (r.logabsdet, r.sign, diag.numpy(), perm_out)
    if return_info:
        import dataclasses
        return out + (dataclasses.asdict(r),)
    return out


class FitLogdet:
    """The regression of Alg. 2 behind the ``fit`` / ``eval`` pair of the software appendix:
    ``fit(n, ell)`` takes consecutive integers ``n`` (the fit interval) and the log-determinants
    ``ell`` of the leading principal blocks of those orders (every d-th cumulative sum of
    ``log|diag|``, already sub-sampled by the caller as in the appendix); ``eval(n)`` returns the
    extrapolated log-determinants ``n * Lhat_n``.  Both run in the library (``mdet_flodance_fit``,
    ``mdet_flodance_eval``); this class only arranges the arrays."""

    def __init__(self, q: int = 0):
        self.q = int(q)
        self.coef = None

    def fit(self, n, ell):
        import numpy as np
        import torch
        n = np.asarray(n)
        ell = np.asarray(ell, dtype=np.float64)
        ni = np.rint(n).astype(np.int64)
        if n.ndim != 1 or n.shape != ell.shape or n.size < self.q + 3 or np.any(ni != n) or \
                np.any(np.diff(ni) != 1) or ni[0] < 1:
            raise ValueError("n must be consecutive integers >= 1, with one log-determinant each")
        # the library reads ell[j - 1] for j = n0 .. ns (one sample per order: d = 1)
        full = np.zeros(int(ni[-1]), dtype=np.float64)
        full[ni - 1] = ell
        self.coef = B.mdet_flodance_fit(torch.from_numpy(full).cuda(), 1, int(ni[0]), int(ni[-1]), self.q)
        return self

    def eval(self, n):
        import numpy as np
        import torch
        if self.coef is None:
            raise ValueError("fit first")
        nv = torch.from_numpy(np.asarray(n, dtype=np.float64).reshape(-1).copy()).cuda()
        lhat = B.mdet_flodance_eval(self.coef, self.q, nv)
        return (lhat * nv).cpu().numpy().reshape(np.shape(n))

    @property
    def parameters(self):
        """c_0, nu_0 .. nu_q, L_{n0}, residual norm, as the library returns them."""
        return None if self.coef is None else self.coef.cpu().numpy()
