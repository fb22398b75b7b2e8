"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only *builds matrices*; it holds none of the log-determinant
method's arithmetic and imports neither the GPU library nor the oracle.  Both
sides are always handed the same matrix bits: small cases are formed once on
the CPU with numpy, large ones are formed tile by tile with torch on whatever
device the caller names and sampled sub-blocks are downloaded for the oracle.

The matrices stand in for the workloads of the paper (NTK Gram matrices
J J^T, Sec. 2.1; a Matern Gaussian-process covariance, App. G.2; generic SPD
matrices of order 2^10..2^16, App. E.3), whose real data are not available
here.  Shapes, spectra and conditioning follow the benchmark configurations.

Random factors come from numpy's counter-based Philox generator keyed by the
seed, so a given (seed, shape) always yields the same factor on any machine.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def normal_factor(rows: int, cols: int, seed: int, chunk_rows: int = 8192) -> np.ndarray:
    """rows x cols iid N(0,1), float64, generated in row chunks (same stream)."""
    g = _rng(seed)
    out = np.empty((rows, cols), dtype=np.float64)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = g.standard_normal((r1 - r0, cols))
    return out


def uniform_points(n: int, dim: int, seed: int) -> np.ndarray:
    return _rng(seed).random((n, dim))


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------
@dataclass
class Workload:
    """A symmetric positive-definite test matrix given by compact factors.

    kind:
      'gram'    K = F F^T / p + shift I,  F = G * colscale   (F is n x p)
      'se'      K_ij = exp(-|x_i-x_j|^2 / (2 ell^2)) + shift delta_ij
      'matern32' K_ij = (1 + sqrt3 r/ell) exp(-sqrt3 r/ell) + shift delta_ij
      'kms'     K_ij = rho^|i-j|   (Kac-Murdock-Szego / AR(1))
    """
    name: str
    kind: str
    n: int
    dtype: str = "f64"          # storage/compute type the library is run in
    block_size: int = 128
    seed: int = 0
    p: int = 0                  # gram: inner dimension
    decay: float = 0.0          # gram: column k (1-based) scaled by k^-decay
    shift: float = 0.0
    dim: int = 0                # kernels: point dimension
    ell: float = 1.0            # kernels: length scale
    rho: float = 0.0            # kms
    mem_budget: int = 0         # bytes; 0 = unconstrained (in-core)
    _factor: Optional[np.ndarray] = field(default=None, repr=False)

    # ---- factors (CPU, float64) ------------------------------------------
    def factor(self) -> Optional[np.ndarray]:
        if self._factor is None:
            if self.kind == "gram":
                f = normal_factor(self.n, self.p, self.seed)
                if self.decay != 0.0:
                    f *= np.arange(1, self.p + 1, dtype=np.float64) ** (-self.decay)
                self._factor = f
            elif self.kind in ("se", "matern32"):
                self._factor = uniform_points(self.n, self.dim, self.seed)
        return self._factor

    # ---- dense formation on the CPU (numpy, float64 then cast) -----------
    def dense(self) -> np.ndarray:
        """Full n x n matrix in this workload's dtype (small n only)."""
        return self.block_numpy(0, self.n, 0, self.n)

    def np_dtype(self):
        return np.float64 if self.dtype == "f64" else np.float32

    def block_numpy(self, r0: int, r1: int, c0: int, c1: int) -> np.ndarray:
        k = self._block(_NumpyNS(), self.factor(), r0, r1, c0, c1)
        return np.ascontiguousarray(k.astype(self.np_dtype()))

    # ---- tile formation with torch on a device ---------------------------
    def factor_torch(self, device):
        import torch
        f = self.factor()
        return None if f is None else torch.from_numpy(f).to(device)

    def block_torch(self, f_dev, r0: int, r1: int, c0: int, c1: int, device=None):
        """K[r0:r1, c0:c1] as a torch tensor of this workload's dtype.

        ``f_dev`` is ``factor_torch(device)`` (None for 'kms', then pass device).
        """
        import torch
        k = self._block(_TorchNS(torch, device if f_dev is None else f_dev.device),
                        f_dev, r0, r1, c0, c1)
        return k.to(torch.float64 if self.dtype == "f64" else torch.float32)

    # ---- the formulas (array-namespace generic) --------------------------
    def _block(self, xp, f, r0, r1, c0, c1):
        if self.kind == "gram":
            k = (f[r0:r1] @ f[c0:c1].T) / float(self.p)
        elif self.kind in ("se", "matern32"):
            a, b = f[r0:r1], f[c0:c1]
            # squared distances by explicit differences per coordinate: no
            # cancellation from the |a|^2+|b|^2-2ab form.
            d2 = xp.zeros((r1 - r0, c1 - c0))
            for t in range(self.dim):
                diff = a[:, t][:, None] - b[:, t][None, :]
                d2 = d2 + diff * diff
            if self.kind == "se":
                k = xp.exp(-d2 / (2.0 * self.ell * self.ell))
            else:
                s = math.sqrt(3.0) * xp.sqrt(d2) / self.ell
                k = (1.0 + s) * xp.exp(-s)
        elif self.kind == "kms":
            i = xp.arange(r0, r1)[:, None]
            j = xp.arange(c0, c1)[None, :]
            k = xp.power_scalar(self.rho, xp.abs(i - j))
        else:
            raise ValueError(self.kind)
        if self.shift != 0.0 and self.kind != "kms":
            # add shift on the global diagonal
            lo, hi = max(r0, c0), min(r1, c1)
            if lo < hi:
                idx = xp.arange(lo, hi)
                k[idx - r0, idx - c0] = k[idx - r0, idx - c0] + self.shift
        return k

    # ---- closed forms where they exist -----------------------------------
    def closed_form_logdet(self) -> Optional[float]:
        if self.kind == "kms":
            return (self.n - 1) * math.log1p(-self.rho * self.rho)
        return None

    def lower_tri_bytes(self) -> int:
        beta = 8 if self.dtype == "f64" else 4
        return self.n * (self.n + 1) // 2 * beta


class _NumpyNS:
    """The same minimal array namespace over numpy (float64)."""

    def zeros(self, shape):
        return np.zeros(shape, dtype=np.float64)

    def arange(self, a, b):
        return np.arange(a, b)

    def exp(self, x):
        return np.exp(x)

    def sqrt(self, x):
        return np.sqrt(x)

    def abs(self, x):
        return np.abs(x)

    def power_scalar(self, base, e):
        return np.power(float(base), e.astype(np.float64))


class _TorchNS:
    """Minimal array namespace over torch, pinned to one device, float64."""

    def __init__(self, torch, device):
        self.t = torch
        self.device = device

    def zeros(self, shape):
        return self.t.zeros(shape, dtype=self.t.float64, device=self.device)

    def arange(self, a, b):
        return self.t.arange(a, b, device=self.device)

    def exp(self, x):
        return self.t.exp(x)

    def sqrt(self, x):
        return self.t.sqrt(x)

    def abs(self, x):
        return self.t.abs(x)

    def power_scalar(self, base, e):
        return self.t.pow(self.t.tensor(float(base), dtype=self.t.float64, device=self.device),
                          e.to(self.t.float64))


# --------------------------------------------------------------------------
# The five benchmark configurations, in order
# --------------------------------------------------------------------------
GIB = 1 << 30


def config(idx: int, dtype: Optional[str] = None) -> Workload:
    """Workload for benchmark configuration ``idx`` (1-based)."""
    if idx == 1:
        return Workload("cfg1_wishart_n512", "gram", 512, "f64", 128, seed=1001,
                        p=1024, shift=1e-3)
    if idx == 2:
        return Workload("cfg2_se_n8192", "se", 8192, "f64", 1024, seed=1002,
                        dim=8, ell=0.5, shift=1e-6)
    if idx == 3:
        return Workload("cfg3_ntk_n32768", "gram", 32768, dtype or "f64", 2048,
                        seed=1003, p=8192, decay=0.75, shift=1e-8)
    if idx == 4:
        return Workload("cfg4_matern32_n131072", "matern32", 131072, "f64", 4096,
                        seed=1004, dim=16, ell=0.3, shift=1e-6, mem_budget=16 * GIB)
    if idx == 5:
        return Workload("cfg5_ntk_n196608", "gram", 196608, "f64", 8192, seed=1005,
                        p=4096, decay=1.0, shift=1e-10, mem_budget=32 * GIB)
    raise ValueError("config index 1..5")


def kms(n: int, rho: float, dtype: str = "f64", block_size: int = 128,
        mem_budget: int = 0) -> Workload:
    return Workload(f"kms_n{n}_rho{rho}", "kms", n, dtype, block_size, rho=rho,
                    mem_budget=mem_budget)


def scaled_down(w: Workload, n: int, block_size: Optional[int] = None) -> Workload:
    """Same construction at a smaller order.

    Keeps p/n and the budget/size ratio.  For Gram matrices the shift is scaled
    with the diagonal (mean_k k^(-2 decay) / p grows when p shrinks), so the ratio
    of the trailing pivots to the matrix entries -- what decides how many digits
    any double-precision factorisation can deliver -- stays that of the full-size
    configuration.
    """
    ratio = n / w.n
    p = max(1, int(round(w.p * ratio))) if w.p else 0
    budget = int(w.mem_budget * ratio * ratio) if w.mem_budget else 0
    shift = w.shift
    if w.kind == "gram" and w.p:
        def diag_scale(q):
            return float(np.sum(np.arange(1, q + 1, dtype=np.float64) ** (-2.0 * w.decay))) / q
        shift = w.shift * diag_scale(p) / diag_scale(w.p)
    return Workload(f"{w.name}_scaled_n{n}", w.kind, n, w.dtype,
                    block_size or max(16, int(w.block_size * ratio)), seed=w.seed,
                    p=p, decay=w.decay, shift=shift, dim=w.dim, ell=w.ell,
                    rho=w.rho, mem_budget=budget)
