"""CPU oracle for the principal-minor sequence and the FLODANCE fit (Sec. 3.2, Alg. 2).

TEST INFRASTRUCTURE ONLY.  Import this from tests, from the smoke check and from
the benchmark's CPU-baseline leg; the GPU library never touches it and shares no
code with it.

What is computed, in the paper's notation (Alg. 2; the regression is Eq. (7) of
Sec. 3.2, its covariates are derived in App. "Derivation of FLODANCE
Parameterization"):

    ell_k = sum_{i <= k} log|D_ii|            log|det| of the k x k leading block
    L_j   = ell_{j d} / j                      every d-th entry, normalised
    n_j   = n_0 + j,  j = 1 .. n_s - n_0
    y_j   = n_j (n_j - 1)^{-1/2} (L_{n_j} - L_{n_0})
    X_j,1 = (n_j - 1)^{1/2}
    X_j,i+1 = -(n_j - 1)^{-1/2} n_j^{-i+1} logGamma(n_j + 1),   i = 1 .. q + 1
    beta  = argmin |X beta - y|_2  ( = (X^T X)^{-1} X^T y )
    (c_0, nu_0, .., nu_q) = beta
    Lhat_n = L_{n_0} + c_0 (1 - 1/n) - sum_{i=1}^{q+1} nu_{i-1} n^{-i} logGamma(n + 1)

Everything is float64 (the paper fixes no precision); the running sum of the
logarithms is kept in long double.  The least-squares problem is handed to
numpy.linalg.lstsq on X with its columns scaled to unit length (an exact change of
variables that keeps the library routine away from its rank cut-off: the columns of
X differ by a factor n per power of 1/n).
"""
from dataclasses import dataclass

import numpy as np
from scipy.special import gammaln


def principal_logdets(diag: np.ndarray) -> np.ndarray:
    """ell_k = log|det| of the k x k leading principal block, k = 1 .. len(diag), from the
    pivots D_ii of the LDL^T factorisation (Alg. 2, first step)."""
    d = np.asarray(diag, dtype=np.float64)
    return np.cumsum(np.log(np.abs(d)).astype(np.longdouble)).astype(np.float64)


def normalised_sequence(ell: np.ndarray, d: int, n_s: int) -> np.ndarray:
    """L_j = ell_{j d} / j for j = 1 .. n_s (returned with L[0] = L_1)."""
    ell = np.asarray(ell, dtype=np.float64)
    j = np.arange(1, n_s + 1)
    return ell[j * d - 1] / j


def design(ell: np.ndarray, d: int, n_0: int, n_s: int, q: int):
    """Design matrix X ((n_s - n_0) x (q + 2)), response y and L_{n_0} of Alg. 2."""
    if not (1 <= n_0 < n_s and q >= 0 and d >= 1 and n_s * d <= len(ell)):
        raise ValueError("need 1 <= n_0 < n_s, q >= 0, d >= 1 and n_s d <= len(ell)")
    L = normalised_sequence(ell, d, n_s)
    L_n0 = L[n_0 - 1]
    nj = np.arange(n_0 + 1, n_s + 1, dtype=np.float64)
    y = nj / np.sqrt(nj - 1.0) * (L[n_0:] - L_n0)
    X = np.empty((len(nj), q + 2))
    X[:, 0] = np.sqrt(nj - 1.0)
    lg = gammaln(nj + 1.0)
    for i in range(1, q + 2):
        X[:, i] = -lg / (np.sqrt(nj - 1.0) * nj ** (i - 1))
    return X, y, L_n0


@dataclass
class FlodanceFit:
    beta: np.ndarray      # (c_0, nu_0, .., nu_q)
    L_n0: float
    q: int
    residual: float       # |X beta - y|_2

    def eval(self, n) -> np.ndarray:
        """Lhat_n of Alg. 2 (last step) at the given n (scalars or array)."""
        n = np.asarray(n, dtype=np.float64)
        lg = gammaln(n + 1.0)
        out = self.L_n0 + self.beta[0] * (1.0 - 1.0 / n)
        for i in range(1, self.q + 2):
            out = out - self.beta[i] * lg / n ** i
        return out


def fit(ell: np.ndarray, d: int, n_0: int, n_s: int, q: int) -> FlodanceFit:
    X, y, L_n0 = design(ell, d, n_0, n_s, q)
    scale = np.sqrt((X * X).sum(axis=0))
    beta_s, *_ = np.linalg.lstsq(X / scale, y, rcond=None)
    beta = beta_s / scale
    return FlodanceFit(beta=beta, L_n0=float(L_n0), q=q, residual=float(np.linalg.norm(X @ beta - y)))
