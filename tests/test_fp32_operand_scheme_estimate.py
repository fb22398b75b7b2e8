"""Why configuration 3 has no fp32-matrix-core mode that meets its 1e-4 bar: a numpy model of
the candidate scheme (the trailing matrix carried in fp64, block columns factored in fp64, the
Schur update's operands rounded to fp32 and its products summed in fp32 over chunks of K, each
chunk's sum then added to the fp64 value), on the scaled-down configuration-3 matrix stored in
fp32, against the oracle on the same bits.  What fails is the fp32 accumulator, not the fp32
operands: with exact sums the rounded operands cost 1e-6, with fp32 sums over 64 or more terms
the result is outside 1e-4 (Sec. 2.1: the rank-p part of the Gram matrix is eight orders above
the shift, and its leading columns carry most of it, so a chunk's partial sum is the size of
the matrix entry while the pivot is the size of the shift).  CPU only; shares nothing with the
library."""
import numpy as np
import pytest

import oracle
import workloads as W


def blocked_ldlt(a32, bs, chunk):
    """chunk = 0: operands rounded to fp32, products and sums exact (fp64)."""
    n = a32.shape[0]
    c = a32.astype(np.float64)
    d = np.zeros(n)
    for k0 in range(0, n, bs):
        k1 = min(n, k0 + bs)
        for j in range(k0, k1):
            d[j] = c[j, j]
            c[j + 1:, j] /= d[j]
            if j + 1 < k1:
                c[j + 1:, j + 1:k1] -= np.outer(c[j + 1:, j] * d[j], c[j + 1:k1, j])
        if k1 >= n:
            break
        l = c[k1:, k0:k1]
        lf, wf = l.astype(np.float32), (l * d[k0:k1]).astype(np.float32)
        if chunk == 0:
            c[k1:, k1:] -= wf.astype(np.float64) @ lf.astype(np.float64).T
        else:
            for c0 in range(0, k1 - k0, chunk):
                c[k1:, k1:] -= (wf[:, c0:c0 + chunk] @ lf[:, c0:c0 + chunk].T).astype(np.float64)
    return float(np.sum(np.log(np.abs(d)))), int(np.prod(np.sign(d)))


def test_fp32_accumulation_not_fp32_operands_is_what_misses_the_bar():
    n, bs = 1024, 128
    w = W.scaled_down(W.config(3, "f32"), n, bs)
    a = w.dense()
    o = oracle.ldlt_logdet(a)
    assert o.sign == 1
    err = {}
    for chunk in (0, 32, 128):
        ld, sg = blocked_ldlt(a, bs, chunk)
        assert sg == 1
        err[chunk] = abs(ld - o.logabsdet) / abs(o.logabsdet)
    assert err[0] <= 5e-6                     # fp32 operands alone: far inside the bar
    assert err[128] > 1e-4                    # a matrix instruction's fp32 accumulator over a usable K: outside
    assert err[32] > 10 * err[0] and err[128] > 2 * err[32]     # and the loss grows with the chunk
