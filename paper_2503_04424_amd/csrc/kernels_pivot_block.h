// Symmetric pivoting over a whole diagonal block (MDET_FLAG_PIVOT_BLOCK).
//
// Sec. 2.2 of the paper: the symmetric form handles permutations, pivoting is done inside
// each block and not between blocks; the software appendix returns `perm` with
// P^T M P = L D L^T.  Here the candidates of every elimination step are ALL entries left
// on the diagonal of the current Schur complement inside the block column's w x w diagonal
// block (the 64-column leaf of MDET_FLAG_PIVOT is the special case w = 64); the pivot is
// the one of largest magnitude, the one that came first in the input on ties, a NaN counts
// as the largest.  D stays diagonal (1 x 1 pivots only).
//
// A pivot anywhere in the block needs that candidate's column up to date with every pivot
// taken before it.  The scheme is the blocked one with a running diagonal: the diagonal
// block is kept as a full symmetric matrix S in the workspace, brought up to date with 64
// pivots at a time (one product S -= L_p D L_p^T on the matrix cores); inside such a group
// of 64 each step is one small launch over the block's rows,
//     v_i   = S[p][i] - sum_{k < j, this group} L[i][k] (d_k L[p][k])      (column of pivot p)
//     l_ij  = v_i / d_j,      d_j = running diagonal of p,
//     diag_i <- diag_i - l_ij v_i,
// and leaves the partial maxima from which the next launch picks its pivot.  Nothing is
// swapped while the block is eliminated: rows keep their input positions, columns are in
// pivot order (`Lfull`), and the rows below the diagonal block get their 64 new columns by
// a gather of the pivots' columns, a product with everything solved before (matrix cores),
// and the leaf solve of the unpivoted path.  At the end the factor is put in place in
// pivot order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_leaf.h"

namespace mdet {

constexpr int PB_THREADS = 256;

// A candidate: magnitude as its bit pattern (IEEE magnitudes order like their patterns; NaN
// mapped to the pattern of infinity plus one so that it wins), and the row; no candidate: key 0.
struct PbCand {
  unsigned long long key;
  long long row;
};

__device__ __forceinline__ unsigned long long pb_key(double v) {
  if (!(v == v)) return 0x7ff0000000000001ull;
  return (unsigned long long)__double_as_longlong(fabs(v)) + 1ull;     // +1: a zero is still a candidate
}
__device__ __forceinline__ unsigned long long pb_key(float v) {
  if (!(v == v)) return 0x7f800001ull;
  return (unsigned long long)(unsigned)__float_as_int(fabsf(v)) + 1ull;
}
// larger magnitude wins, the smaller row on ties
__device__ __forceinline__ bool pb_better(const PbCand& a, const PbCand& b) {
  return a.key > b.key || (a.key == b.key && a.key != 0ull && a.row < b.row);
}

// Best candidate of the workgroup, in every thread.  s: PB_THREADS entries of LDS.
__device__ __forceinline__ PbCand pb_block_best(PbCand mine, PbCand* s) {
  s[threadIdx.x] = mine;
  __syncthreads();
  for (int h = PB_THREADS / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h && pb_better(s[threadIdx.x + h], s[threadIdx.x])) s[threadIdx.x] = s[threadIdx.x + h];
    __syncthreads();
  }
  const PbCand r = s[0];
  __syncthreads();
  return r;
}

// S <- the w x w diagonal block as a full symmetric matrix (only its lower triangle is read
// from P): 32 x 32 tiles on and below the diagonal, each written straight and transposed
// through LDS so that both the reads and the writes run along rows.  Grid: (tiles per side)^2.
template <typename T>
__global__ __launch_bounds__(256) void pb_symmetrize_kernel(const T* __restrict__ P, int64_t ld, int w,
                                                            T* __restrict__ S, int64_t lds) {
  __shared__ T t[32][33];
  const int nt = (w + 31) / 32;
  const int bi = blockIdx.x / nt, bj = blockIdx.x % nt;
  if (bj > bi) return;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;         // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int gr = bi * 32 + r, gc = bj * 32 + tx;
    T v = T(0);
    if (gr < w && gc < w) v = gc <= gr ? P[(int64_t)gr * ld + gc] : P[(int64_t)gc * ld + gr];
    t[r][tx] = v;
    if (gr < w && gc < w) S[(int64_t)gr * lds + gc] = v;
  }
  __syncthreads();
  if (bi != bj)
    for (int r = ty; r < 32; r += 8) {
      const int gr = bj * 32 + r, gc = bi * 32 + tx;            // the mirrored tile
      if (gr < w && gc < w) S[(int64_t)gr * lds + gc] = t[tx][r];
    }
}

// The running diagonal, all rows candidates, columns w .. ldl of Lfull zero, and the first
// step's partial maxima.
template <typename T>
__global__ __launch_bounds__(PB_THREADS) void pb_init_kernel(const T* __restrict__ P, int64_t ld, int w,
                                                             T* __restrict__ Lfull, int64_t ldl,
                                                             T* __restrict__ dg, int* __restrict__ active,
                                                             PbCand* __restrict__ part) {
  __shared__ PbCand red[PB_THREADS];
  const int i = blockIdx.x * PB_THREADS + threadIdx.x;
  PbCand mine{0ull, 0};
  if (i < w) {
    const T d = P[(int64_t)i * ld + i];
    dg[i] = d;
    active[i] = 1;
    mine = PbCand{pb_key(d), i};
    for (int64_t c = w; c < ldl; ++c) Lfull[(int64_t)i * ldl + c] = T(0);
  }
  const PbCand best = pb_block_best(mine, red);
  if (threadIdx.x == 0) part[blockIdx.x] = best;
}

// One elimination step: step jj of the group of 64 that starts at column c0 (pivot order).
template <typename T>
__global__ __launch_bounds__(PB_THREADS) void pb_step_kernel(
    const T* __restrict__ S, int64_t lds, T* __restrict__ Lfull, int64_t ldl, T* __restrict__ dg,
    int* __restrict__ active, const PbCand* __restrict__ part_in, PbCand* __restrict__ part_out, int nparts,
    int* __restrict__ piv, T* __restrict__ dvec, T* __restrict__ dinv, int* __restrict__ perm, int w, int c0,
    int jj, long long pivot0, DevFlags* flags) {
  __shared__ PbCand red[PB_THREADS];
  __shared__ T wrow[LEAF];
  // the pivot: best of the partial maxima the step before left (every workgroup finds it alone)
  PbCand mine{0ull, 0};
  for (int q = threadIdx.x; q < nparts; q += PB_THREADS)
    if (pb_better(part_in[q], mine)) mine = part_in[q];
  const PbCand top = pb_block_best(mine, red);
  const int p = (int)top.row;
  const T d = dg[p];
  // the pivot row's entries of this group, times their pivots: w_k = d_k L[p][k]
  if ((int)threadIdx.x < jj) wrow[threadIdx.x] = Lfull[(int64_t)p * ldl + c0 + threadIdx.x] * dvec[c0 + threadIdx.x];
  __syncthreads();
  const int i = blockIdx.x * PB_THREADS + threadIdx.x;
  PbCand next{0ull, 0};
  if (i < w) {
    T l = T(0);
    if (active[i] != 0 && i != p) {
      T v = S[(int64_t)p * lds + i];
      const T* Li = Lfull + (int64_t)i * ldl + c0;
      for (int k = 0; k < jj; ++k) v = fma(-Li[k], wrow[k], v);
      l = v / d;
      const T nd = fma(-l, v, dg[i]);
      dg[i] = nd;
      next = PbCand{pb_key(nd), i};
    }
    Lfull[(int64_t)i * ldl + c0 + jj] = l;
    if (i == p) {
      active[i] = 0;
      piv[c0 + jj] = p;
      dvec[c0 + jj] = d;
      dinv[c0 + jj] = T(1) / d;
      perm[c0 + jj] = (int)pivot0 + p;
      const bool zero = d == T(0);
      const bool finite = fabs((double)d) <= 1.7976931348623157e308;
      if (zero || !finite) {
        const unsigned long long idx = (unsigned long long)(pivot0 + c0 + jj);
        const unsigned long long old = atomicMin(&flags->first_bad, idx);
        if (idx <= old) atomicExch(&flags->bad_kind, zero ? 1ull : 2ull);
      }
    }
  }
  const PbCand best = pb_block_best(next, red);
  if (threadIdx.x == 0) part_out[blockIdx.x] = best;
}

// The group's own lw x lw leaf in pivot order (strictly lower part; 64 x 64, leading
// dimension 64) and the inverses of its 16 x 16 diagonal sub-blocks, as the leaf solve
// wants them.  One workgroup of 256 threads.
template <typename T>
__global__ __launch_bounds__(256) void pb_leaf_kernel(const T* __restrict__ Lfull, int64_t ldl,
                                                      const int* __restrict__ piv, int c0, int lw,
                                                      T* __restrict__ leaf, T* __restrict__ linv) {
  __shared__ T tile[LEAF * LEAF_PAD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15;
  for (int e = tid; e < LEAF * LEAF; e += 256) {
    const int r = e >> 6, c = e & 63;
    const T v = (r < lw && c < r) ? Lfull[(int64_t)piv[c0 + r] * ldl + c0 + c] : T(0);
    tile[r * LEAF_PAD + c] = v;
    leaf[r * LEAF + c] = v;
  }
  __syncthreads();
  leaf_invert_sub<T>(tile, linv, wave, l16);
}

// Rows below the diagonal block: their columns of the group's pivots, side by side in pivot
// order, into Y[:, c0 .. c0 + 64) (columns past lw zero); and the pivots' own rows of
// everything solved before, Bg[t][0 .. c0) = Lfull[piv[c0 + t]][0 .. c0).
template <typename T>
__global__ __launch_bounds__(256) void pb_gather_kernel(const T* __restrict__ X, int64_t ldx, int64_t rows,
                                                        T* __restrict__ Y, int64_t ldy,
                                                        const T* __restrict__ Lfull, int64_t ldl,
                                                        T* __restrict__ Bg, int64_t ldb,
                                                        const int* __restrict__ piv, int c0, int lw) {
  const int t = threadIdx.x & 63, sub = threadIdx.x >> 6;
  const int src = t < lw ? piv[c0 + t] : 0;
  for (int64_t r = (int64_t)blockIdx.x * 4 + sub; r < rows; r += (int64_t)gridDim.x * 4)
    Y[r * ldy + c0 + t] = t < lw ? X[r * ldx + src] : T(0);
  // the first workgroups also copy the pivots' rows (64 rows of c0 entries)
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < (int64_t)LEAF * c0; e += (int64_t)gridDim.x * 256) {
    const int row = (int)(e / c0), k = (int)(e % c0);
    Bg[(int64_t)row * ldb + k] = row < lw ? Lfull[(int64_t)piv[c0 + row] * ldl + k] : T(0);
  }
}

// The factor into its place, in pivot order: unit-lower L of the diagonal block (row r =
// the multipliers of the row taken at step r), D on the diagonal, the rows below from Y.
template <typename T>
__global__ __launch_bounds__(256) void pb_store_kernel(T* __restrict__ P, int64_t ld, int64_t m, int w,
                                                       const T* __restrict__ Lfull, int64_t ldl,
                                                       const int* __restrict__ piv, const T* __restrict__ dvec,
                                                       const T* __restrict__ Y, int64_t ldy) {
  for (int64_t r = blockIdx.x; r < m; r += gridDim.x) {
    if (r < w) {
      const int src = piv[r];
      for (int c = threadIdx.x; c <= r; c += 256)
        P[r * ld + c] = c == r ? dvec[r] : Lfull[(int64_t)src * ldl + c];
    } else {
      for (int c = threadIdx.x; c < w; c += 256) P[r * ld + c] = Y[(r - w) * ldy + c];
    }
  }
}

}  // namespace mdet
