// Leaf kernels of the block-column factorisation (LEAF = 64 columns at a time).
//
// leaf_factor_kernel : in-place A = L D L^T of one <= 64 x 64 diagonal leaf
//                      (Sec. 2.2: "in-place ... decomposition" of the diagonal block,
//                      symmetric case: unit-lower L, diagonal D, no pivoting).
// leaf_solve_kernel  : rows below the leaf, X = A_rows L^-T D^-1
//                      (Sec. 2.2: in-place triangular solve of the off-diagonal
//                      blocks; App. E.1 "solve lower triangular system"; the
//                      D^-1 is the LDL^T "diagonal scaling").
//
// Both keep one matrix row per lane in registers; tiles travel between HBM and
// registers through LDS so that every global access is a coalesced 16-byte vector.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mdet {

constexpr int LEAF = 64;
constexpr int LEAF_PAD = LEAF + 1;   // LDS row stride: lane-per-row reads hit distinct banks

// Device-side status words shared by all kernels of one call.
struct DevFlags {
  unsigned long long first_bad;   // (global pivot index) of first zero/non-finite pivot; ~0ull = none
  unsigned long long bad_kind;    // 1 = zero, 2 = non-finite (kind of *some* bad pivot; refined on host)
};

// Coalesced copy of a rows x cols tile (<= 64 x 64) from global memory into an LDS
// array with row stride `stride`, by one wavefront.  Missing rows/columns read as 0
// (diagonal entries of the padding as 1 when unit_pad is set).  With transpose the
// element (r, c) lands at lds[c * stride + r].  Loads are issued in batches of 16
// independent requests so that their latencies overlap.
template <typename T, bool TRANSPOSE, bool STRICT_LOWER>
__device__ __forceinline__ void tile_to_lds(T* lds, int stride, const T* g, int64_t ld, int rows,
                                            int cols, bool unit_pad, int lane) {
  constexpr int BATCH = 16;
#pragma unroll 1
  for (int e0 = 0; e0 < LEAF * LEAF; e0 += 64 * BATCH) {
    T v[BATCH];
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {
      const int e = e0 + q * 64 + lane;
      const int r = e >> 6, c = e & 63;
      const bool in = r < rows && c < cols && (!STRICT_LOWER || c < r);
      v[q] = in ? g[(int64_t)r * ld + c] : ((unit_pad && r == c) ? T(1) : T(0));
    }
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {
      const int e = e0 + q * 64 + lane;
      const int r = e >> 6, c = e & 63;
      lds[TRANSPOSE ? c * stride + r : r * stride + c] = v[q];
    }
  }
}

// One wavefront factors one leaf.  Lane i holds row i (64 registers).  At step j
// every lane publishes its entry of the pivot column through a 64-element LDS
// line; the pivot and the other lanes' entries come back as broadcast reads, and
// the rank-1 update of the remaining columns is 63-j independent multiply-adds.
// The steps are spelled out with templates so that every register index is a
// compile-time constant.
// a[c] -= lj * cj[c] for c in [C0, LEAF), eight columns per stage; the LDS reads of
// the next stage are issued before the products of the current one.
template <typename T, int C0>
__device__ __forceinline__ void leaf_fetch(T (&v)[8], const T* cj) {
#pragma unroll
  for (int q = 0; q < 8; ++q)
    if (C0 + q < LEAF) v[q] = cj[C0 + q];
}
template <typename T, int C0>
__device__ __forceinline__ void leaf_rank1(T (&a)[LEAF], const T lj, const T* cj, T (&cur)[8]) {
  if constexpr (C0 < LEAF) {
    T nxt[8];
    leaf_fetch<T, C0 + 8>(nxt, cj);
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (C0 + q < LEAF) a[C0 + q] -= lj * cur[q];   // a_ic -= l_ij d_j l_cj
    // stage boundary: nothing moves across it, so at most two stages of the pivot
    // column are in registers at any time
    __builtin_amdgcn_sched_barrier(0);
    leaf_rank1<T, C0 + 8>(a, lj, cj, nxt);
  }
}

template <typename T, int J>
__device__ __forceinline__ void leaf_step(T (&a)[LEAF], T (*col)[LEAF], T* dsave, T* rsave,
                                          const int lane) {
  if constexpr (J < LEAF) {
    const T wj = a[J];                         // lane i > J: unscaled w_iJ = l_iJ d_J
    T* cj = col[J & 1];
    cj[lane] = wj;
    __syncthreads();
    const T dj = cj[J];                        // pivot d_J (uniform)
    const T rj = T(1) / dj;
    const T lj = wj * rj;
    dsave[J] = dj;                             // same value from every lane
    rsave[J] = rj;
    {
      T first[8];
      leaf_fetch<T, J + 1>(first, cj);
      leaf_rank1<T, J + 1>(a, lj, cj, first);
    }
    a[J] = lane > J ? lj : a[J];
    leaf_step<T, J + 1>(a, col, dsave, rsave, lane);
  }
}

template <typename T>
__global__ __launch_bounds__(64) void leaf_factor_kernel(T* __restrict__ A, int64_t ld, int w,
                                                         T* __restrict__ dvec,
                                                         T* __restrict__ dinv,
                                                         long long pivot0, DevFlags* flags) {
  __shared__ T tile[LEAF * LEAF_PAD];
  __shared__ __attribute__((aligned(16))) T col[2][LEAF];
  __shared__ T dsave[LEAF], rsave[LEAF];
  const int lane = threadIdx.x;
  tile_to_lds<T, false, false>(tile, LEAF_PAD, A, ld, w, w, true, lane);
  __syncthreads();
  T a[LEAF];
#pragma unroll
  for (int j = 0; j < LEAF; ++j) a[j] = tile[lane * LEAF_PAD + j];

  leaf_step<T, 0>(a, col, dsave, rsave, lane);
  __syncthreads();

  // pivots out; first zero / non-finite pivot reported through the flags
  const T myd = dsave[lane];
  const bool zero = myd == T(0);
  const bool bad = lane < w && (zero || !(fabs((double)myd) <= 1.7976931348623157e308));
  if (lane < w) { dvec[lane] = myd; dinv[lane] = rsave[lane]; }
  const unsigned long long mask = __ballot(bad);
  if (mask != 0ull) {
    const int first = __ffsll((long long)mask) - 1;
    if (lane == first) {
      unsigned long long idx = (unsigned long long)(pivot0 + first);
      unsigned long long old = atomicMin(&flags->first_bad, idx);
      if (idx <= old) atomicExch(&flags->bad_kind, zero ? 1ull : 2ull);
    }
  }
  // write back the lower triangle (L below the diagonal, D on it)
#pragma unroll
  for (int j = 0; j < LEAF; ++j) tile[lane * LEAF_PAD + j] = a[j];
  __syncthreads();
  for (int e = lane; e < LEAF * LEAF; e += 64) {
    int r = e >> 6, c = e & 63;
    if (r < w && c <= r) A[(int64_t)r * ld + c] = tile[r * LEAF_PAD + c];
  }
}

// Rows below a factored leaf.  One wavefront per workgroup takes 64 rows; lane = row.
// X (m x w, in place) <- X L^-T D^-1 by forward substitution along the row,
//    w_j = x_j - sum_{p<j} w_p L[j][p] ;  l_j = w_j / d_j  (as w_j * dinv_j),
// arranged column by column (once w_p is final it is subtracted from every later
// entry), so the multiply-adds of one step are independent while each entry still
// receives its terms in the order p = 0, 1, 2, ...  L is kept transposed in LDS and
// read as broadcasts.
constexpr int LT_STRIDE = LEAF + 2;   // even: rows stay 16-byte aligned

template <typename T>
__global__ __launch_bounds__(64) void leaf_solve_kernel(
    T* __restrict__ X, int64_t ld, int m, int w, const T* __restrict__ Lleaf, int64_t ldl,
    const T* __restrict__ dinv) {
  __shared__ __attribute__((aligned(16))) T Lt[LEAF * LT_STRIDE];   // Lt[p][j] = L[j][p], j > p
  __shared__ T rinv[LEAF];
  __shared__ T stage[LEAF * LEAF_PAD];
  const int lane = threadIdx.x;

  tile_to_lds<T, true, true>(Lt, LT_STRIDE, Lleaf, ldl, w, w, false, lane);
  rinv[lane] = lane < w ? dinv[lane] : T(0);

  const int64_t r0 = (int64_t)blockIdx.x * LEAF;
  int rows = m - r0 < LEAF ? (int)(m - r0) : LEAF;
  T* Xw = X + r0 * ld;
  tile_to_lds<T, false, false>(stage, LEAF_PAD, Xw, ld, rows, w, false, lane);
  __syncthreads();

  T x[LEAF];
#pragma unroll
  for (int j = 0; j < LEAF; ++j) x[j] = stage[lane * LEAF_PAD + j];
#pragma unroll
  for (int p = 0; p < LEAF - 1; ++p) {
    const T xp = x[p];
#pragma unroll
    for (int j = p + 1; j < LEAF; ++j) x[j] -= xp * Lt[p * LT_STRIDE + j];
  }
#pragma unroll
  for (int j = 0; j < LEAF; ++j) stage[lane * LEAF_PAD + j] = x[j] * rinv[j];
  __syncthreads();
  for (int e = lane; e < LEAF * LEAF; e += 64) {
    int r = e >> 6, c = e & 63;
    if (r < rows && c < w) Xw[(int64_t)r * ld + c] = stage[r * LEAF_PAD + c];
  }
}

}  // namespace mdet
