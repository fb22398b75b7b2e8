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

__device__ __forceinline__ double lane_bcast(double v, int src) {
  int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ float lane_bcast(float v, int src) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}

// Coalesced copy of a rows x cols tile (<= 64 x 64) between global memory and an
// LDS array with row stride LEAF_PAD.  Missing rows/columns read as `fill`
// (diagonal entries of the padding read as 1 when unit_pad is set).
template <typename T, int NTHREADS>
__device__ __forceinline__ void tile_to_lds(T* lds, const T* g, int64_t ld, int rows, int cols,
                                            bool unit_pad, int tid) {
  for (int e = tid; e < LEAF * LEAF; e += NTHREADS) {
    int r = e >> 6, c = e & 63;
    T v = (r < rows && c < cols) ? g[(int64_t)r * ld + c] : ((unit_pad && r == c) ? T(1) : T(0));
    lds[r * LEAF_PAD + c] = v;
  }
}

// One wavefront factors one leaf.  Lane i holds row i (64 registers); the pivot
// column is broadcast lane by lane with v_readlane, so no barrier is needed.
template <typename T>
__global__ __launch_bounds__(64) void leaf_factor_kernel(T* __restrict__ A, int64_t ld, int w,
                                                         T* __restrict__ dvec,
                                                         T* __restrict__ dinv,
                                                         long long pivot0, DevFlags* flags) {
  __shared__ T tile[LEAF * LEAF_PAD];
  const int lane = threadIdx.x;
  tile_to_lds<T, 64>(tile, A, ld, w, w, true, lane);
  __syncthreads();
  T a[LEAF];
#pragma unroll
  for (int j = 0; j < LEAF; ++j) a[j] = tile[lane * LEAF_PAD + j];

  int bad_at = -1, bad_kind = 0;
#pragma unroll
  for (int j = 0; j < LEAF; ++j) {
    const T dj = lane_bcast(a[j], j);          // pivot d_j (uniform)
    if (bad_at < 0 && j < w) {
      if (dj == T(0)) { bad_at = j; bad_kind = 1; }
      else if (!(fabs((double)dj) <= 1.7976931348623157e308)) { bad_at = j; bad_kind = 2; }
    }
    const T rj = T(1) / dj;
    const T wj = a[j];                         // lane i > j: unscaled w_ij = l_ij d_j
    const T lj = wj * rj;
    if (lane == j && j < w) { dvec[j] = dj; dinv[j] = rj; }
#pragma unroll
    for (int c = j + 1; c < LEAF; ++c) a[c] -= lj * lane_bcast(wj, c);   // a_ic -= l_ij d_j l_cj
    if (lane > j) a[j] = lj;
  }
  if (bad_at >= 0 && lane == 0) {
    unsigned long long idx = (unsigned long long)(pivot0 + bad_at);
    unsigned long long old = atomicMin(&flags->first_bad, idx);
    if (idx <= old) atomicExch(&flags->bad_kind, (unsigned long long)bad_kind);
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

// Rows below a factored leaf.  Each wavefront takes 64 rows; lane = row.
// X (m x w, in place) <- X L^-T D^-1 by forward substitution along the row:
//    w_j = x_j - sum_{p<j} w_p L[j][p] ;  l_j = w_j / d_j  (as w_j * dinv_j).
constexpr int SOLVE_WAVES = 2;

template <typename T>
__global__ __launch_bounds__(64 * SOLVE_WAVES) void leaf_solve_kernel(
    T* __restrict__ X, int64_t ld, int m, int w, const T* __restrict__ Lleaf, int64_t ldl,
    const T* __restrict__ dinv) {
  __shared__ T Ls[LEAF * LEAF];
  __shared__ T rinv[LEAF];
  __shared__ T stage[SOLVE_WAVES][LEAF * LEAF_PAD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  for (int e = tid; e < LEAF * LEAF; e += 64 * SOLVE_WAVES) {
    int r = e >> 6, c = e & 63;
    Ls[e] = (r < w && c < r) ? Lleaf[(int64_t)r * ldl + c] : T(0);
  }
  if (tid < LEAF) rinv[tid] = tid < w ? dinv[tid] : T(0);

  const int64_t r0 = ((int64_t)blockIdx.x * SOLVE_WAVES + wave) * LEAF;
  int rows = m - r0 < LEAF ? (int)(m - r0) : LEAF;
  if (rows < 0) rows = 0;
  T* st = stage[wave];
  T* Xw = X + r0 * ld;
  tile_to_lds<T, 64>(st, Xw, ld, rows, w, false, lane);
  __syncthreads();

  T x[LEAF];
#pragma unroll
  for (int j = 0; j < LEAF; ++j) x[j] = st[lane * LEAF_PAD + j];
#pragma unroll
  for (int j = 1; j < LEAF; ++j) {
    T s = x[j];
#pragma unroll
    for (int p = 0; p < j; ++p) s -= x[p] * Ls[j * LEAF + p];
    x[j] = s;
  }
#pragma unroll
  for (int j = 0; j < LEAF; ++j) st[lane * LEAF_PAD + j] = x[j] * rinv[j];
  __syncthreads();
  for (int e = lane; e < LEAF * LEAF; e += 64) {
    int r = e >> 6, c = e & 63;
    if (r < rows && c < w) Xw[(int64_t)r * ld + c] = st[r * LEAF_PAD + c];
  }
}

}  // namespace mdet
