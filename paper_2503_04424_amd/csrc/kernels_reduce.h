// Fused log|d| / sign reduction.
//
// App. D of the paper accumulates, after each diagonal block is decomposed,
//     l <- l + logabsdet(block),   sigma <- sigma * sgn(block);
// for LDL^T the block's determinant is the product of its pivots.  One workgroup
// per block column reduces that column's pivots (always in double, also for
// float pivots); a second tiny kernel adds the per-column terms in column order,
// so the result does not depend on how the launches were scheduled.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mdet {

constexpr int RED_THREADS = 256;

// partial[3*k + 0] = sum log|d_j|, [3*k+1] = number of negative pivots, [3*k+2] = number of zeros
template <typename T>
__global__ __launch_bounds__(RED_THREADS) void logdet_partial_kernel(const T* __restrict__ d,
                                                                     int64_t n, int64_t bs,
                                                                     double* __restrict__ partial) {
  __shared__ double s_log[RED_THREADS];
  __shared__ unsigned s_neg[RED_THREADS], s_zero[RED_THREADS];
  const int64_t k = blockIdx.x;
  const int64_t lo = k * bs, hi = (lo + bs < n) ? lo + bs : n;
  double acc = 0.0;
  unsigned neg = 0, zero = 0;
  for (int64_t j = lo + threadIdx.x; j < hi; j += RED_THREADS) {
    const double v = (double)d[j];
    neg += v < 0.0;
    zero += v == 0.0;
    acc += log(fabs(v));
  }
  s_log[threadIdx.x] = acc; s_neg[threadIdx.x] = neg; s_zero[threadIdx.x] = zero;
  __syncthreads();
  for (int s = RED_THREADS / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      s_log[threadIdx.x] += s_log[threadIdx.x + s];
      s_neg[threadIdx.x] += s_neg[threadIdx.x + s];
      s_zero[threadIdx.x] += s_zero[threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    partial[3 * k + 0] = s_log[0];
    partial[3 * k + 1] = (double)s_neg[0];
    partial[3 * k + 2] = (double)s_zero[0];
  }
}

// out[0] = logabsdet, out[1] = sign (-1, 0, +1), out[2] = negative pivots;
// running[k] (optional) = sum of the first k+1 column terms (log-determinant of the
// leading principal sub-matrix that ends with block column k).
__global__ void logdet_combine_kernel(const double* __restrict__ partial, int64_t nblk,
                                      double* __restrict__ out, double* __restrict__ running) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double acc = 0.0, neg = 0.0, zero = 0.0;
  for (int64_t k = 0; k < nblk; ++k) {
    acc += partial[3 * k + 0];
    neg += partial[3 * k + 1];
    zero += partial[3 * k + 2];
    if (running) running[k] = acc;
  }
  const long long ineg = (long long)neg;
  out[0] = zero > 0.0 ? -HUGE_VAL : acc;
  out[1] = zero > 0.0 ? 0.0 : ((ineg & 1) ? -1.0 : 1.0);
  out[2] = neg;
}

// Storage formats that are only ever widened: IEEE binary16 and bfloat16, as raw bits.
struct StoredF16 { uint16_t bits; };
struct StoredBF16 { uint16_t bits; };
__device__ __forceinline__ double widen_exact(float v) { return (double)v; }
__device__ __forceinline__ double widen_exact(StoredF16 v) {
  _Float16 h;
  __builtin_memcpy(&h, &v.bits, 2);
  return (double)h;
}
__device__ __forceinline__ double widen_exact(StoredBF16 v) {
  return (double)__uint_as_float((uint32_t)v.bits << 16);     // bfloat16 = the upper half of a float
}

// fp32 / fp16 / bf16 -> fp64 copy of the part of a row-major matrix the factorisation
// reads: row i up to the end of its 64-column leaf on the diagonal.  Widening is exact.
template <typename S>
__global__ __launch_bounds__(256) void widen_lower_kernel(const S* __restrict__ src, int64_t lds,
                                                          double* __restrict__ dst, int64_t ldd,
                                                          int64_t n) {
  const int64_t i = blockIdx.x;
  int64_t end = (i / 64 + 1) * 64;
  if (end > n) end = n;
  for (int64_t j = threadIdx.x; j < end; j += 256) dst[i * ldd + j] = widen_exact(src[i * lds + j]);
}

// The same for a rows x cols rectangle (a piece of a block column on its way from host
// memory): src with leading dimension lds, dst with ldd.
template <typename S>
__global__ __launch_bounds__(256) void widen_rows_kernel(const S* __restrict__ src, int64_t lds,
                                                         double* __restrict__ dst, int64_t ldd,
                                                         int64_t rows, int64_t cols) {
  const int64_t total = rows * cols;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t i = e / cols, j = e - i * cols;
    dst[i * ldd + j] = widen_exact(src[i * lds + j]);
  }
}

// dst[c][r] = src[r][c] for a rows x cols rectangle on its way from host memory (a block of
// the upper triangle of a general matrix into the transposed store).  32 x 32 tiles through
// LDS, reads and writes along rows.  Grid: (ceil(cols / 32), ceil(rows / 32)).
template <typename T>
__global__ __launch_bounds__(256) void transpose_rows_kernel(const T* __restrict__ src, int64_t lds,
                                                             T* __restrict__ dst, int64_t ldd,
                                                             int64_t rows, int64_t cols) {
  __shared__ T t[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;         // 32 x 8
  const int64_t r0 = (int64_t)blockIdx.y * 32, c0 = (int64_t)blockIdx.x * 32;
  for (int r = ty; r < 32; r += 8)
    if (r0 + r < rows && c0 + tx < cols) t[r][tx] = src[(r0 + r) * lds + c0 + tx];
  __syncthreads();
  for (int c = ty; c < 32; c += 8)
    if (c0 + c < cols && r0 + tx < rows) dst[(c0 + c) * ldd + r0 + tx] = t[tx][c];
}

// X[r][c] *= d[c] in place, rows x cols with leading dimension ld (cols and ld multiples
// of the 16-byte vector): rows of L of a finished block column become rows of W = L D,
// each product rounded once, as the update kernels round it when they scale on the fly.
template <typename T>
__global__ __launch_bounds__(256) void scale_columns_kernel(T* __restrict__ X, int64_t ld, int64_t rows,
                                                            int cols, const T* __restrict__ d) {
  constexpr int VEC = 16 / (int)sizeof(T);
  using vec_t = T __attribute__((ext_vector_type(VEC)));
  const int per_row = cols / VEC;
  const int64_t total = rows * per_row;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t r = e / per_row;
    const int c = (int)(e % per_row) * VEC;
    vec_t v = *reinterpret_cast<vec_t*>(X + r * ld + c);
    const vec_t s = *reinterpret_cast<const vec_t*>(d + c);
#pragma unroll
    for (int q = 0; q < VEC; ++q) v[q] *= s[q];
    *reinterpret_cast<vec_t*>(X + r * ld + c) = v;
  }
}

}  // namespace mdet
