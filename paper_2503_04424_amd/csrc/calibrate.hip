// Two measuring sticks for the benchmark, behind the same C ABI as the path itself.
//
//  * copy_kernel: a plain copy of a known number of bytes.  What the profiler's memory
//    counters (FETCH_SIZE, WRITE_SIZE) read for it, against the bytes it is known to move,
//    is the scale factor applied to the same counters read for the path's kernels.
//  * mfma_peak_*_kernel: nothing but matrix-core instructions on registers, accumulators in
//    AGPRs: the rate the matrix pipe delivers when a wavefront always has its next product
//    queued - the measured counterpart of the published peak that the trailing update
//    (the dense contraction of Sec. 2.2, S <- S - C B) is priced against.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/memdet.h"

namespace mdet {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                   int64_t vecs) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < vecs; i += (int64_t)gridDim.x * 256)
    dst[i] = src[i];
}

typedef double d4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

// Each wavefront: `iters` rounds of 16 products, NACC accumulators in turn, 16 / NACC products
// in a row on each.  One 16 x 16 x 4 product is 2048 flop in either type.  The whole loop is
// one assembly statement, so the accumulators stay in the AGPRs that the constraints name
// (written with the builtin, or with one statement per product, the compiler carries them in
// VGPRs around the loop and copies all of them to AGPRs and back in every round, which more
// than halves the rate the probe shows).
#define MDET_P(INS, acc, a, b) INS " %" #acc ", %" #a ", %" #b ", %" #acc "\n\t"
// operands: %0..%15 accumulators, %16..%19 a, %20..%23 b, %24 counter
#define MDET_ROUND16(INS)                                                                         \
  MDET_P(INS, 0, 16, 20) MDET_P(INS, 1, 16, 21) MDET_P(INS, 2, 16, 22) MDET_P(INS, 3, 16, 23)     \
  MDET_P(INS, 4, 17, 20) MDET_P(INS, 5, 17, 21) MDET_P(INS, 6, 17, 22) MDET_P(INS, 7, 17, 23)     \
  MDET_P(INS, 8, 18, 20) MDET_P(INS, 9, 18, 21) MDET_P(INS, 10, 18, 22) MDET_P(INS, 11, 18, 23)   \
  MDET_P(INS, 12, 19, 20) MDET_P(INS, 13, 19, 21) MDET_P(INS, 14, 19, 22) MDET_P(INS, 15, 19, 23)
// operands: %0..%3 accumulators, %4..%7 a, %8..%11 b, %12 counter
#define MDET_ROUND4(INS)                                                                          \
  MDET_P(INS, 0, 4, 8) MDET_P(INS, 0, 5, 9) MDET_P(INS, 0, 6, 10) MDET_P(INS, 0, 7, 11)           \
  MDET_P(INS, 1, 4, 9) MDET_P(INS, 1, 5, 10) MDET_P(INS, 1, 6, 11) MDET_P(INS, 1, 7, 8)           \
  MDET_P(INS, 2, 4, 10) MDET_P(INS, 2, 5, 11) MDET_P(INS, 2, 6, 8) MDET_P(INS, 2, 7, 9)           \
  MDET_P(INS, 3, 4, 11) MDET_P(INS, 3, 5, 8) MDET_P(INS, 3, 6, 9) MDET_P(INS, 3, 7, 10)
#define MDET_LOOP_TAIL(cnt) "s_sub_u32 %" #cnt ", %" #cnt ", 1\n\ts_cmp_lg_u32 %" #cnt ", 0\n\ts_cbranch_scc1 1b\n\t"

template <typename T, typename V4, int NACC>
__device__ __forceinline__ void mfma_peak_body(T* out, int iters) {
  V4 acc[NACC];
  for (int i = 0; i < NACC; ++i) acc[i] = V4{0, 0, 0, 0};
  T a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = (T)(threadIdx.x * 1e-3 + i);
    b[i] = (T)(1.0 + threadIdx.x * 1e-4 * (i + 1));
  }
  int cnt = iters;
  constexpr bool f64 = sizeof(T) == 8;
  if constexpr (NACC == 16) {
#define MDET_ASM16(INS)                                                                               \
    asm volatile("1:\n\t" MDET_ROUND16(INS) MDET_LOOP_TAIL(24)                                        \
                 : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]), "+a"(acc[5]), \
                   "+a"(acc[6]), "+a"(acc[7]), "+a"(acc[8]), "+a"(acc[9]), "+a"(acc[10]),             \
                   "+a"(acc[11]), "+a"(acc[12]), "+a"(acc[13]), "+a"(acc[14]), "+a"(acc[15])          \
                 : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(b[0]), "v"(b[1]), "v"(b[2]),       \
                   "v"(b[3]), "s"(cnt)                                                                \
                 : "scc")
    if constexpr (f64) MDET_ASM16("v_mfma_f64_16x16x4_f64");
    else MDET_ASM16("v_mfma_f32_16x16x4_f32");
#undef MDET_ASM16
  } else {
#define MDET_ASM4(INS)                                                                                \
    asm volatile("1:\n\t" MDET_ROUND4(INS) MDET_LOOP_TAIL(12)                                         \
                 : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3])                             \
                 : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(b[0]), "v"(b[1]), "v"(b[2]),       \
                   "v"(b[3]), "s"(cnt)                                                                \
                 : "scc")
    if constexpr (f64) MDET_ASM4("v_mfma_f64_16x16x4_f64");
    else MDET_ASM4("v_mfma_f32_16x16x4_f32");
#undef MDET_ASM4
  }
  T s = 0;
  for (int i = 0; i < NACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(blockIdx.x * 256 + threadIdx.x) & 0xFFFF] = s;
}

template <int NACC>
__global__ __launch_bounds__(256) void mfma_peak_f64_kernel(double* out, int iters) {
  mfma_peak_body<double, d4, NACC>(out, iters);
}
template <int NACC>
__global__ __launch_bounds__(256) void mfma_peak_f32_kernel(float* out, int iters) {
  mfma_peak_body<float, f4, NACC>(out, iters);
}

}  // namespace mdet

extern "C" int mdet_step_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
  if (!dst || !src || bytes % 16 != 0 || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return MDET_EINVAL;
  if (bytes == 0) return MDET_OK;
  const int64_t vecs = (int64_t)(bytes / 16);
  int64_t grid = (vecs + 255) / 256;
  if (grid > 16384) grid = 16384;
  hipLaunchKernelGGL(mdet::copy_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream,
                     (mdet::u32x4*)dst, (const mdet::u32x4*)src, vecs);
  return hipGetLastError() == hipSuccess ? MDET_OK : MDET_EHIP;
}

extern "C" int mdet_step_mfma_peak(int32_t dtype, int32_t accumulators, int32_t workgroups, int32_t iters,
                                   void* out, double* flop, void* stream) {
  if (!out || workgroups <= 0 || iters <= 0 || (dtype != MDET_F64 && dtype != MDET_F32)) return MDET_EINVAL;
  if (accumulators != 4 && accumulators != 16) return MDET_EINVAL;
  const dim3 grid((unsigned)workgroups), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MDET_F64) {
    if (accumulators == 4) hipLaunchKernelGGL(mdet::mfma_peak_f64_kernel<4>, grid, block, 0, st, (double*)out, iters);
    else hipLaunchKernelGGL(mdet::mfma_peak_f64_kernel<16>, grid, block, 0, st, (double*)out, iters);
  } else {
    if (accumulators == 4) hipLaunchKernelGGL(mdet::mfma_peak_f32_kernel<4>, grid, block, 0, st, (float*)out, iters);
    else hipLaunchKernelGGL(mdet::mfma_peak_f32_kernel<16>, grid, block, 0, st, (float*)out, iters);
  }
  if (flop) *flop = (double)workgroups * 4.0 * (double)iters * 16.0 * 2048.0;
  return hipGetLastError() == hipSuccess ? MDET_OK : MDET_EHIP;
}
