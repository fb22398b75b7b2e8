// Two measuring sticks for the benchmark, behind the same C ABI as the path itself.
//
//  * copy_kernel: a plain copy of a known number of bytes.  What the profiler's memory
//    counters (FETCH_SIZE, WRITE_SIZE) read for it, against the bytes it is known to move,
//    is the scale factor applied to the same counters read for the path's kernels.
//  * mfma_peak_kernel: nothing but matrix-core instructions on registers, accumulators in
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

// Each wavefront: `iters` rounds of 16 products, four accumulators in turn, four products
// in a row on each.  One 16 x 16 x 4 product is 2048 flop in either type.
__global__ __launch_bounds__(256) void mfma_peak_f64_kernel(double* out, int iters) {
  d4 acc[4];
  for (int i = 0; i < 4; ++i) acc[i] = d4{0, 0, 0, 0};
  double a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = threadIdx.x * 1e-3 + i;
    b[i] = 1.0 + threadIdx.x * 1e-4 * (i + 1);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        asm volatile("v_mfma_f64_16x16x4_f64 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a[c]), "v"(b[(i + c) & 3]));
    }
  }
  double s = 0;
  for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(blockIdx.x * 256 + threadIdx.x) & 0xFFFF] = s;
}

__global__ __launch_bounds__(256) void mfma_peak_f32_kernel(float* out, int iters) {
  f4 acc[4];
  for (int i = 0; i < 4; ++i) acc[i] = f4{0, 0, 0, 0};
  float a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = threadIdx.x * 1e-3f + i;
    b[i] = 1.0f + threadIdx.x * 1e-4f * (i + 1);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a[c]), "v"(b[(i + c) & 3]));
    }
  }
  float s = 0;
  for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[(blockIdx.x * 256 + threadIdx.x) & 0xFFFF] = s;
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

extern "C" int mdet_step_mfma_peak(int32_t dtype, int32_t workgroups, int32_t iters, void* out, double* flop,
                                   void* stream) {
  if (!out || workgroups <= 0 || iters <= 0 || (dtype != MDET_F64 && dtype != MDET_F32)) return MDET_EINVAL;
  if (dtype == MDET_F64)
    hipLaunchKernelGGL(mdet::mfma_peak_f64_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                       (double*)out, iters);
  else
    hipLaunchKernelGGL(mdet::mfma_peak_f32_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                       (float*)out, iters);
  if (flop) *flop = (double)workgroups * 4.0 * (double)iters * 16.0 * 2048.0;
  return hipGetLastError() == hipSuccess ? MDET_OK : MDET_EHIP;
}
