// Matrix-core (MFMA) instruction traits for gfx950, 16 x 16 x 4 shapes.
//
// Operand layout of v_mfma_{f64,f32}_16x16x4: lane l supplies A[i = l % 16][k = l / 16]
// and B[k = l / 16][j = l % 16]; the 16 x 16 result is spread over 4 registers per
// lane with column j = l % 16 and a row that depends on the type (acc_row).
#pragma once
#include <hip/hip_runtime.h>

namespace mdet {

template <typename T> struct Mfma;

template <> struct Mfma<double> {
  typedef double acc_t __attribute__((ext_vector_type(4)));
  typedef double vec_t __attribute__((ext_vector_type(2)));   // 16 bytes
  static constexpr int VEC = 2;
  static constexpr int BK = 16;
  static __device__ __forceinline__ acc_t mfma(double a, double b, acc_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
  }
  // row inside the 16 x 16 tile held by accumulator register r of this lane
  static __device__ __forceinline__ int acc_row(int lane, int r) { return 4 * r + (lane >> 4); }
};

template <> struct Mfma<float> {
  typedef float acc_t __attribute__((ext_vector_type(4)));
  typedef float vec_t __attribute__((ext_vector_type(4)));    // 16 bytes
  static constexpr int VEC = 4;
  static constexpr int BK = 32;
  static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int acc_row(int lane, int r) { return 4 * (lane >> 4) + r; }
};

}  // namespace mdet
