// Principal-minor sequence and the FLODANCE regression (Sec. 3.2, Alg. 2).
//
// The LDL^T factorisation yields the log-determinants of all leading principal
// blocks at once, ell_k = sum_{i<=k} log|D_ii| (Sec. 2.1: the diagonal factors give
// every leading principal minor), and Alg. 2 fits a curve to that sequence:
//
//   L_j = ell_{j d} / j,   n_j = n_0 + j   (j = 1 .. n_s - n_0)
//   y_j = n_j (n_j-1)^-1/2 (L_{n_j} - L_{n_0})
//   X_j1 = (n_j-1)^1/2,   X_j,i+1 = -(n_j-1)^-1/2 n_j^(1-i) logGamma(n_j+1),  i = 1 .. q+1
//   beta = argmin |X beta - y|_2,   (c_0, nu_0 .. nu_q) = beta
//   Lhat_n = L_{n_0} + c_0 (1 - 1/n) - sum_{i=1}^{q+1} nu_{i-1} n^-i logGamma(n+1)
//
// Kernels here: the running sum (a three-pass scan), the least-squares problem as a
// tree of Householder QR factorisations of [X y] (one row per thread, 256 rows per
// workgroup; the normal equations X^T X of Alg. 2 would square a condition number
// that grows like n^q), and the evaluation of Lhat_n.  All arithmetic is fp64.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mdet {

// ---------------------------------------------------------------------------
// ell_k = sum_{i<=k} log|d_i|
// ---------------------------------------------------------------------------
constexpr int SEQ_THREADS = 256;
constexpr int SEQ_PER_THREAD = 16;
constexpr int SEQ_CHUNK = SEQ_THREADS * SEQ_PER_THREAD;   // entries per workgroup

// Sum of `v` over the workgroup's 256 threads, the same value in every thread; the
// four wavefronts' sums are added in a fixed order.  `red`: 4 doubles of LDS; two
// barriers inside.
__device__ __forceinline__ double block_sum256(double v, double* red) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return ((red[0] + red[1]) + red[2]) + red[3];
}

template <typename T>
__device__ __forceinline__ double log_abs_entry(const T* __restrict__ d, int64_t i, int64_t n) {
  return i < n ? log(fabs((double)d[i])) : 0.0;
}

// pass 1: one sum per chunk
template <typename T>
__global__ __launch_bounds__(SEQ_THREADS) void seq_chunk_sums_kernel(const T* __restrict__ d, int64_t n,
                                                                    double* __restrict__ sums) {
  __shared__ double red[4];
  const int64_t base = (int64_t)blockIdx.x * SEQ_CHUNK + (int64_t)threadIdx.x * SEQ_PER_THREAD;
  double s = 0.0;
#pragma unroll
  for (int e = 0; e < SEQ_PER_THREAD; ++e) s += log_abs_entry(d, base + e, n);
  s = block_sum256(s, red);
  if (threadIdx.x == 0) sums[blockIdx.x] = s;
}

// pass 2: exclusive running sum of the chunk sums, in order (a few hundred at most):
// one workgroup stages them through LDS, one thread adds them up
__global__ __launch_bounds__(SEQ_THREADS) void seq_chunk_offsets_kernel(double* __restrict__ sums,
                                                                       int64_t nchunks) {
  __shared__ double tile[4 * SEQ_THREADS];
  __shared__ double carry;
  if (threadIdx.x == 0) carry = 0.0;
  for (int64_t base = 0; base < nchunks; base += 4 * SEQ_THREADS) {
    const int64_t m = nchunks - base < 4 * SEQ_THREADS ? nchunks - base : 4 * SEQ_THREADS;
    for (int i = threadIdx.x; i < m; i += SEQ_THREADS) tile[i] = sums[base + i];
    __syncthreads();
    if (threadIdx.x == 0) {
      double run = carry;
      for (int i = 0; i < m; ++i) {
        const double v = tile[i];
        tile[i] = run;
        run += v;
      }
      carry = run;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < m; i += SEQ_THREADS) sums[base + i] = tile[i];
    __syncthreads();
  }
}

// pass 3: running sum inside each chunk on top of its offset
template <typename T>
__global__ __launch_bounds__(SEQ_THREADS) void seq_running_sum_kernel(const T* __restrict__ d, int64_t n,
                                                                     const double* __restrict__ offsets,
                                                                     double* __restrict__ ell) {
  __shared__ double tsum[SEQ_THREADS];
  const int tid = threadIdx.x;
  const int64_t base = (int64_t)blockIdx.x * SEQ_CHUNK + (int64_t)tid * SEQ_PER_THREAD;
  double v[SEQ_PER_THREAD];
  double s = 0.0;
#pragma unroll
  for (int e = 0; e < SEQ_PER_THREAD; ++e) {
    s += log_abs_entry(d, base + e, n);
    v[e] = s;
  }
  tsum[tid] = s;
  __syncthreads();
  // Hillis-Steele scan of the 256 thread sums
  for (int off = 1; off < SEQ_THREADS; off <<= 1) {
    const double add = tid >= off ? tsum[tid - off] : 0.0;
    __syncthreads();
    tsum[tid] += add;
    __syncthreads();
  }
  const double before = offsets[blockIdx.x] + (tid > 0 ? tsum[tid - 1] : 0.0);
#pragma unroll
  for (int e = 0; e < SEQ_PER_THREAD; ++e)
    if (base + e < n) ell[base + e] = before + v[e];
}

// ---------------------------------------------------------------------------
// least squares by a tree of Householder QR factorisations
// ---------------------------------------------------------------------------
constexpr int FLO_MAX_Q = 10;
constexpr int FLO_MAX_COLS = FLO_MAX_Q + 3;      // q + 2 covariates and y
constexpr int FLO_ROWS = 256;                    // rows per workgroup = threads

// What the fit leaves in device memory: beta[0 .. q+1] = (c_0, nu_0 .. nu_q), then
// L_{n_0}, then the residual norm |X beta - y|_2.
struct FloProblem {
  const double* ell;
  int64_t d, n0, ns;
  int q;
};

// Row r (0-based) of [X y] of Alg. 2, P = q + 2 covariates then y.
__device__ __forceinline__ void flo_make_row(const FloProblem& pb, int64_t r, int ncols, double* row) {
  const double Ln0 = pb.ell[pb.n0 * pb.d - 1] / (double)pb.n0;
  const int64_t nj_i = pb.n0 + 1 + r;
  const double nj = (double)nj_i;
  const double Lnj = pb.ell[nj_i * pb.d - 1] / nj;
  const double root = sqrt(nj - 1.0);
  const double lg = lgamma(nj + 1.0);
  row[0] = root;
  double pw = 1.0;                                // n_j^(i-1)
  for (int i = 1; i < ncols - 1; ++i) {
    row[i] = -lg / (root * pw);
    pw *= nj;
  }
  row[ncols - 1] = nj / root * (Lnj - Ln0);
}

// One workgroup reduces up to 256 rows of ncols columns to the upper-triangular
// ncols x ncols factor R of their QR factorisation (Householder reflections; the
// orthogonal factor is never formed).  Level 0 builds its rows from ell, higher
// levels read them from `in` (row-major, nrows x ncols: the stacked R factors of the
// level below).  out: ncols x ncols per workgroup, row-major, zeros below the
// diagonal.  If `coef` is given (last level, one workgroup), thread 0 also solves
// R[0:P, 0:P] beta = R[0:P, P] and writes beta, L_{n_0} and |R[P][P]|.
__global__ __launch_bounds__(FLO_ROWS) void flo_qr_kernel(FloProblem pb, const double* __restrict__ in,
                                                         int64_t nrows, int ncols,
                                                         double* __restrict__ out,
                                                         double* __restrict__ coef) {
  __shared__ double red[2][4][FLO_MAX_COLS];
  __shared__ double pivot_row[2][FLO_MAX_COLS];
  __shared__ double Rs[FLO_MAX_COLS][FLO_MAX_COLS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t r = (int64_t)blockIdx.x * FLO_ROWS + tid;
  double a[FLO_MAX_COLS];
#pragma unroll
  for (int c = 0; c < FLO_MAX_COLS; ++c) a[c] = 0.0;
  if (r < nrows) {
    if (in == nullptr) {
      double row[FLO_MAX_COLS];
      flo_make_row(pb, r, ncols, row);
#pragma unroll
      for (int c = 0; c < FLO_MAX_COLS; ++c) a[c] = c < ncols ? row[c] : 0.0;
    } else {
#pragma unroll
      for (int c = 0; c < FLO_MAX_COLS; ++c) a[c] = c < ncols ? in[r * ncols + c] : 0.0;
    }
  }
  for (int k = 0; k < ncols; ++k) {
    const int buf = k & 1;
    // dot products of column k with columns k.. over rows k.. (row t = thread t)
    double x = 0.0;
#pragma unroll
    for (int c = 0; c < FLO_MAX_COLS; ++c) x = c == k ? a[c] : x;
    const bool in_play = tid >= k;
    double dot[FLO_MAX_COLS];
#pragma unroll
    for (int c = 0; c < FLO_MAX_COLS; ++c) {
      double p = (in_play && c >= k && c < ncols) ? x * a[c] : 0.0;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) p += __shfl_xor(p, off, 64);
      dot[c] = p;
    }
    if (lane == 0) {
#pragma unroll
      for (int c = 0; c < FLO_MAX_COLS; ++c) red[buf][wave][c] = dot[c];
    }
    if (tid == k) {
#pragma unroll
      for (int c = 0; c < FLO_MAX_COLS; ++c) pivot_row[buf][c] = a[c];
    }
    __syncthreads();
    const double sigma = ((red[buf][0][k] + red[buf][1][k]) + red[buf][2][k]) + red[buf][3][k];
    const double xk = pivot_row[buf][k];
    // reflector v = x - alpha e_k, alpha = -sign(x_k) |x|; H = I - 2 v v^T / (v^T v)
    const double alpha = xk > 0.0 ? -sqrt(sigma) : sqrt(sigma);
    const double vtv = 2.0 * (sigma - alpha * xk);
    if (vtv > 0.0) {
      const double v = in_play ? (tid == k ? x - alpha : x) : 0.0;
#pragma unroll
      for (int c = 0; c < FLO_MAX_COLS; ++c) {
        if (c > k && c < ncols) {
          const double xc = ((red[buf][0][c] + red[buf][1][c]) + red[buf][2][c]) + red[buf][3][c];
          const double vta = xc - alpha * pivot_row[buf][c];      // v^T A_c
          a[c] -= (2.0 * vta / vtv) * v;
        }
      }
    }
    // column k becomes (.., alpha, 0, ..)
#pragma unroll
    for (int c = 0; c < FLO_MAX_COLS; ++c)
      if (c == k && in_play) a[c] = tid == k ? (vtv > 0.0 ? alpha : xk) : 0.0;
  }
  // rows 0 .. ncols-1 now hold R
  if (tid < ncols) {
#pragma unroll
    for (int c = 0; c < FLO_MAX_COLS; ++c)
      if (c < ncols) {
        const double v = c >= tid ? a[c] : 0.0;
        out[((int64_t)blockIdx.x * ncols + tid) * ncols + c] = v;
        Rs[tid][c] = v;
      }
  }
  if (coef != nullptr) {
    __syncthreads();
    if (tid == 0) {
      const int P = ncols - 1;
      double beta[FLO_MAX_COLS];
      for (int i = P - 1; i >= 0; --i) {
        double s = Rs[i][P];
        for (int c = i + 1; c < P; ++c) s -= Rs[i][c] * beta[c];
        beta[i] = s / Rs[i][i];
      }
      for (int i = 0; i < P; ++i) coef[i] = beta[i];
      coef[P] = pb.ell[pb.n0 * pb.d - 1] / (double)pb.n0;
      coef[P + 1] = fabs(Rs[P][P]);
    }
  }
}

// Lhat_n for each n in n_values (last step of Alg. 2)
__global__ void flo_eval_kernel(const double* __restrict__ coef, int q, const double* __restrict__ n_values,
                                int64_t count, double* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const double n = n_values[i];
  const double lg = lgamma(n + 1.0);
  double acc = coef[q + 2] + coef[0] * (1.0 - 1.0 / n);
  double pw = n;                                   // n^i
  for (int t = 1; t <= q + 1; ++t) {
    acc -= coef[t] * lg / pw;
    pw *= n;
  }
  out[i] = acc;
}

}  // namespace mdet
