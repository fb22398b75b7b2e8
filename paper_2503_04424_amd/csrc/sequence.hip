// C ABI of the principal-minor sequence and the FLODANCE fit (Sec. 3.2, Alg. 2):
// argument checks, workspace layout and kernel launches.  Every call only queues
// work on the caller's stream; nothing is allocated and nothing is waited for.
#include <hip/hip_runtime.h>

#include "../../include/memdet.h"
#include "kernels_sequence.h"

namespace {

using namespace mdet;

inline uint64_t up256(uint64_t x) { return (x + 255) / 256 * 256; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// workspace of mdet_principal_logdets: one double per chunk
inline uint64_t scan_bytes(int64_t n) { return up256((uint64_t)(n > 0 ? ceil_div(n, SEQ_CHUNK) : 1) * 8); }

// workspace of mdet_flodance_fit: the R factors of two consecutive levels of the tree
struct FitLayout {
  int64_t blocks0, blocks1;
  uint64_t bytes0, bytes1;
};
inline FitLayout fit_layout(int64_t rows, int ncols) {
  FitLayout f;
  f.blocks0 = ceil_div(rows > 0 ? rows : 1, FLO_ROWS);
  f.blocks1 = ceil_div(f.blocks0 * ncols, FLO_ROWS);
  f.bytes0 = up256((uint64_t)f.blocks0 * ncols * ncols * 8);
  f.bytes1 = up256((uint64_t)f.blocks1 * ncols * ncols * 8);
  return f;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? MDET_OK : MDET_EHIP; }

}  // namespace

extern "C" {

int mdet_sequence_workspace_query(int64_t n, int64_t rows, int32_t q, uint64_t* bytes) {
  if (!bytes || n < 0 || rows < 0 || q < 0 || q > FLO_MAX_Q) return MDET_EINVAL;
  const FitLayout f = fit_layout(rows, q + 3);
  const uint64_t fit = f.bytes0 + f.bytes1;
  const uint64_t scan = scan_bytes(n);
  *bytes = fit > scan ? fit : scan;
  return MDET_OK;
}

int mdet_principal_logdets(int32_t dtype, const void* d, int64_t n, double* ell, void* workspace,
                           uint64_t workspace_bytes, void* stream) {
  if (n < 0 || (dtype != MDET_F32 && dtype != MDET_F64)) return MDET_EINVAL;
  if (n == 0) return MDET_OK;
  if (!d || !ell || !workspace) return MDET_EINVAL;
  if (workspace_bytes < scan_bytes(n)) return MDET_ENOMEM_DEVICE;
  const int64_t chunks = ceil_div(n, SEQ_CHUNK);
  if (chunks > INT32_MAX) return MDET_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  double* sums = (double*)workspace;
  if (dtype == MDET_F64) {
    hipLaunchKernelGGL((seq_chunk_sums_kernel<double>), dim3((unsigned)chunks), dim3(SEQ_THREADS), 0, st,
                       (const double*)d, n, sums);
    hipLaunchKernelGGL(seq_chunk_offsets_kernel, dim3(1), dim3(SEQ_THREADS), 0, st, sums, chunks);
    hipLaunchKernelGGL((seq_running_sum_kernel<double>), dim3((unsigned)chunks), dim3(SEQ_THREADS), 0, st,
                       (const double*)d, n, (const double*)sums, ell);
  } else {
    hipLaunchKernelGGL((seq_chunk_sums_kernel<float>), dim3((unsigned)chunks), dim3(SEQ_THREADS), 0, st,
                       (const float*)d, n, sums);
    hipLaunchKernelGGL(seq_chunk_offsets_kernel, dim3(1), dim3(SEQ_THREADS), 0, st, sums, chunks);
    hipLaunchKernelGGL((seq_running_sum_kernel<float>), dim3((unsigned)chunks), dim3(SEQ_THREADS), 0, st,
                       (const float*)d, n, (const double*)sums, ell);
  }
  return launch_status();
}

int mdet_flodance_fit(const double* ell, int64_t len, int64_t d, int64_t n0, int64_t ns, int32_t q,
                      double* coef, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!ell || !coef || !workspace) return MDET_EINVAL;
  if (q < 0 || q > FLO_MAX_Q || d < 1 || n0 < 1 || ns <= n0) return MDET_EINVAL;
  if (ns > INT64_MAX / d || ns * d > len) return MDET_EINVAL;
  const int ncols = q + 3;
  const int64_t rows = ns - n0;
  if (rows < q + 2) return MDET_EINVAL;            // fewer samples than coefficients
  const FitLayout f = fit_layout(rows, ncols);
  if (f.blocks0 > INT32_MAX) return MDET_EINVAL;
  if (workspace_bytes < f.bytes0 + f.bytes1) return MDET_ENOMEM_DEVICE;
  hipStream_t st = (hipStream_t)stream;
  double* buf[2] = {(double*)workspace, (double*)((char*)workspace + f.bytes0)};
  const FloProblem pb{ell, d, n0, ns, (int)q};
  // level 0 builds its rows; every further level factors the stacked R's of the one below
  int64_t blocks = f.blocks0;
  hipLaunchKernelGGL(flo_qr_kernel, dim3((unsigned)blocks), dim3(FLO_ROWS), 0, st, pb,
                     (const double*)nullptr, rows, ncols, buf[0], blocks == 1 ? coef : (double*)nullptr);
  int cur = 0;
  while (blocks > 1) {
    const int64_t nrows = blocks * ncols;
    blocks = ceil_div(nrows, FLO_ROWS);
    hipLaunchKernelGGL(flo_qr_kernel, dim3((unsigned)blocks), dim3(FLO_ROWS), 0, st, pb,
                       (const double*)buf[cur], nrows, ncols, buf[cur ^ 1],
                       blocks == 1 ? coef : (double*)nullptr);
    cur ^= 1;
  }
  return launch_status();
}

int mdet_flodance_eval(const double* coef, int32_t q, const double* n_values, int64_t count,
                       double* out, void* stream) {
  if (q < 0 || q > FLO_MAX_Q || count < 0) return MDET_EINVAL;
  if (count == 0) return MDET_OK;
  if (!coef || !n_values || !out) return MDET_EINVAL;
  const int64_t blocks = ceil_div(count, 256);
  if (blocks > INT32_MAX) return MDET_EINVAL;
  hipLaunchKernelGGL(flo_eval_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, coef,
                     (int)q, n_values, count, out);
  return launch_status();
}

}  // extern "C"
