// C ABI, host scheduler and kernel launchers of the MI355X log-determinant library.
//
// The path (symmetric / LDL^T case of the paper's memory-constrained algorithm,
// Sec. 2.2 and App. D), one block column k at a time:
//   1. factor the block column: its diagonal block in place (A_kk = L D L^T) and
//      the rows below it (L_ik = A_ik L_kk^-T D^-1), recursively by halves down to
//      64-column leaves, every product inside it on the matrix cores;
//   2. reduce log|d| and sign of its pivots;
//   3. Schur-update every block of the trailing lower triangle:
//      A_ij -= L_ik D_k L_jk^T   (full products off the diagonal, lower-triangle
//      "Gramian" products on it);
// and, when the matrix does not fit the device budget, block columns are kept
// resident a group at a time while factored columns stream past from host memory.
#include <hip/hip_runtime.h>

#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <functional>
#include <memory>
#include <mutex>
#include <new>
#include <thread>
#include <type_traits>
#include <vector>

#include "../../include/memdet.h"
#include "kernels_leaf.h"
#include "kernels_pivot_block.h"
#include "kernels_reduce.h"
#include "kernels_update.h"
#include "plan.h"

namespace mdet {

// ---------------------------------------------------------------------------
// error plumbing
// ---------------------------------------------------------------------------
struct HipFail {
  hipError_t code = hipSuccess;
  bool ok() const { return code == hipSuccess; }
  void check(hipError_t e) { if (code == hipSuccess && e != hipSuccess) code = e; }
};

#define MDET_HIP(ctx, call) (ctx).check((call))

// ---------------------------------------------------------------------------
// per-device stream / event cache (streams are created once and reused)
// ---------------------------------------------------------------------------
// Streams of one device, created on first use and kept for the life of the process.
// The runtime multiplexes streams onto a few hardware queues (four by default), and
// a wait at the head of a hardware queue holds up every stream that shares it; so
// the two compute streams are created first, and the two copy streams only when a
// host entry point needs them.
struct StreamSet {
  hipStream_t main = nullptr, side = nullptr, h2d = nullptr, d2h = nullptr;
  bool ready = false, copy_ready = false;
};
static std::mutex g_mu;
static StreamSet g_streams[64];

static hipError_t get_streams(int dev, StreamSet** out, bool with_copy_streams) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  StreamSet& s = g_streams[dev];
  hipError_t e;
  if (!s.ready) {
    if ((e = hipStreamCreateWithFlags(&s.main, hipStreamNonBlocking)) != hipSuccess) return e;
    if ((e = hipStreamCreateWithFlags(&s.side, hipStreamNonBlocking)) != hipSuccess) return e;
    s.ready = true;
  }
  if (with_copy_streams && !s.copy_ready) {
    if ((e = hipStreamCreateWithFlags(&s.h2d, hipStreamNonBlocking)) != hipSuccess) return e;
    if ((e = hipStreamCreateWithFlags(&s.d2h, hipStreamNonBlocking)) != hipSuccess) return e;
    s.copy_ready = true;
  }
  *out = &s;
  return hipSuccess;
}

// Events with timing, for MDET_FLAG_PROFILE: taken from and returned to a free list
// kept for the life of the process (creating one costs the calling thread about as
// much as a kernel launch).
static std::vector<hipEvent_t> g_timing_events;
static hipEvent_t timing_event_get(HipFail* fail) {
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_timing_events.empty()) {
      hipEvent_t e = g_timing_events.back();
      g_timing_events.pop_back();
      return e;
    }
  }
  hipEvent_t e = nullptr;
  fail->check(hipEventCreate(&e));
  return e;
}
static void timing_event_put(hipEvent_t e) {
  if (!e) return;
  std::lock_guard<std::mutex> lk(g_mu);
  g_timing_events.push_back(e);
}

// A small pool of reusable events (timing disabled).
struct EventPool {
  std::vector<hipEvent_t> ev;
  size_t next = 0;
  HipFail* fail;
  explicit EventPool(HipFail* f) : fail(f) {}
  hipEvent_t get() {
    if (next == ev.size()) {
      hipEvent_t e = nullptr;
      fail->check(hipEventCreateWithFlags(&e, hipEventDisableTiming));
      ev.push_back(e);
    }
    return ev[next++];
  }
  ~EventPool() { for (auto e : ev) if (e) (void)hipEventDestroy(e); }
};

// ---------------------------------------------------------------------------
// kernel launchers
// ---------------------------------------------------------------------------
template <typename T>
struct Launcher {
  HipFail* fail;
  T* dvec = nullptr;
  T* dinv = nullptr;
  T* linv = nullptr;          // inverses of a leaf's diagonal sub-blocks (see linv_of)
  // 64 x 64 elements (or none): where leaf_pair_kernel leaves the solved rows of the
  // second leaf of a pair until the next solve launch copies them into place.  With it
  // linv is two arrays, used by leaves in turn: that kernel reads one leaf's while one
  // of its workgroups already writes the next leaf's.
  T* l10 = nullptr;
  const T* fix_src = nullptr; // pending copy for the next solve launch
  T* fix_dst = nullptr;
  int64_t fix_ld = 0;
  DevFlags* flags = nullptr;
  bool spd = false;           // positive-definite form (MDET_FLAG_ASSUME_SPD)
  // n indices (or none): every leaf is factored with the pivot taken from its own
  // diagonal, and perm[j] is the row/column of the input that ended at position j
  // (MDET_FLAG_PIVOT).  The leaf then has a launch of its own.
  int* perm = nullptr;
  // MDET_FLAG_PIVOT_BLOCK: the pivot is looked for on the whole diagonal block of a block
  // column (see kernels_pivot_block.h); the workspace it needs, or none
  struct PivotBlock {
    T* S = nullptr;
    T* Lfull = nullptr;
    T* Y = nullptr;
    T* Bg = nullptr;
    T* leaf = nullptr;
    T* linv = nullptr;
    T* dg = nullptr;
    int* active = nullptr;
    int* piv = nullptr;
    PbCand* part = nullptr;       // two sets of 64, used in turn
    int64_t ldl = 0, max_w = 0, max_below = 0;
  } pb;
  // General matrices (MDET_FLAG_GENERAL; Sec. 2.2, Eq. 1: M = P L U): distance in elements
  // from an entry (i, j), i >= j, of the array the driver works on to the place that holds
  // entry (j, i) of the matrix, in a second array of the same shape.  Every pointer the
  // driver passes refers to the first array; 0 = symmetric matrix, no second array.
  int64_t qoff = 0;
  T* linv_u = nullptr;        // with qoff: the inverses of the sub-blocks of a leaf's U^T (linv: of its L)
  // Two arrays of n x wld elements (or none): while a block column is factored its rows
  // are also stored scaled by the pivots, W = L D, so that the updates that use the
  // column read their left operand ready-made (MDET_FLAG_SCALED_COPY).  Column k uses
  // wbuf[k & 1]: its bulk update may still be reading while column k + 1 is factored.
  T* wbuf[2] = {nullptr, nullptr};
  int64_t wld = 0;
  int slots = 0;              // trailing-update workgroups the device holds at one time
  double fma = 0.0;
  uint64_t launches = 0;
  // optional timing of the trailing-update launches (MDET_FLAG_PROFILE): every launch of
  // the two trailing-update kernels (kind 0: 128 x 128 blocks, kind 1: 64 x 64 blocks)
  // bracketed by events on its own stream; prof_ref, recorded once at the start of the
  // call, places the launches on one time axis
  bool profile = false;
  struct ProfLaunch { hipEvent_t e0, e1; int kind; };
  std::vector<ProfLaunch> prof_events;
  hipEvent_t prof_ref = nullptr;
  double prof_fma[2] = {0.0, 0.0};

  static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

  // C[M x N] -= A[M x K] diag(d) B[N x K]^T ; lower: only column <= row.
  // trailing = true marks the Schur update of the trailing matrix by a whole block
  // column (as opposed to the updates inside a block column's own factorisation);
  // it runs the same code under its own kernel name so profiles tell them apart.
  // fuse: the launch also factors the leaf at C's top-left corner (lower only).
  // leave_free >= 0 (trailing only): several launches in a row, each that many
  // workgroups short of what the device holds, so that other streams' kernels find room.
  int update(hipStream_t st, T* C, int64_t ldc, const T* A, int64_t lda, const T* B, int64_t ldb,
             const T* d, int64_t M, int64_t N, int64_t K, bool lower, bool trailing = false,
             const FusedLeaf<T>* fuse = nullptr, int leave_free = -1, bool a_scaled = false) {
    // general matrix: one launch updates both arrays (see update_one)
    return update_one(st, C, ldc, A, lda, B, ldb, d, M, N, K, lower, trailing, qoff ? nullptr : fuse, leave_free,
                      qoff ? false : a_scaled);
  }

  int update_one(hipStream_t st, T* C, int64_t ldc, const T* A, int64_t lda, const T* B, int64_t ldb,
                 const T* d, int64_t M, int64_t N, int64_t K, bool lower, bool trailing,
                 const FusedLeaf<T>* fuse, int leave_free, bool a_scaled) {
    // a_scaled: A holds rows of L D already (see wbuf): same kernels as the
    // positive-definite form, which read no pivots
    const bool scaled = spd || a_scaled;
    if (M <= 0 || N <= 0 || K <= 0) return MDET_OK;
    if (lower && N > M) N = M;     // columns right of the last row lie above the diagonal
    constexpr int vec = 16 / (int)sizeof(T);
    if (K % 64 != 0 || lda % vec != 0 || ldb % vec != 0 || !aligned16(A) || !aligned16(B) ||
        !aligned16(d) || M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || ldc < N)
      return MDET_EINVAL;
    // the kernels address an operand's 128-row strip with 32-bit byte offsets
    if ((uint64_t)lda * sizeof(T) * 128 >= (1ull << 32) || (uint64_t)ldb * sizeof(T) * 128 >= (1ull << 32))
      return MDET_EINVAL;
    // kernel choice: the trailing update always uses 128 x 128 blocks; inside a
    // block column a K = 64 update runs single-shot from LDS and short launches
    // use 64 x 64 blocks so that they reach more compute units
    const bool leaf_k = !trailing && K == 64;
    // general matrix: the launch has two rows of workgroups, one per array
    const int64_t dual = qoff != 0 ? 2 : 1;
    if (dual == 2 && (spd || a_scaled || fuse || (qoff * (int64_t)sizeof(T)) % 16 != 0)) return MDET_EINVAL;
    const int64_t wg128 = dual * 8 * update_grid(M, N, lower, 128).per;
    const bool small = !trailing && !leaf_k && wg128 < 1024;
    // A trailing update whose 128 x 128 blocks would not fill the device's slots (the
    // next block column of a small matrix, the bulk of the last few block columns)
    // lasts as long as one workgroup's walk along K, twice that where two workgroups
    // share a compute unit; 64 x 64 blocks quarter the walk and spread evenly
    // (n = 8192: the seven next-column updates 1.48 -> 1.20 ms; measured cross-over at
    // about 0.8 of the slots).
    const bool small_trailing = trailing && slots > 0 && 5 * wg128 <= 4 * slots;
    const int tile = (leaf_k || small || small_trailing) ? 64 : 128;
    const UpdGrid ug = update_grid(M, N, lower, tile);
    if (8 * ug.per > INT32_MAX) return MDET_EINVAL;
    FusedLeaf<T> fl{0, nullptr, nullptr, nullptr, 0, nullptr, 0};
    if (fuse && !perm) {
      if (!lower || fuse->w > LEAF || fuse->w > N || fuse->w > M) return MDET_EINVAL;
      fl = *fuse;
    }
    // workgroups per launch and XCD: everything at once, or rounds that fill all but
    // leave_free of the device's slots
    int64_t per_launch = ug.per;
    if (trailing && !small_trailing && leave_free >= 0 && slots - leave_free >= 8 * dual &&
        dual * 8 * ug.per > slots - leave_free)
      per_launch = (slots - leave_free) / (8 * dual);
    dim3 block(UPD_THREADS);
    const bool timed = profile && trailing;
    for (int64_t k0 = 0; k0 < ug.per; k0 += per_launch) {
      const int64_t kn = ug.per - k0 < per_launch ? ug.per - k0 : per_launch;
      dim3 grid((unsigned)(8 * kn));
      hipEvent_t e0 = nullptr, e1 = nullptr;
      if (timed) {
        e0 = timing_event_get(fail);
        e1 = timing_event_get(fail);
        fail->check(hipEventRecord(e0, st));
      }
#define MDET_LAUNCH_UPD_AS(KERNEL, SCALED)                                                         \
  hipLaunchKernelGGL((KERNEL<T, SCALED>), grid, block, 0, st, C, ldc, A, lda, B, ldb, d, (int)M,  \
                     (int)N, (int)K, ug.nsn, ug.swl, (int)lower, (int)ug.per, (int)k0, fl)
#define MDET_LAUNCH_UPD(KERNEL)                                                                   \
  do {                                                                                            \
    if (scaled) MDET_LAUNCH_UPD_AS(KERNEL, true);                                                 \
    else MDET_LAUNCH_UPD_AS(KERNEL, false);                                                       \
  } while (0)
      if (dual == 2) {
        const dim3 grid2((unsigned)(8 * kn), 2);
#define MDET_LAUNCH_GENERAL(KERNEL)                                                                 \
  hipLaunchKernelGGL((KERNEL<T>), grid2, block, 0, st, C, ldc, A, lda, B, ldb, d, (int)M, (int)N,   \
                     (int)K, ug.nsn, ug.swl, (int)lower, (int)ug.per, (int)k0, qoff)
        if (small_trailing) MDET_LAUNCH_GENERAL(trailing_update64_general_kernel);
        else if (trailing) MDET_LAUNCH_GENERAL(trailing_update_general_kernel);
        else if (leaf_k)
          hipLaunchKernelGGL((leaf_update_general_kernel<T>), grid2, block, 0, st, C, ldc, A, lda, B, ldb, d,
                             (int)M, (int)N, ug.nsn, ug.swl, (int)lower, (int)ug.per, qoff);
        else if (small) MDET_LAUNCH_GENERAL(panel_update64_general_kernel);
        else MDET_LAUNCH_GENERAL(panel_update_general_kernel);
#undef MDET_LAUNCH_GENERAL
      } else if (small_trailing) MDET_LAUNCH_UPD(trailing_update64_kernel);
      else if (trailing) MDET_LAUNCH_UPD(trailing_update_kernel);
      else if (leaf_k) {
        if (scaled)
          hipLaunchKernelGGL((leaf_update_kernel<T, true>), grid, block, 0, st, C, ldc, A, lda, B, ldb,
                             d, (int)M, (int)N, ug.nsn, ug.swl, (int)lower, (int)ug.per, fl);
        else
          hipLaunchKernelGGL((leaf_update_kernel<T, false>), grid, block, 0, st, C, ldc, A, lda, B, ldb,
                             d, (int)M, (int)N, ug.nsn, ug.swl, (int)lower, (int)ug.per, fl);
      } else if (small) MDET_LAUNCH_UPD(panel_update64_kernel);
      else MDET_LAUNCH_UPD(panel_update_kernel);
#undef MDET_LAUNCH_UPD
#undef MDET_LAUNCH_UPD_AS
      ++launches;
      if (timed) {
        fail->check(hipEventRecord(e1, st));
        prof_events.push_back(ProfLaunch{e0, e1, small_trailing ? 1 : 0});
      }
    }
    fail->check(hipGetLastError());
    double f;
    if (lower) {
      // entries (r, c), c <= r, of an M x N trapezoid whose (0,0) is on the diagonal
      double t = (double)(M < N ? M : N);
      f = (t * (t + 1) / 2 + (double)(M - (int64_t)t) * (double)N) * (double)K;
    } else {
      f = (double)M * (double)N * (double)K;
    }
    f *= (double)dual;
    fma += f;
    if (timed) prof_fma[small_trailing ? 1 : 0] += f;
    return MDET_OK;
  }

  // Workgroup slots the bulk update leaves to the factorisation of a block column
  // of m rows that runs beside it; -1: none, the update is one launch.  Leaving
  // room pays while that factorisation is a chain of short, latency-bound kernels
  // (measured: a gain up to about 8192 rows, a small loss at 16384 and beyond, where
  // its own updates are large enough to want the whole device in turn).
  int leave_free_for(int64_t m) const {
    if (slots <= 0 || m > 8192) return -1;
    return slots / 8;
  }

  // What an update launch needs to factor the leaf of width w whose first pivot has
  // index d0 (see FusedLeaf).
  FusedLeaf<T> fused_leaf(int64_t w, int64_t d0) const {
    return FusedLeaf<T>{(int)(w < LEAF ? w : LEAF), dvec + d0, dinv + d0, linv_of(d0), (long long)d0, flags,
                        spd ? 1 : 0};
  }
  // The array that holds the inverses of the leaf whose first pivot has index d0.
  T* linv_of(int64_t d0) const { return l10 ? linv + ((d0 / LEAF) & 1) * (LEAF * SUB) : linv; }

  // Factor block column: P at its diagonal entry, m rows, w columns (w <= m).
  // d0: index of its first pivot in dvec/dinv.  first_done: the first leaf has
  // been factored already, by the update launch that produced it.
  // Wp, if given, points at the same entry of the column's pivot-scaled copy (leading
  // dimension wld): the rows from wskip on (those below the block column's diagonal
  // block, which the trailing updates read) are written there too.  The updates inside
  // the column keep scaling on the fly: with one array for both operands they read
  // half as much (measured at n = 8192: 6.66 ms against 6.97).
  int factor_cols(hipStream_t st, T* P, int64_t ld, int64_t m, int64_t w, int64_t d0,
                  bool first_done = false, T* Wp = nullptr, int64_t wskip = 0) {
    if (w <= 0) return MDET_OK;
    if (pb.S != nullptr) return factor_cols_pivot_block(st, P, ld, m, w, d0);
    if (w <= LEAF && qoff != 0) {
      // P A = L D U of the leaf, then the rows below it in both halves: the lower half
      // against U^T, the transposed upper half against L with the leaf's row order
      if (spd || !perm || !linv_u) return MDET_EINVAL;
      T* linvL = linv;
      T* linvU = linv_u;
      hipLaunchKernelGGL((leaf_lu_kernel<T, LU_WAVES>), dim3(1), dim3(64 * LU_WAVES), 0, st, P, P + qoff, ld,
                         (int)w, dvec + d0, dinv + d0, linvL, linvU, perm + d0, (long long)d0, flags);
      fail->check(hipGetLastError());
      ++launches;
      fma += ((double)w * w * w - (double)w) / 3.0;
      const int64_t below = m - w;
      if (below > 0) {
        if (below > INT32_MAX) return MDET_EINVAL;
        const int64_t nblk = (below + SOLVE_ROWS - 1) / SOLVE_ROWS;
        hipLaunchKernelGGL((leaf_solve_general_kernel<T>), dim3((unsigned)nblk, 2), dim3(256), 0, st, P + w * ld,
                           ld, (int)below, (int)w, (const T*)P, (const T*)(dinv + d0), (const T*)linvL,
                           (const T*)linvU, (const T*)(dvec + d0), (const int*)(perm + d0), (int)d0, qoff);
        fail->check(hipGetLastError());
        ++launches;
        fma += 2.0 * (double)below * ((double)w * (w - 1) / 2.0);
      }
      return MDET_OK;
    }
    if (w <= LEAF) {
      if (perm) {
        if (spd) return MDET_EINVAL;
        hipLaunchKernelGGL((leaf_factor_pivoted_kernel<T>), dim3(1), dim3(FACTOR_THREADS), 0, st, P, ld,
                           (int)w, dvec + d0, dinv + d0, linv_of(d0), perm + d0, (long long)d0, flags);
        fail->check(hipGetLastError());
        ++launches;
      } else if (!first_done) {
        hipLaunchKernelGGL((leaf_factor_kernel<T>), dim3(1), dim3(FACTOR_THREADS), 0, st, P, ld,
                           (int)w, dvec + d0, dinv + d0, linv_of(d0), (long long)d0, flags, spd ? 1 : 0);
        fail->check(hipGetLastError());
        ++launches;
      }
      fma += ((double)w * w * w - (double)w) / 6.0;
      int64_t below = m - w;
      if (below > 0) {
        if (below > INT32_MAX) return MDET_EINVAL;
        int64_t nblk = (below + SOLVE_ROWS - 1) / SOLVE_ROWS;
        hipLaunchKernelGGL((leaf_solve_kernel<T>), dim3((unsigned)(nblk + (fix_src ? 1 : 0))), dim3(256), 0,
                           st, P + w * ld, ld, (int)below, (int)w, (const T*)P, ld,
                           (const T*)(dinv + d0), (const T*)linv_of(d0), Wp ? Wp + w * wld : (T*)nullptr, wld,
                           (const T*)(dvec + d0), (int)(wskip > w ? wskip - w : 0),
                           perm ? (const int*)(perm + d0) : (const int*)nullptr, (int)d0, fix_src, fix_dst,
                           fix_ld);
        fix_src = nullptr;
        fail->check(hipGetLastError());
        ++launches;
        fma += (double)below * ((double)w * (w - 1) / 2.0);
      }
      return MDET_OK;
    }
    // Two whole leaves with rows below them: the first leaf's solve, the update of the
    // second leaf's columns and the second leaf's factorisation are one launch.  The
    // solve launch of the second leaf, which must exist, puts a block in place that this
    // one leaves aside.
    if (w == 2 * LEAF && m > w && l10 && !perm && m - LEAF <= INT32_MAX) {
      if (!first_done) {
        hipLaunchKernelGGL((leaf_factor_kernel<T>), dim3(1), dim3(FACTOR_THREADS), 0, st, P, ld, (int)LEAF,
                           dvec + d0, dinv + d0, linv_of(d0), (long long)d0, flags, spd ? 1 : 0);
        ++launches;
      }
      const int64_t below = m - LEAF;
      const FusedLeaf<T> fl = fused_leaf(LEAF, d0 + LEAF);
      const dim3 grid((unsigned)((below + SOLVE_ROWS - 1) / SOLVE_ROWS)), block(256);
      T* Wrows = Wp ? Wp + LEAF * wld : (T*)nullptr;
      const int wfrom = (int)(wskip > LEAF ? wskip - LEAF : 0);
      if (spd)
        hipLaunchKernelGGL((leaf_pair_kernel<T, true>), grid, block, 0, st, P + LEAF * ld, ld, (int)below,
                           (const T*)P, ld, (const T*)(dinv + d0), (const T*)linv_of(d0),
                           (const T*)(dvec + d0), Wrows, wld, wfrom, l10, fl);
      else
        hipLaunchKernelGGL((leaf_pair_kernel<T, false>), grid, block, 0, st, P + LEAF * ld, ld, (int)below,
                           (const T*)P, ld, (const T*)(dinv + d0), (const T*)linv_of(d0),
                           (const T*)(dvec + d0), Wrows, wld, wfrom, l10, fl);
      fail->check(hipGetLastError());
      ++launches;
      fma += ((double)LEAF * LEAF * LEAF - (double)LEAF) / 6.0;                 // first leaf
      fma += (double)below * ((double)LEAF * (LEAF - 1) / 2.0);                  // its solve
      fma += ((double)LEAF * (LEAF + 1) / 2 + (double)(below - LEAF) * LEAF) * LEAF;   // the update
      fix_src = l10;
      fix_dst = P + LEAF * ld;
      fix_ld = ld;
      return factor_cols(st, P + LEAF * ld + LEAF, ld, below, LEAF, d0 + LEAF, true,
                         Wp ? Wp + LEAF * wld + LEAF : (T*)nullptr, wskip > LEAF ? wskip - LEAF : 0);
    }
    // split at a multiple of the leaf width nearest the middle
    int64_t leaves = (w + LEAF - 1) / LEAF;
    int64_t w1 = (leaves / 2) * LEAF;
    int rc = factor_cols(st, P, ld, m, w1, d0, first_done, Wp, wskip);
    if (rc != MDET_OK) return rc;
    // columns [w1, w), rows [w1, m)  -=  L[rows, 0:w1] D L[cols, 0:w1]^T, and the
    // first leaf of those columns factored by the same launch
    T* C = P + w1 * ld + w1;
    const T* A = P + w1 * ld;
    const FusedLeaf<T> fl = fused_leaf(w - w1, d0 + w1);
    rc = update(st, C, ld, A, ld, A, ld, dvec + d0, m - w1, w - w1, w1, true, false, &fl);
    if (rc != MDET_OK) return rc;
    return factor_cols(st, C, ld, m - w1, w - w1, d0 + w1, true, Wp ? Wp + w1 * wld + w1 : (T*)nullptr,
                       wskip > w1 ? wskip - w1 : 0);
  }

  // Start of the profiled region (MDET_FLAG_PROFILE): the origin of the launches' time axis.
  void profile_begin(hipStream_t st) {
    if (!profile) return;
    prof_ref = timing_event_get(fail);
    fail->check(hipEventRecord(prof_ref, st));
  }

  // A whole block column with the pivots taken from anywhere on its w x w diagonal block
  // (MDET_FLAG_PIVOT_BLOCK; the scheme is described in kernels_pivot_block.h).  Same
  // arguments and same result layout as factor_cols: L and D in pivot order in place,
  // dvec / dinv / perm filled for the columns d0 .. d0 + w.
  int factor_cols_pivot_block(hipStream_t st, T* P, int64_t ld, int64_t m, int64_t w, int64_t d0) {
    if (spd || qoff != 0 || !perm || w > pb.max_w || m - w > pb.max_below || m > INT32_MAX) return MDET_EINVAL;
    const int64_t ldl = pb.ldl, below = m - w;
    const int nparts = (int)((w + PB_THREADS - 1) / PB_THREADS);
    if (nparts > 64) return MDET_EINVAL;
    PbCand* part[2] = {pb.part, pb.part + 64};
    const int64_t nt = (w + 31) / 32;
    hipLaunchKernelGGL((pb_symmetrize_kernel<T>), dim3((unsigned)(nt * nt)), dim3(256), 0, st, (const T*)P, ld, (int)w,
                       pb.S, ldl);
    hipLaunchKernelGGL((pb_init_kernel<T>), dim3((unsigned)nparts), dim3(PB_THREADS), 0, st, (const T*)P, ld, (int)w,
                       pb.Lfull, ldl, pb.dg, pb.active, part[0]);
    fail->check(hipGetLastError());
    launches += 2;
    int cur = 0;
    int rc = MDET_OK;
    for (int64_t c0 = 0; c0 < w && rc == MDET_OK; c0 += LEAF) {
      const int lw = (int)(w - c0 < LEAF ? w - c0 : LEAF);
      for (int jj = 0; jj < lw; ++jj) {
        hipLaunchKernelGGL((pb_step_kernel<T>), dim3((unsigned)nparts), dim3(PB_THREADS), 0, st, (const T*)pb.S, ldl,
                           pb.Lfull, ldl, pb.dg, pb.active, (const PbCand*)part[cur], part[cur ^ 1], nparts, pb.piv,
                           dvec + d0, dinv + d0, perm + d0, (int)w, (int)c0, jj, (long long)d0, flags);
        cur ^= 1;
        ++launches;
      }
      fail->check(hipGetLastError());
      fma += (double)w * lw * (lw - 1) / 2.0;
      hipLaunchKernelGGL((pb_leaf_kernel<T>), dim3(1), dim3(256), 0, st, (const T*)pb.Lfull, ldl, (const int*)pb.piv,
                         (int)c0, lw, pb.leaf, pb.linv);
      fail->check(hipGetLastError());
      ++launches;
      // candidates remain: the diagonal block up to date with this group's 64 pivots
      if (c0 + lw < w)
        rc = update(st, pb.S, ldl, pb.Lfull + c0, ldl, pb.Lfull + c0, ldl, dvec + d0 + c0, w, w, LEAF, false);
      if (below > 0 && rc == MDET_OK) {
        const unsigned grid = (unsigned)std::min<int64_t>((below + 3) / 4, 2048);
        hipLaunchKernelGGL((pb_gather_kernel<T>), dim3(grid), dim3(256), 0, st, (const T*)(P + w * ld), ld, below, pb.Y,
                           ldl, (const T*)pb.Lfull, ldl, pb.Bg, ldl, (const int*)pb.piv, (int)c0, lw);
        fail->check(hipGetLastError());
        ++launches;
        // the gathered columns receive everything solved before: Y_new -= Y_old D Bg^T
        if (c0 > 0) rc = update(st, pb.Y + c0, ldl, pb.Y, ldl, pb.Bg, ldl, dvec + d0, below, lw, c0, false);
        if (rc != MDET_OK) break;
        const int64_t nblk = (below + SOLVE_ROWS - 1) / SOLVE_ROWS;
        hipLaunchKernelGGL((leaf_solve_kernel<T>), dim3((unsigned)nblk), dim3(256), 0, st, pb.Y + c0, ldl, (int)below,
                           lw, (const T*)pb.leaf, (int64_t)LEAF, (const T*)(dinv + d0 + c0), (const T*)pb.linv,
                           (T*)nullptr, (int64_t)0, (const T*)(dvec + d0 + c0), 0, (const int*)nullptr, 0,
                           (const T*)nullptr, (T*)nullptr, (int64_t)0);
        fail->check(hipGetLastError());
        ++launches;
        fma += (double)below * ((double)lw * (lw - 1) / 2.0);
      }
    }
    if (rc != MDET_OK) return rc;
    const unsigned grid = (unsigned)std::min<int64_t>(m, 4096);
    hipLaunchKernelGGL((pb_store_kernel<T>), dim3(grid), dim3(256), 0, st, P, ld, m, (int)w, (const T*)pb.Lfull, ldl,
                       (const int*)pb.piv, (const T*)(dvec + d0), (const T*)pb.Y, ldl);
    fail->check(hipGetLastError());
    ++launches;
    return MDET_OK;
  }

  // After all streams are idle: per kernel the number of timed launches, the sum of their
  // durations and their flops; and the length of the union of all their intervals, i.e. the
  // time during which at least one trailing-update launch was running (launches on the two
  // compute streams overlap, so the sum of the durations counts some time twice).
  void collect_profile(mdet_result* res) {
    double ms_sum[2] = {0.0, 0.0};
    uint64_t count[2] = {0, 0};
    std::vector<std::pair<double, double>> iv;
    iv.reserve(prof_events.size());
    for (auto& pr : prof_events) {
      float ms = 0.f, at = 0.f;
      if (hipEventElapsedTime(&ms, pr.e0, pr.e1) == hipSuccess) {
        ms_sum[pr.kind] += ms;
        ++count[pr.kind];
        if (prof_ref && hipEventElapsedTime(&at, prof_ref, pr.e0) == hipSuccess)
          iv.emplace_back((double)at, (double)at + (double)ms);
      }
      timing_event_put(pr.e0);
      timing_event_put(pr.e1);
    }
    std::sort(iv.begin(), iv.end());
    double busy = 0.0, lo = 0.0, hi = -1.0;
    for (auto& x : iv) {
      if (hi < lo || x.first > hi) {
        if (hi > lo) busy += hi - lo;
        lo = x.first;
        hi = x.second;
      } else if (x.second > hi) {
        hi = x.second;
      }
    }
    if (hi > lo) busy += hi - lo;
    res->trailing_update_launches = count[0];
    res->t_trailing_update = ms_sum[0] * 1e-3;
    res->trailing_update_flops = 2.0 * prof_fma[0];
    res->trailing_update64_launches = count[1];
    res->t_trailing_update64 = ms_sum[1] * 1e-3;
    res->trailing_update64_flops = 2.0 * prof_fma[1];
    res->t_trailing_update_busy = busy * 1e-3;
    prof_events.clear();
    timing_event_put(prof_ref);
    prof_ref = nullptr;
  }

  void reduce(hipStream_t st, int64_t n, int64_t bs, int64_t T_, double* partial, double* out,
              double* running) {
    if (T_ > 0) {
      hipLaunchKernelGGL((logdet_partial_kernel<T>), dim3((unsigned)T_), dim3(RED_THREADS), 0, st,
                         (const T*)dvec, n, bs, partial);
      fail->check(hipGetLastError());
      ++launches;
    }
    hipLaunchKernelGGL(logdet_combine_kernel, dim3(1), dim3(64), 0, st, (const double*)partial, T_,
                       out, running);
    fail->check(hipGetLastError());
    ++launches;
  }
};

// One block column as the device sees it: `base` points at its diagonal entry.
template <typename T>
struct ColRef {
  T* base;
  int64_t ld;
};

// ---------------------------------------------------------------------------
// in-core driver: right-looking over block columns, optional look-ahead
// ---------------------------------------------------------------------------
// cols[j] for j in [jb, je) must be resident and hold columns already updated by
// every block column < jb.  `dense`: all columns live in one row-major array, so
// the bulk of a trailing update can be a single launch.
// Hooks let the out-of-core driver wait for a column's upload before its first use
// on a stream and start its write-back as soon as it is final.
struct ResidentHooks {
  std::function<void(hipStream_t, int64_t)> before_touch;   // (stream, column)
  std::function<void(int64_t)> column_final;                // column k factored (on s0)
  // Called once the work of the step after column k's has been queued: the place for
  // anything that may block the calling thread (a copy to pageable host memory does),
  // since the device then has a whole step of kernels to run meanwhile.
  std::function<void(int64_t)> column_flush;
};

template <typename T>
static int factor_resident(Launcher<T>& L, const Plan& pl, std::vector<ColRef<T>>& cols, int64_t jb,
                           int64_t je, bool dense, bool lookahead, hipStream_t s0, hipStream_t s1,
                           EventPool& events, const ResidentHooks* hooks = nullptr) {
  const int64_t bs = pl.bs, n = pl.n;
  hipEvent_t ev_bulk_prev = nullptr;
  if (!lookahead) s1 = s0;
  auto touch = [&](hipStream_t st, int64_t j) {
    if (hooks && hooks->before_touch) hooks->before_touch(st, j);
  };
  for (int64_t k = jb; k < je; ++k) {
    const int64_t wk = pl.col_width(k);
    const int64_t mk = n - k * bs;
    touch(s0, k);
    // every column but the group's first had its first leaf factored by the update
    // launch that finished it
    T* Wk = L.wbuf[0] ? L.wbuf[k & 1] : nullptr;      // this column's pivot-scaled copy
    int rc = L.factor_cols(s0, cols[k].base, cols[k].ld, mk, wk, k * bs, k > jb, Wk, wk);
    if (rc != MDET_OK) return rc;
    // left operand of the updates by column k: rows from block row j down
    auto left = [&](int64_t j) -> const T* {
      return Wk ? Wk + (j - k) * bs * L.wld : cols[k].base + (j - k) * bs * cols[k].ld;
    };
    const int64_t lda_k = Wk ? L.wld : cols[k].ld;
    if (hooks && hooks->column_final) hooks->column_final(k);
    if (k + 1 >= je) {
      if (hooks && hooks->column_flush) {
        if (k > jb) hooks->column_flush(k - 1);
        hooks->column_flush(k);
      }
      break;
    }
    // While the rest of the trailing matrix is updated on the side stream, the next
    // block column is factored on the panel stream.  For a short block column that
    // is a chain of small kernels with little work each: the bulk update then runs
    // in rounds that leave them room, and starts once the next column's own update
    // (which wants the whole device) is through.
    const int leave_free = lookahead && k + 2 < je ? L.leave_free_for(mk - wk) : -1;
    hipEvent_t ev_panel = nullptr;
    if (lookahead && k + 2 < je && leave_free < 0) {
      ev_panel = events.get();
      L.fail->check(hipEventRecord(ev_panel, s0));
    }
    // next column first (on the panel stream), so its factorisation can start early
    if (lookahead && ev_bulk_prev) L.fail->check(hipStreamWaitEvent(s0, ev_bulk_prev, 0));
    {
      const int64_t j = k + 1;
      touch(s0, j);
      const T* B = cols[k].base + (j - k) * bs * cols[k].ld;
      const FusedLeaf<T> fl = L.fused_leaf(pl.col_width(j), j * bs);
      rc = L.update(s0, cols[j].base, cols[j].ld, left(j), lda_k, B, cols[k].ld, L.dvec + k * bs,
                    n - j * bs, pl.col_width(j), wk, true, true, &fl, -1, Wk != nullptr);
      if (rc != MDET_OK) return rc;
    }
    if (lookahead && k + 2 < je && leave_free >= 0) {
      ev_panel = events.get();
      L.fail->check(hipEventRecord(ev_panel, s0));
    }
    if (k + 2 < je) {
      if (lookahead) L.fail->check(hipStreamWaitEvent(s1, ev_panel, 0));
      // One launch for all remaining columns, or one per block column: where a block
      // column alone fills the device many times over (here: 16 times), its launch
      // re-uses one set of B rows throughout and the ends of the launches cost little
      // (n = 131072, b = 4096: 11.18 -> 10.92 s); smaller ones lose more at their ends
      // than they gain (n = 32768, b = 2048: 190.8 -> 196.0 ms).
      const int64_t col_blocks = ((n - (k + 2) * bs + 127) / 128) * ((bs + 127) / 128);
      const bool one_launch = dense && (L.slots <= 0 || col_blocks < 16 * (int64_t)L.slots);
      if (one_launch) {
        const int64_t j = k + 2;
        const T* B = cols[k].base + (j - k) * bs * cols[k].ld;
        // all remaining resident columns in one launch (they are contiguous in memory)
        int64_t ncols = (je < pl.T ? je * bs : n) - j * bs;
        rc = L.update(s1, cols[j].base, cols[j].ld, left(j), lda_k, B, cols[k].ld, L.dvec + k * bs,
                      n - j * bs, ncols, wk, true, true, nullptr, leave_free, Wk != nullptr);
        if (rc != MDET_OK) return rc;
      } else {
        for (int64_t j = k + 2; j < je; ++j) {
          touch(s1, j);
          const T* B = cols[k].base + (j - k) * bs * cols[k].ld;
          rc = L.update(s1, cols[j].base, cols[j].ld, left(j), lda_k, B, cols[k].ld,
                        L.dvec + k * bs, n - j * bs, pl.col_width(j), wk, true, true, nullptr,
                        leave_free, Wk != nullptr);
          if (rc != MDET_OK) return rc;
        }
      }
      if (lookahead) {
        ev_bulk_prev = events.get();
        L.fail->check(hipEventRecord(ev_bulk_prev, s1));
      }
    }
    if (hooks && hooks->column_flush && k > jb) hooks->column_flush(k - 1);
  }
  // join the side stream back into the main one
  if (lookahead && ev_bulk_prev) L.fail->check(hipStreamWaitEvent(s0, ev_bulk_prev, 0));
  return MDET_OK;
}

// ---------------------------------------------------------------------------
// result collection
// ---------------------------------------------------------------------------
struct DeviceOut {
  double out[3];
  DevFlags flags;
};

static int finish_result(const DeviceOut& o, mdet_result* r) {
  r->negative_pivots = (int64_t)o.out[2];
  if (o.flags.first_bad != ~0ull) {
    r->bad_pivot_index = (int64_t)o.flags.first_bad;
    if (o.flags.bad_kind == 1) {
      r->sign = 0;
      r->logabsdet = -HUGE_VAL;
      return MDET_ESINGULAR;
    }
    if (o.flags.bad_kind == 4) {
      r->sign = 0;
      r->logabsdet = std::nan("");
      return MDET_ENOTPOSDEF;
    }
    r->sign = 0;
    r->logabsdet = std::nan("");
    return MDET_ENONFINITE;
  }
  r->bad_pivot_index = -1;
  r->logabsdet = o.out[0];
  r->sign = (int)o.out[1];
  if (!std::isfinite(r->logabsdet)) return MDET_ENONFINITE;
  return MDET_OK;
}

static void init_result(mdet_result* r, const Plan& pl) {
  std::memset(r, 0, sizeof(*r));
  r->bad_pivot_index = -1;
  r->sign = 1;
  r->block_size_used = pl.bs;
  r->num_blocks = pl.T;
  r->out_of_core = pl.out_of_core;
  r->num_superpanels = (int32_t)pl.panels.size();
}

// Workspace: either the caller's buffer or a library allocation.
struct Workspace {
  char* base = nullptr;
  uint64_t bytes = 0;
  bool owned = false;
  int acquire(const mdet_params& p, uint64_t need, HipFail& f) {
    if (p.dev_workspace) {
      if (p.dev_workspace_bytes < need || ((uintptr_t)p.dev_workspace & 255u)) return MDET_ENOMEM_DEVICE;
      base = (char*)p.dev_workspace;
      bytes = p.dev_workspace_bytes;
      return MDET_OK;
    }
    void* q = nullptr;
    hipError_t e = hipMalloc(&q, need ? need : 256);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      f.code = e;
      return MDET_ENOMEM_DEVICE;
    }
    base = (char*)q;
    bytes = need;
    owned = true;
    return MDET_OK;
  }
  ~Workspace() { if (owned && base) (void)hipFree(base); }
};

// The plan's workspace; if it cannot be had and the plan holds the pivot-scaled copies
// without having been asked for them, once more without them.
static int acquire_workspace(Workspace& ws, const mdet_params& p, Plan& pl, HipFail& fail) {
  int rc = ws.acquire(p, pl.dev_bytes, fail);
  if (rc == MDET_ENOMEM_DEVICE && pl.wcopy_optional && pl.wcopy_bytes) {
    pl.dev_bytes -= pl.wcopy_bytes;
    pl.wcopy_bytes = 0;
    fail.code = hipSuccess;
    rc = ws.acquire(p, pl.dev_bytes, fail);
  }
  return rc;
}

template <typename T>
static void bind_small(Launcher<T>& L, char* base, const SmallArea& sa) {
  L.dvec = (T*)(base + sa.dvec);
  L.dinv = (T*)(base + sa.dinv);
  L.linv = (T*)(base + sa.linv);
  L.l10 = (T*)(base + sa.l10);
  L.linv_u = L.linv + LEAF * SUB;      // linv is two arrays here
  L.flags = (DevFlags*)(base + sa.flags);
  L.perm = sa.total > sa.perm ? (int*)(base + sa.perm) : nullptr;
  // two workgroups of the trailing update fit one compute unit (registers and LDS)
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
    L.slots = 2 * cus;
}

// first_bad = ~0 (none), no odd leaves.  A kernel, not a memset: a caller may record the
// launches of the allocation-free entry point into a graph.
__global__ void reset_flags_kernel(DevFlags* f) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    f->first_bad = ~0ull;
    f->bad_kind = ~0ull;
    f->odd_leaves = 0ull;
  }
}

// The workspace of MDET_FLAG_PIVOT_BLOCK, which follows the small area.
template <typename T>
static void bind_pivot_block(Launcher<T>& L, char* base, const Plan& pl) {
  if (!pl.pivot_block) return;
  const PivotBlockArea a = pivot_block_area(pl.n, pl.bs, pl.beta);
  L.pb.S = (T*)(base + a.S);
  L.pb.Lfull = (T*)(base + a.Lfull);
  L.pb.Y = (T*)(base + a.Y);
  L.pb.Bg = (T*)(base + a.Bg);
  L.pb.leaf = (T*)(base + a.leaf);
  L.pb.linv = (T*)(base + a.linv);
  L.pb.dg = (T*)(base + a.dg);
  L.pb.active = (int*)(base + a.active);
  L.pb.piv = (int*)(base + a.piv);
  L.pb.part = (PbCand*)(base + a.part);
  L.pb.ldl = a.ldl;
  L.pb.max_w = pl.bs;
  L.pb.max_below = pl.n > pl.bs ? pl.n - pl.bs : 0;
}

template <typename T>
static void reset_flags(Launcher<T>& L, hipStream_t st) {
  hipLaunchKernelGGL(reset_flags_kernel, dim3(1), dim3(64), 0, st, L.flags);
  L.fail->check(hipGetLastError());
}

// ---------------------------------------------------------------------------
// mdet_logdet_device
// ---------------------------------------------------------------------------
template <typename T>
static int logdet_device_t(const mdet_params& p, const Plan& plan, T* dA, int64_t ld, mdet_result* res,
                           T* diag, const void* widen_from = nullptr) {
  HipFail fail;
  int dev = 0;
  MDET_HIP(fail, hipGetDevice(&dev));
  StreamSet* ss = nullptr;
  MDET_HIP(fail, get_streams(dev, &ss, false));
  if (!fail.ok()) { res->hip_error = fail.code; return MDET_EHIP; }

  Plan pl = plan;
  Workspace ws;
  int rc = acquire_workspace(ws, p, pl, fail);
  if (rc != MDET_OK) { res->hip_error = fail.code; return rc; }
  res->dev_bytes_high_water = pl.dev_bytes;

  const SmallArea sa = small_area(pl.n, pl.T, pl.beta, pl.pivot);
  Launcher<T> L;
  L.fail = &fail;
  L.profile = (p.flags & MDET_FLAG_PROFILE) != 0;
  L.spd = (p.flags & MDET_FLAG_ASSUME_SPD) != 0;
  bind_small(L, ws.base, sa);
  bind_pivot_block(L, ws.base + sa.total, pl);
  const uint64_t fixed = sa.total + pl.pb_bytes;       // what follows starts here
  double* partial = (double*)(ws.base + sa.partial);
  double* out = (double*)(ws.base + sa.out);
  double* running = (double*)(ws.base + sa.running);

  EventPool events(&fail);
  hipStream_t user = (hipStream_t)p.stream;
  hipStream_t s0 = ss->main, s1 = ss->side;
  // order our work after whatever the caller queued on its stream
  hipEvent_t ev_in = events.get();
  MDET_HIP(fail, hipEventRecord(ev_in, user));
  MDET_HIP(fail, hipStreamWaitEvent(s0, ev_in, 0));

  T* W = dA;
  int64_t ldw = ld;
  if (pl.need_copy && pl.n > 0) {
    constexpr int vec = 16 / (int)sizeof(T);
    ldw = round_up(pl.n, vec);
    W = (T*)(ws.base + fixed);
    if (widen_from) {
      const dim3 grid((unsigned)pl.n), block(256);
      if (p.dtype == MDET_F16)
        hipLaunchKernelGGL((widen_lower_kernel<StoredF16>), grid, block, 0, s0,
                           (const StoredF16*)widen_from, ld, (double*)W, ldw, pl.n);
      else if (p.dtype == MDET_BF16)
        hipLaunchKernelGGL((widen_lower_kernel<StoredBF16>), grid, block, 0, s0,
                           (const StoredBF16*)widen_from, ld, (double*)W, ldw, pl.n);
      else
        hipLaunchKernelGGL((widen_lower_kernel<float>), grid, block, 0, s0, (const float*)widen_from,
                           ld, (double*)W, ldw, pl.n);
      MDET_HIP(fail, hipGetLastError());
    } else {
      MDET_HIP(fail, hipMemcpy2DAsync(W, ldw * sizeof(T), dA, ld * sizeof(T), pl.n * sizeof(T), pl.n,
                                      hipMemcpyDeviceToDevice, s0));
    }
  }
  reset_flags(L, s0);
  L.profile_begin(s0);
  T* Q = nullptr;
  const int nb64 = (int)((pl.n + LEAF - 1) / LEAF);
  if (pl.general && pl.n > 0) {
    // the entries above the diagonal go, transposed, into an array of their own
    Q = (T*)(ws.base + fixed + pl.copy_bytes + pl.wcopy_bytes);
    L.qoff = Q - W;
    if (L.qoff == 0 || !L.perm) return MDET_EINVAL;
    hipLaunchKernelGGL((transpose_strict_kernel<T>), dim3((unsigned)((int64_t)nb64 * (nb64 + 1) / 2)),
                       dim3(256), 0, s0, (const T*)W, Q, ldw, pl.n, nb64, 0);
    MDET_HIP(fail, hipGetLastError());
  }
  if (pl.wcopy_bytes) {
    char* wb = ws.base + fixed + pl.copy_bytes;
    L.wbuf[0] = (T*)wb;
    L.wbuf[1] = (T*)(wb + pl.wcopy_bytes / 2);
    L.wld = pl.bs;
  }

  std::vector<ColRef<T>> cols((size_t)pl.T);
  for (int64_t j = 0; j < pl.T; ++j) cols[j] = {W + j * pl.bs * ldw + j * pl.bs, ldw};
  const bool lookahead = !(p.flags & MDET_FLAG_NO_LOOKAHEAD);
  rc = factor_resident(L, pl, cols, 0, pl.T, true, lookahead, s0, s1, events);
  if (rc == MDET_OK) {
    L.reduce(s0, pl.n, pl.bs, pl.T, partial, out, running);
    if (Q && !pl.need_copy) {
      // the caller's array is the output: U back above the diagonal
      hipLaunchKernelGGL((transpose_strict_kernel<T>), dim3((unsigned)((int64_t)nb64 * (nb64 + 1) / 2)),
                         dim3(256), 0, s0, (const T*)Q, W, ldw, pl.n, nb64, 1);
      MDET_HIP(fail, hipGetLastError());
    }
    if (diag && pl.n > 0)
      MDET_HIP(fail, hipMemcpyAsync(diag, L.dvec, pl.n * sizeof(T), hipMemcpyDeviceToDevice, s0));
    if (L.perm && p.perm && pl.n > 0)
      MDET_HIP(fail, hipMemcpyAsync(p.perm, L.perm, pl.n * sizeof(int), hipMemcpyDeviceToDevice, s0));
  }
  DeviceOut o;
  std::memset(&o, 0, sizeof(o));
  if (rc == MDET_OK) {
    MDET_HIP(fail, hipMemcpyAsync(o.out, out, sizeof(o.out), hipMemcpyDeviceToHost, s0));
    MDET_HIP(fail, hipMemcpyAsync(&o.flags, L.flags, sizeof(DevFlags), hipMemcpyDeviceToHost, s0));
  }
  MDET_HIP(fail, hipStreamSynchronize(s1));
  MDET_HIP(fail, hipStreamSynchronize(s0));
  res->flops = 2.0 * L.fma;
  res->kernel_launches = L.launches;
  L.collect_profile(res);
  if (!fail.ok()) { res->hip_error = fail.code; return MDET_EHIP; }
  if (rc != MDET_OK) return rc;
  rc = finish_result(o, res);
  // the permutation's sign: one factor of -1 for every leaf with an odd row order
  if (pl.general && (o.flags.odd_leaves & 1ull)) res->sign = -res->sign;
  return rc;
}


// ---------------------------------------------------------------------------
// mdet_logdet_device_noalloc: the same path for callers that cannot allocate
// ---------------------------------------------------------------------------
// The workspace of mdet_logdet_device (pivots, reciprocals, inverses of the leaves' diagonal
// sub-blocks, flags, partial sums, permutation) lives in a fixed array in device memory that
// belongs to the library; each GPU holds its own copy of it until the process ends.
constexpr uint64_t NOALLOC_SCRATCH_BYTES = MDET_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
// In host code the array's name is only a handle: its address on a device is asked for once,
// with that device current, and kept.
static char* g_scratch_ptr[64];

static hipError_t scratch_address(int dev, char** out) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = (char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// out[0] = log|det|, out[1] = sign, out[2] = negative pivots, out[3] = index of the first zero
// or non-finite pivot (-1: none), out[4] = the status the synchronous entry point would return
__global__ void noalloc_finish_kernel(const double* __restrict__ red, const DevFlags* __restrict__ flags,
                                      double* __restrict__ out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double logabs = red[0], sign = red[1];
  int status = MDET_OK;
  double bad = -1.0;
  if (flags->first_bad != ~0ull) {
    bad = (double)flags->first_bad;
    sign = 0.0;
    if (flags->bad_kind == 1ull) { logabs = -HUGE_VAL; status = MDET_ESINGULAR; }
    else if (flags->bad_kind == 4ull) { logabs = __builtin_nan(""); status = MDET_ENOTPOSDEF; }
    else { logabs = __builtin_nan(""); status = MDET_ENONFINITE; }
  } else if (!(logabs - logabs == 0.0)) {
    status = MDET_ENONFINITE;
  }
  out[0] = logabs;
  out[1] = sign;
  out[2] = red[2];
  out[3] = bad;
  out[4] = (double)status;
}

template <typename T>
static int logdet_device_noalloc_t(const mdet_params& p, const Plan& pl, char* base, T* dA, int64_t ld,
                                   double* out_dev, T* diag) {
  HipFail fail;
  const SmallArea sa = small_area(pl.n, pl.T, pl.beta, pl.pivot);
  Launcher<T> L;
  L.fail = &fail;
  L.spd = (p.flags & MDET_FLAG_ASSUME_SPD) != 0;
  bind_small(L, base, sa);
  double* partial = (double*)(base + sa.partial);
  double* red = (double*)(base + sa.out);
  double* running = (double*)(base + sa.running);
  hipStream_t st = (hipStream_t)p.stream;
  // everything on the caller's stream, in order: no second stream, no events
  EventPool events(&fail);       // never asked for an event without look-ahead
  reset_flags(L, st);
  std::vector<ColRef<T>> cols((size_t)pl.T);
  for (int64_t j = 0; j < pl.T; ++j) cols[j] = {dA + j * pl.bs * ld + j * pl.bs, ld};
  int rc = factor_resident(L, pl, cols, 0, pl.T, true, false, st, st, events);
  if (rc != MDET_OK) return rc;
  L.reduce(st, pl.n, pl.bs, pl.T, partial, red, running);
  hipLaunchKernelGGL(noalloc_finish_kernel, dim3(1), dim3(64), 0, st, (const double*)red,
                     (const DevFlags*)L.flags, out_dev);
  MDET_HIP(fail, hipGetLastError());
  if (diag && pl.n > 0)
    MDET_HIP(fail, hipMemcpyAsync(diag, L.dvec, pl.n * sizeof(T), hipMemcpyDeviceToDevice, st));
  if (L.perm && p.perm && pl.n > 0)
    MDET_HIP(fail, hipMemcpyAsync(p.perm, L.perm, pl.n * sizeof(int), hipMemcpyDeviceToDevice, st));
  return fail.ok() ? MDET_OK : MDET_EHIP;
}

// ---------------------------------------------------------------------------
// mdet_logdet_host: packed lower block-column layout in host memory
// ---------------------------------------------------------------------------
// Copy of rows [r0, r1) of block column j between the host layout (leading
// dimension w_j) and its device image (leading dimension col_ld(j)).
// With MDET_FLAG_PROFILE: every host <-> device copy of the host path bracketed by
// events on its stream; copies of one direction share a stream, so the sum of their
// durations is the time the link was busy in that direction.
struct CopyProfile {
  bool on = false;
  HipFail* fail = nullptr;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev[2];   // [0] host -> device, [1] device -> host
  struct Scope {
    CopyProfile* p; int dir; hipStream_t st; hipEvent_t e0 = nullptr, e1 = nullptr;
    Scope(CopyProfile* p_, int dir_, hipStream_t st_) : p(p_), dir(dir_), st(st_) {
      if (!p->on) return;
      e0 = timing_event_get(p->fail);
      e1 = timing_event_get(p->fail);
      p->fail->check(hipEventRecord(e0, st));
    }
    ~Scope() {
      if (!p->on) return;
      p->fail->check(hipEventRecord(e1, st));
      p->ev[dir].emplace_back(e0, e1);
    }
  };
  double collect(int dir) {   // seconds; call when the streams are idle
    double ms_total = 0.0;
    for (auto& pr : ev[dir]) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) ms_total += ms;
      timing_event_put(pr.first);
      timing_event_put(pr.second);
    }
    ev[dir].clear();
    return ms_total * 1e-3;
  }
};

// ---------------------------------------------------------------------------
// pageable host memory
// ---------------------------------------------------------------------------
// A copy between device memory and host memory that is not pinned is staged by the
// runtime on the calling thread, one memcpy at a time (measured 28 GB/s towards the
// device and 17 GB/s back, against 57 each way for pinned memory).  The host entry
// points move such memory themselves: through a few pinned chunks, each filled or
// emptied by several threads at once, one chunk's transfer under way while the next is
// copied.  The calling thread is held for the length of the copy either way.

// A few threads that split one transfer between them (and the caller): a memcpy, or a
// read or write of a file at a given offset (pread and pwrite take their own offsets, so
// the parts do not disturb each other).  A short read or a failed call sets `failed`.
class CopyThreads {
 public:
  explicit CopyThreads(int n) {
    for (int i = 0; i < n; ++i) workers_.emplace_back([this] { loop(); });
  }
  ~CopyThreads() {
    {
      std::lock_guard<std::mutex> lk(m_);
      stop_ = true;
    }
    cv_.notify_all();
    for (auto& t : workers_) t.join();
  }
  void copy(void* dst, const void* src, size_t bytes) { run_job(0, (char*)dst, (const char*)src, -1, 0, bytes); }
  void read_file(void* dst, int fd, uint64_t off, size_t bytes) { run_job(1, (char*)dst, nullptr, fd, off, bytes); }
  void write_file(int fd, uint64_t off, const void* src, size_t bytes) {
    run_job(2, nullptr, (const char*)src, fd, off, bytes);
  }
  std::atomic<bool> failed{false};

 private:
  static constexpr size_t PART = 4u << 20;
  struct Job {
    int op;                 // 0 memcpy, 1 file -> memory, 2 memory -> file
    char* dst;
    const char* src;
    int fd;
    uint64_t off;
    size_t bytes, parts;
    std::atomic<size_t> next{0}, done{0};
  };
  void run_job(int op, char* dst, const char* src, int fd, uint64_t off, size_t bytes) {
    if (bytes == 0) return;
    auto job = std::make_shared<Job>();
    job->op = op; job->dst = dst; job->src = src; job->fd = fd; job->off = off;
    job->bytes = bytes;
    job->parts = (bytes + PART - 1) / PART;
    if (job->parts < 2 || workers_.empty()) { run(*job); return; }
    {
      std::lock_guard<std::mutex> lk(m_);
      job_ = job;
      ++generation_;
    }
    cv_.notify_all();
    run(*job);
    std::unique_lock<std::mutex> lk(m_);
    done_cv_.wait(lk, [&] { return job->done.load() == job->parts; });
    job_.reset();
  }
  void one_part(const Job& j, size_t off, size_t len) {
    if (j.op == 0) { std::memcpy(j.dst + off, j.src + off, len); return; }
    size_t got = 0;
    while (got < len) {
      const ssize_t r = j.op == 1 ? ::pread(j.fd, j.dst + off + got, len - got, (off_t)(j.off + off + got))
                                  : ::pwrite(j.fd, j.src + off + got, len - got, (off_t)(j.off + off + got));
      if (r <= 0) { failed = true; return; }       // error, or the file ends early
      got += (size_t)r;
    }
  }
  void run(Job& j) {
    for (;;) {
      const size_t p = j.next.fetch_add(1);
      if (p >= j.parts) return;
      const size_t off = p * PART, len = j.bytes - off < PART ? j.bytes - off : PART;
      one_part(j, off, len);
      if (j.done.fetch_add(1) + 1 == j.parts) {
        std::lock_guard<std::mutex> lk(m_);
        done_cv_.notify_all();
      }
    }
  }
  void loop() {
    unsigned seen = 0;
    for (;;) {
      std::shared_ptr<Job> job;
      {
        std::unique_lock<std::mutex> lk(m_);
        cv_.wait(lk, [&] { return stop_ || generation_ != seen; });
        if (stop_) return;
        seen = generation_;
        job = job_;
      }
      if (job) run(*job);
    }
  }
  std::vector<std::thread> workers_;
  std::mutex m_;
  std::condition_variable cv_, done_cv_;
  std::shared_ptr<Job> job_;
  unsigned generation_ = 0;
  bool stop_ = false;
};

// Pinned chunks between the device and either pageable host memory or a file.  One per
// store and call; the chunks are allocated when the first copy needs them.  With a file
// (fd >= 0) the host "pointers" handed to it are byte offsets into that file, and every
// copy goes through the chunks; with memory, small copies are left to the runtime.
class HostStager {
 public:
  static constexpr size_t CHUNK = 32u << 20;
  static constexpr int NCHUNK = 4;
  static constexpr size_t DIRECT_BELOW = 1u << 20;
  HostStager(HipFail* f, int fd) : fail_(f), fd_(fd) {}
  ~HostStager() {
    for (int c = 0; c < NCHUNK; ++c) {
      if (ev_[c]) { (void)hipEventSynchronize(ev_[c]); (void)hipEventDestroy(ev_[c]); }
      if (buf_[c]) (void)hipHostFree(buf_[c]);
    }
  }
  bool is_file() const { return fd_ >= 0; }
  // a read or write of the file failed or came up short, or the chunks could not be had
  bool io_failed() const { return broken_ || (threads_ && threads_->failed.load()); }
  // true if p is ordinary (pageable) host memory
  static bool pageable(const void* p) {
    hipPointerAttribute_t a;
    if (hipPointerGetAttributes(&a, p) != hipSuccess) { (void)hipGetLastError(); return true; }
    return a.type == hipMemoryTypeUnregistered;
  }
  // rows x row_bytes, packed on the host side, pitch_bytes apart on the device
  void to_device(void* dst, size_t pitch_bytes, const void* src, size_t row_bytes, size_t rows,
                 hipStream_t st) {
    const bool flat = pitch_bytes == row_bytes;
    const size_t bytes = row_bytes * rows;
    if (bytes == 0) return;
    if (!is_file() && (bytes < DIRECT_BELOW || !ready())) {
      fail_->check(flat ? hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st)
                        : hipMemcpy2DAsync(dst, pitch_bytes, src, row_bytes, row_bytes, rows,
                                           hipMemcpyHostToDevice, st));
      return;
    }
    if (!ready()) { broken_ = true; return; }
    const size_t rows_per = flat ? rows : (CHUNK / row_bytes ? CHUNK / row_bytes : 1);
    const size_t step = flat ? CHUNK : rows_per * row_bytes;
    if (step > CHUNK) { broken_ = true; return; }
    for (size_t off = 0; off < bytes; off += step) {
      const size_t len = bytes - off < step ? bytes - off : step;
      const int c = take();
      if (is_file()) threads_->read_file(buf_[c], fd_, (uint64_t)(uintptr_t)src + off, len);
      else threads_->copy(buf_[c], (const char*)src + off, len);
      if (flat)
        fail_->check(hipMemcpyAsync((char*)dst + off, buf_[c], len, hipMemcpyHostToDevice, st));
      else
        fail_->check(hipMemcpy2DAsync((char*)dst + (off / row_bytes) * pitch_bytes, pitch_bytes, buf_[c],
                                      row_bytes, row_bytes, len / row_bytes, hipMemcpyHostToDevice, st));
      fail_->check(hipEventRecord(ev_[c], st));
      busy_[c] = true;
    }
  }
  void to_host(void* dst, const void* src, size_t pitch_bytes, size_t row_bytes, size_t rows,
               hipStream_t st) {
    const bool flat = pitch_bytes == row_bytes;
    const size_t bytes = row_bytes * rows;
    if (bytes == 0) return;
    if (!is_file() && (bytes < DIRECT_BELOW || !ready())) {
      fail_->check(flat ? hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, st)
                        : hipMemcpy2DAsync(dst, row_bytes, src, pitch_bytes, row_bytes, rows,
                                           hipMemcpyDeviceToHost, st));
      return;
    }
    if (!ready()) { broken_ = true; return; }
    const size_t rows_per = flat ? rows : (CHUNK / row_bytes ? CHUNK / row_bytes : 1);
    const size_t step = flat ? CHUNK : rows_per * row_bytes;
    if (step > CHUNK) { broken_ = true; return; }
    int prev = -1;
    size_t prev_off = 0, prev_len = 0;
    auto drain = [&] {
      if (prev < 0) return;
      fail_->check(hipEventSynchronize(ev_[prev]));
      if (is_file()) threads_->write_file(fd_, (uint64_t)(uintptr_t)dst + prev_off, buf_[prev], prev_len);
      else threads_->copy((char*)dst + prev_off, buf_[prev], prev_len);
      busy_[prev] = false;
      prev = -1;
    };
    for (size_t off = 0; off < bytes; off += step) {
      const size_t len = bytes - off < step ? bytes - off : step;
      const int c = take(prev);
      if (flat)
        fail_->check(hipMemcpyAsync(buf_[c], (const char*)src + off, len, hipMemcpyDeviceToHost, st));
      else
        fail_->check(hipMemcpy2DAsync(buf_[c], row_bytes, (const char*)src + (off / row_bytes) * pitch_bytes,
                                      pitch_bytes, row_bytes, len / row_bytes, hipMemcpyDeviceToHost, st));
      fail_->check(hipEventRecord(ev_[c], st));
      busy_[c] = true;
      drain();                 // the chunk before this one, while this one is on its way
      prev = c;
      prev_off = off;
      prev_len = len;
    }
    drain();
  }

 private:
  bool ready() {
    if (state_ != 0) return state_ > 0;
    state_ = -1;
    for (int c = 0; c < NCHUNK; ++c) {
      if (hipHostMalloc(&buf_[c], CHUNK, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); buf_[c] = nullptr; return false; }
      if (hipEventCreateWithFlags(&ev_[c], hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); ev_[c] = nullptr; return false; }
    }
    unsigned hw = std::thread::hardware_concurrency();
    int n = hw >= 16 ? 7 : (hw >= 8 ? 3 : 1);
    threads_.reset(new CopyThreads(n));
    state_ = 1;
    return true;
  }
  // the next chunk in turn (not `keep`), once whatever last used it is through
  int take(int keep = -1) {
    int c = next_;
    if (c == keep) c = (c + 1) % NCHUNK;
    next_ = (c + 1) % NCHUNK;
    if (busy_[c]) { fail_->check(hipEventSynchronize(ev_[c])); busy_[c] = false; }
    return c;
  }
  HipFail* fail_;
  int fd_;
  bool broken_ = false;
  void* buf_[NCHUNK] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t ev_[NCHUNK] = {nullptr, nullptr, nullptr, nullptr};
  bool busy_[NCHUNK] = {false, false, false, false};
  int next_ = 0;
  int state_ = 0;   // 0 not tried, 1 ready, -1 unavailable
  std::unique_ptr<CopyThreads> threads_;
};

template <typename T>
static void copy_col_rows(HipFail& fail, const Plan& pl, int64_t j, int64_t r0, int64_t r1, T* dev_col,
                          T* host_col, bool to_device, hipStream_t st, uint64_t* bytes,
                          CopyProfile* prof, HostStager* stager = nullptr) {
  if (r1 <= r0) return;
  CopyProfile::Scope timed(prof, to_device ? 0 : 1, st);
  const int64_t w = pl.col_width(j), ldd = pl.col_ld(j);
  T* d = dev_col + (r0 - j * pl.bs) * ldd;
  T* h = host_col + (r0 - j * pl.bs) * w;
  const size_t nbytes = (size_t)(r1 - r0) * w * sizeof(T);
  if (stager) {
    if (to_device) stager->to_device(d, ldd * sizeof(T), h, w * sizeof(T), (size_t)(r1 - r0), st);
    else stager->to_host(h, d, ldd * sizeof(T), w * sizeof(T), (size_t)(r1 - r0), st);
  } else if (ldd == w) {
    fail.check(to_device ? hipMemcpyAsync(d, h, nbytes, hipMemcpyHostToDevice, st)
                         : hipMemcpyAsync(h, d, nbytes, hipMemcpyDeviceToHost, st));
  } else {
    fail.check(to_device ? hipMemcpy2DAsync(d, ldd * sizeof(T), h, w * sizeof(T), w * sizeof(T),
                                            (size_t)(r1 - r0), hipMemcpyHostToDevice, st)
                         : hipMemcpy2DAsync(h, w * sizeof(T), d, ldd * sizeof(T), w * sizeof(T),
                                            (size_t)(r1 - r0), hipMemcpyDeviceToHost, st));
  }
  *bytes += nbytes;
}

// Pinned host buffer owned by the library.
struct PinnedBuf {
  void* p = nullptr;
  int alloc(size_t bytes) {
    hipError_t e = hipHostMalloc(&p, bytes ? bytes : 1, hipHostMallocDefault);
    if (e != hipSuccess) { (void)hipGetLastError(); p = nullptr; return MDET_ENOMEM_HOST; }
    return MDET_OK;
  }
  ~PinnedBuf() { if (p) (void)hipHostFree(p); }
};

// Where the original blocks come from when it is not host memory or a file in the
// arithmetic's own type laid out like the factors.
struct HostSource {
  // the matrix as stored, narrower than the arithmetic (MDET_FLAG_COMPUTE_F64): base address
  // (or byte offset in the file) of the packed layout in elements of `dtype`
  const char* narrow = nullptr;
  int32_t dtype = MDET_F64;
  // blocks fetched through the caller's function instead (mdet_logdet_provider)
  mdet_block_provider provider = nullptr;
  // or produced in device memory by the caller's function (mdet_logdet_provider_device)
  mdet_block_provider_device provider_dev = nullptr;
  void* user = nullptr;
};

// fd_in / fd_out >= 0: the store is a file and hA / hOut the byte offset of the layout in it
// (as a pointer), see mdet_logdet_file.
template <typename T>
static int logdet_host_t(const mdet_params& p, const Plan& plan, T* hA, T* hOut, mdet_result* res,
                         T* diag_host, int fd_in = -1, int fd_out = -1, const HostSource* source = nullptr) {
  HipFail fail;
  int dev = 0;
  MDET_HIP(fail, hipGetDevice(&dev));
  StreamSet* ss = nullptr;
  MDET_HIP(fail, get_streams(dev, &ss, true));
  if (!fail.ok()) { res->hip_error = fail.code; return MDET_EHIP; }

  Plan pl = plan;
  Workspace ws;
  int rc = acquire_workspace(ws, p, pl, fail);
  if (rc != MDET_OK) { res->hip_error = fail.code; return rc; }
  res->dev_bytes_high_water = pl.dev_bytes;

  const SmallArea sa = small_area(pl.n, pl.T, pl.beta, pl.pivot);
  Launcher<T> L;
  L.fail = &fail;
  L.profile = (p.flags & MDET_FLAG_PROFILE) != 0;
  L.spd = (p.flags & MDET_FLAG_ASSUME_SPD) != 0;
  bind_small(L, ws.base, sa);
  double* partial = (double*)(ws.base + sa.partial);
  double* out = (double*)(ws.base + sa.out);
  double* running = (double*)(ws.base + sa.running);
  bind_pivot_block(L, ws.base + sa.total, pl);
  char* const stage = ws.base + sa.total + pl.pb_bytes;   // pl.stage_bytes of staging for narrow uploads
  char* arena = stage + pl.stage_bytes;
  uint64_t arena_used = 0;                           // highest arena offset any group reached
  // A general matrix (Sec. 2.2, Eq. 1: M = P L U) is two lower-triangular arrays, the entries
  // on and below the diagonal and the transposed entries above it: on the host two packed
  // layouts one after the other, on the device two arenas arena_half bytes apart with
  // everything (block columns, streamed blocks) at the same offsets in both.  Every copy below
  // is made once per array; every kernel works on both at once (see Launcher::qoff).
  const int arrays = pl.general ? 2 : 1;
  const int64_t host_half = (int64_t)(pl.layout_bytes / sizeof(T));     // elements between the two host layouts
  const int64_t dev_half = (int64_t)(pl.arena_half / sizeof(T));
  if (pl.general) {
    L.qoff = dev_half;
    if (L.qoff == 0 && pl.n > 0) return MDET_EINVAL;
  }

  EventPool events(&fail);
  hipStream_t s0 = ss->main, s1 = ss->side, sh = ss->h2d, sd = ss->d2h;
  hipEvent_t ev_in = events.get();
  MDET_HIP(fail, hipEventRecord(ev_in, (hipStream_t)p.stream));
  MDET_HIP(fail, hipStreamWaitEvent(s0, ev_in, 0));
  MDET_HIP(fail, hipStreamWaitEvent(sh, ev_in, 0));
  reset_flags(L, s0);
  L.profile_begin(s0);

  const bool lookahead = !(p.flags & MDET_FLAG_NO_LOOKAHEAD);
  const int64_t bs = pl.bs, n = pl.n, T_ = pl.T;
  std::vector<ColRef<T>> cols((size_t)T_, ColRef<T>{nullptr, 0});
  uint64_t h2d_bytes = 0, d2h_bytes = 0;
  CopyProfile cprof;
  cprof.on = L.profile;
  cprof.fail = &fail;
  auto host_col = [&](T* base, int64_t j) { return base + pl.col_offset(j); };
  // pageable host memory goes through pinned chunks (see HostStager)
  HostStager stager_in(&fail, fd_in), stager_out(&fail, fd_out);
  const bool from_provider = source && source->provider;
  const bool from_device = source && source->provider_dev;
  const bool narrow = source && !from_provider && !from_device && pl.widen;
  const void* const in_base = narrow ? (const void*)source->narrow : (const void*)hA;
  HostStager* stage_in = (!from_provider && !from_device && (fd_in >= 0 || (n > 0 && HostStager::pageable(in_base)))) ? &stager_in : nullptr;
  HostStager* stage_out = (fd_out >= 0 || (n > 0 && hOut && HostStager::pageable(hOut))) ? &stager_out : nullptr;
  // two pinned buffers of one block each for the provider's blocks, used in turn
  PinnedBuf prov_buf[2];
  hipEvent_t prov_ev[2] = {nullptr, nullptr};
  int prov_next = 0;
  int prov_rc = MDET_OK;
  if (from_provider && n > 0) {
    for (int q = 0; q < 2; ++q) {
      if (prov_buf[q].alloc((size_t)bs * bs * pl.src_beta) != MDET_OK) return MDET_ENOMEM_HOST;
      prov_ev[q] = events.get();
    }
  }
  // narrow elements of rows x cols at `src` (leading dimension lds, device memory) widened into dst
  auto widen_piece = [&](const void* src, int64_t lds, T* dst, int64_t ldd, int64_t rows, int64_t cols) {
    if constexpr (std::is_same<T, double>::value) {
      const int64_t total = rows * cols;
      const unsigned grid = (unsigned)std::min<int64_t>((total + 255) / 256, 8192);
      const int32_t sdt = source ? source->dtype : MDET_F64;
      if (sdt == MDET_F16)
        hipLaunchKernelGGL((widen_rows_kernel<StoredF16>), dim3(grid), dim3(256), 0, sh, (const StoredF16*)src, lds,
                           (double*)dst, ldd, rows, cols);
      else if (sdt == MDET_BF16)
        hipLaunchKernelGGL((widen_rows_kernel<StoredBF16>), dim3(grid), dim3(256), 0, sh, (const StoredBF16*)src,
                           lds, (double*)dst, ldd, rows, cols);
      else
        hipLaunchKernelGGL((widen_rows_kernel<float>), dim3(grid), dim3(256), 0, sh, (const float*)src, lds,
                           (double*)dst, ldd, rows, cols);
      MDET_HIP(fail, hipGetLastError());
      ++L.launches;
    }
  };
  // rows x cols elements at `src` (leading dimension lds, device memory) transposed into dst
  // (a general matrix is stored in the arithmetic's type)
  auto transpose_piece = [&](const void* src, int64_t lds, T* dst, int64_t ldd, int64_t rows, int64_t cols) {
    const dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
    hipLaunchKernelGGL((transpose_rows_kernel<T>), grid, dim3(256), 0, sh, (const T*)src, lds, dst, ldd, rows, cols);
    MDET_HIP(fail, hipGetLastError());
    ++L.launches;
  };
  // Rows [r0, r1) of the ORIGINAL block column j into its device image, on the upload stream.
  auto upload_orig = [&](int64_t j, int64_t r0, int64_t r1) {
    if (r1 <= r0) return;
    const int64_t w = pl.col_width(j), ldd = pl.col_ld(j);
    T* dcol = cols[j].base;
    if (from_device) {
      // the caller's function puts each block where it belongs, with work queued on the upload stream
      for (int64_t i = r0 / bs; i * bs < r1 && prov_rc == MDET_OK; ++i) {
        const int64_t b0 = i * bs, b1 = std::min<int64_t>(n, b0 + bs);
        if (source->provider_dev(source->user, i, j, b1 - b0, w, dcol + (b0 - j * bs) * ldd, ldd, (void*)sh) != 0)
          prov_rc = MDET_EPROVIDER;
      }
      return;
    }
    if (from_provider) {
      // block by block through the caller's function, each into a pinned buffer and on from there
      for (int64_t i = r0 / bs; i * bs < r1 && prov_rc == MDET_OK; ++i) {
        const int64_t b0 = i * bs, b1 = std::min<int64_t>(n, b0 + bs);
        int q = prov_next;
        prov_next ^= 1;
        MDET_HIP(fail, hipEventSynchronize(prov_ev[q]));     // its last transfer has left the buffer
        if (source->provider(source->user, i, j, b1 - b0, w, prov_buf[q].p, w) != 0) { prov_rc = MDET_EPROVIDER; break; }
        {
          CopyProfile::Scope timed(&cprof, 0, sh);
          T* dst = dcol + (b0 - j * bs) * ldd;
          const size_t row_bytes = (size_t)w * pl.src_beta;
          if (pl.widen) {
            // pieces of at most the staging buffer, widened from there (one stream: in order)
            const int64_t per = std::max<int64_t>(1, (int64_t)(pl.stage_bytes / row_bytes));
            for (int64_t r = b0; r < b1; r += per) {
              const int64_t rn = std::min<int64_t>(per, b1 - r);
              MDET_HIP(fail, hipMemcpyAsync(stage, (const char*)prov_buf[q].p + (size_t)(r - b0) * row_bytes,
                                            (size_t)rn * row_bytes, hipMemcpyHostToDevice, sh));
              widen_piece(stage, w, dcol + (r - j * bs) * ldd, ldd, rn, w);
            }
          } else if (ldd == w) {
            MDET_HIP(fail, hipMemcpyAsync(dst, prov_buf[q].p, (size_t)(b1 - b0) * row_bytes, hipMemcpyHostToDevice, sh));
          } else {
            MDET_HIP(fail, hipMemcpy2DAsync(dst, ldd * sizeof(T), prov_buf[q].p, row_bytes, row_bytes,
                                            (size_t)(b1 - b0), hipMemcpyHostToDevice, sh));
          }
          h2d_bytes += (uint64_t)(b1 - b0) * row_bytes;
        }
        if (arrays == 2) {
          // The same place of the transposed store holds block (j, i) of the matrix, transposed:
          // w x (b1 - b0) as the caller hands it over.  The diagonal block has just arrived.
          const int64_t srows = w, scols = b1 - b0;
          if (i != j) {
            MDET_HIP(fail, hipEventRecord(prov_ev[q], sh));
            q = prov_next;
            prov_next ^= 1;
            MDET_HIP(fail, hipEventSynchronize(prov_ev[q]));
            if (source->provider(source->user, j, i, srows, scols, prov_buf[q].p, scols) != 0) { prov_rc = MDET_EPROVIDER; break; }
          }
          CopyProfile::Scope timed(&cprof, 0, sh);
          const size_t row_bytes = (size_t)scols * pl.src_beta;
          const int64_t per = std::max<int64_t>(1, (int64_t)(pl.stage_bytes / row_bytes));
          T* dst = dcol + dev_half + (b0 - j * bs) * ldd;       // its row c, column r: entry (r, c) of the block
          for (int64_t r = 0; r < srows; r += per) {
            const int64_t rn = std::min<int64_t>(per, srows - r);
            MDET_HIP(fail, hipMemcpyAsync(stage, (const char*)prov_buf[q].p + (size_t)r * row_bytes,
                                          (size_t)rn * row_bytes, hipMemcpyHostToDevice, sh));
            transpose_piece(stage, scols, dst + r, ldd, rn, scols);
          }
          h2d_bytes += (uint64_t)srows * row_bytes;
        }
        MDET_HIP(fail, hipEventRecord(prov_ev[q], sh));
      }
      return;
    }
    if (!narrow) {
      for (int h = 0; h < arrays; ++h)
        copy_col_rows(fail, pl, j, r0, r1, dcol + h * dev_half, host_col(hA, j) + h * host_half, true, sh,
                      &h2d_bytes, &cprof, stage_in);
      return;
    }
    CopyProfile::Scope timed(&cprof, 0, sh);
    const size_t row_bytes = (size_t)w * pl.src_beta;
    const char* scol = source->narrow + (uint64_t)pl.col_offset(j) * pl.src_beta;
    const int64_t per = std::max<int64_t>(1, (int64_t)(pl.stage_bytes / row_bytes));
    for (int64_t r = r0; r < r1; r += per) {
      const int64_t rn = std::min<int64_t>(per, r1 - r);
      const char* src = scol + (size_t)(r - j * bs) * row_bytes;
      if (stage_in) stage_in->to_device(stage, (size_t)rn * row_bytes, src, (size_t)rn * row_bytes, 1, sh);
      else MDET_HIP(fail, hipMemcpyAsync(stage, src, (size_t)rn * row_bytes, hipMemcpyHostToDevice, sh));
      widen_piece(stage, w, dcol + (r - j * bs) * ldd, ldd, rn, w);
    }
    h2d_bytes += (uint64_t)(r1 - r0) * row_bytes;
  };

  if (!pl.out_of_core) {
    // ---- everything resident: upload column by column, factor as columns arrive
    uint64_t off = 0;
    for (int64_t j = 0; j < T_; ++j) {
      cols[j] = {(T*)(arena + off), pl.col_ld(j)};
      off += align256(pl.dev_col_bytes(j));
    }
    if (pl.wcopy_bytes) {
      L.wbuf[0] = (T*)(arena + off);
      L.wbuf[1] = (T*)(arena + off + pl.wcopy_bytes / 2);
      L.wld = pl.bs;
    }
    // A column is uploaded when the first kernel that touches it is about to be
    // queued: columns arrive in the order of need, and a copy that blocks the
    // calling thread (pageable memory) does so while the device works on the
    // columns before it.
    std::vector<hipEvent_t> ready((size_t)T_, nullptr);
    std::vector<char> seen0((size_t)T_, 0), seen1((size_t)T_, 0);
    ResidentHooks hooks;
    hooks.before_touch = [&](hipStream_t st, int64_t j) {
      if (!ready[j]) {
        upload_orig(j, j * bs, n);
        ready[j] = events.get();
        fail.check(hipEventRecord(ready[j], sh));
      }
      std::vector<char>& seen = (st == s0) ? seen0 : seen1;
      if (!seen[j]) { seen[j] = 1; fail.check(hipStreamWaitEvent(st, ready[j], 0)); }
    };
    arena_used = off + pl.wcopy_bytes;
    rc = factor_resident(L, pl, cols, 0, T_, false, lookahead, s0, s1, events, &hooks);
  } else {
    // ---- out-of-core: resident groups of block columns, factored columns stream past
    const uint64_t tile_al = align256(pl.tile_bytes);
    hipEvent_t ev_arena_free = nullptr;   // previous group: compute finished and columns saved
    std::vector<hipEvent_t> saved;        // write-back completion of the previous group
    // A factored column is saved in two steps: an event right behind its last kernel,
    // and, a step later, the copy that waits for it (see ResidentHooks::column_flush).
    std::vector<hipEvent_t> final_ev((size_t)T_, nullptr);
    auto mark_final = [&](int64_t k) {
      final_ev[k] = events.get();
      fail.check(hipEventRecord(final_ev[k], s0));
    };
    auto write_back = [&](int64_t k) {
      fail.check(hipStreamWaitEvent(sd, final_ev[k], 0));
      for (int h = 0; h < arrays; ++h)
        copy_col_rows(fail, pl, k, k * bs, n, cols[k].base + h * dev_half, host_col(hOut, k) + h * host_half, false,
                      sd, &d2h_bytes, &cprof, stage_out);
      hipEvent_t sv = events.get();
      fail.check(hipEventRecord(sv, sd));
      saved.push_back(sv);
    };
    for (size_t g = 0; g < pl.panels.size() && rc == MDET_OK; ++g) {
      const int64_t j0 = pl.panels[g].j0, j1 = pl.panels[g].j1;
      const int64_t wc = j1 - j0;
      // -- carve the arena
      uint64_t off = 0;
      for (int64_t j = j0; j < j1; ++j) {
        cols[j] = {(T*)(arena + off), pl.col_ld(j)};
        off += align256(pl.dev_col_bytes(j));
      }
      T* bpool[2] = {nullptr, nullptr};
      std::vector<T*> ring;
      if (j0 > 0) {
        for (int q = 0; q < 2; ++q) { bpool[q] = (T*)(arena + off); off += (uint64_t)wc * tile_al; }
        for (uint64_t q = 0; q < pl.ring_tiles; ++q) { ring.push_back((T*)(arena + off)); off += tile_al; }
      }
      if (off > arena_used) arena_used = off;
      // -- the arena may be reused once the previous group is saved and idle
      if (ev_arena_free) MDET_HIP(fail, hipStreamWaitEvent(sh, ev_arena_free, 0));
      for (hipEvent_t e : saved) MDET_HIP(fail, hipStreamWaitEvent(sh, e, 0));
      saved.clear();

      const int64_t rows_end_J = (j1 < T_) ? j1 * bs : n;   // first row below the group's own rows
      if (j0 == 0) {
        // first group: nothing to stream; upload column by column and factor as they arrive
        std::vector<hipEvent_t> ready((size_t)T_, nullptr);
        std::vector<char> seen0((size_t)T_, 0), seen1((size_t)T_, 0);
        ResidentHooks hooks;
        hooks.before_touch = [&](hipStream_t st, int64_t j) {
          if (!ready[j]) {   // uploaded when first needed, as in the in-core case
            upload_orig(j, j * bs, n);
            ready[j] = events.get();
            fail.check(hipEventRecord(ready[j], sh));
          }
          std::vector<char>& seen = (st == s0) ? seen0 : seen1;
          if (!seen[j]) { seen[j] = 1; fail.check(hipStreamWaitEvent(st, ready[j], 0)); }
        };
        hooks.column_final = mark_final;
        hooks.column_flush = write_back;
        if (j1 == T_) hooks.column_final = hooks.column_flush = nullptr;   // single group: nothing streams it again
        rc = factor_resident(L, pl, cols, j0, j1, false, lookahead, s0, s1, events, &hooks);
      } else {
        // The group's original blocks are uploaded one block row at a time, each just
        // ahead of the first streamed block that needs it (uploads share one stream, so
        // issue order is arrival order).
        std::vector<hipEvent_t> row_ready((size_t)T_, nullptr);
        auto upload_row = [&](int64_t i) {
          const int64_t r0 = i * bs, r1 = (i + 1) * bs < n ? (i + 1) * bs : n;
          for (int64_t j = j0; j < j1 && j <= i; ++j) upload_orig(j, r0, r1);
          row_ready[i] = events.get();
          MDET_HIP(fail, hipEventRecord(row_ready[i], sh));
        };
        std::vector<hipEvent_t> slot_ready(ring.size(), nullptr), slot_free(ring.size(), nullptr);
        hipEvent_t b_ready[2] = {nullptr, nullptr}, b_free[2] = {nullptr, nullptr};
        size_t slot_next = 0;
        // operands of column k for the group's own rows: rows [j0*bs, rows_end_J) of column k
        auto upload_operands = [&](int64_t k) {
          const int q = (int)(k & 1);
          T* hk = host_col(hOut, k);          // factored column k (bs wide, ld = bs)
          if (b_free[q]) MDET_HIP(fail, hipStreamWaitEvent(sh, b_free[q], 0));
          for (int h = 0; h < arrays; ++h) {
            const size_t nbytes = (size_t)(rows_end_J - j0 * bs) * bs * sizeof(T);
            CopyProfile::Scope timed(&cprof, 0, sh);
            T* dst = bpool[q] + h * dev_half;
            const T* src = hk + h * host_half + (j0 - k) * bs * bs;
            if (stage_out) stage_out->to_device(dst, nbytes, src, nbytes, 1, sh);
            else MDET_HIP(fail, hipMemcpyAsync(dst, src, nbytes, hipMemcpyHostToDevice, sh));
            h2d_bytes += nbytes;
          }
          if (!b_ready[q]) b_ready[q] = events.get();
          MDET_HIP(fail, hipEventRecord(b_ready[q], sh));
          MDET_HIP(fail, hipStreamWaitEvent(s0, b_ready[q], 0));
        };
        // the group's own rows: each target column j gets rows [j*bs, rows_end_J) in one launch
        auto update_group_rows = [&](int64_t k) {
          const int q = (int)(k & 1);
          for (int64_t j = j0; j < j1 && rc == MDET_OK; ++j) {
            const T* A = bpool[q] + (j - j0) * bs * bs;
            rc = L.update(s0, cols[j].base, cols[j].ld, A, bs, A, bs, L.dvec + k * bs, rows_end_J - j * bs,
                          pl.col_width(j), bs, true, true);
          }
        };
        // The same products one block row of the group at a time, for the sweep that brings the
        // originals: block row i can be worked on as soon as it has arrived, instead of the
        // whole group waiting for all of its rows (the last group consists of nothing else).
        auto update_own_row = [&](int64_t k, int64_t i) {
          const int q = (int)(k & 1);
          MDET_HIP(fail, hipStreamWaitEvent(s0, row_ready[i], 0));
          const T* A = bpool[q] + (i - j0) * bs * bs;
          for (int64_t j = j0; j <= i && rc == MDET_OK; ++j) {
            T* C = cols[j].base + (i - j) * bs * cols[j].ld;
            rc = L.update(s0, C, cols[j].ld, A, bs, bpool[q] + (j - j0) * bs * bs, bs, L.dvec + k * bs,
                          pl.col_width(i), pl.col_width(j), bs, i == j, true);
          }
        };
        // block row i below the group: the streamed block (i, k), used by every column of the group
        auto stream_block = [&](int64_t k, int64_t i) {
          const int q = (int)(k & 1);
          T* hk = host_col(hOut, k);
          const T* dk = L.dvec + k * bs;
          const size_t sl = slot_next++ % ring.size();
          const int64_t wi = pl.col_width(i);
          if (slot_free[sl]) MDET_HIP(fail, hipStreamWaitEvent(sh, slot_free[sl], 0));
          const size_t nbytes = (size_t)wi * bs * sizeof(T);
          for (int h = 0; h < arrays; ++h) {
            CopyProfile::Scope timed(&cprof, 0, sh);
            T* dst = ring[sl] + h * dev_half;
            const T* src = hk + h * host_half + (i - k) * bs * bs;
            if (stage_out) stage_out->to_device(dst, nbytes, src, nbytes, 1, sh);
            else MDET_HIP(fail, hipMemcpyAsync(dst, src, nbytes, hipMemcpyHostToDevice, sh));
            h2d_bytes += nbytes;
          }
          if (!slot_ready[sl]) slot_ready[sl] = events.get();
          MDET_HIP(fail, hipEventRecord(slot_ready[sl], sh));
          MDET_HIP(fail, hipStreamWaitEvent(s0, slot_ready[sl], 0));
          if (k == 0) MDET_HIP(fail, hipStreamWaitEvent(s0, row_ready[i], 0));
          // The streamed rows are the left operand of one update per column of the
          // group: scaled by the pivots once, in place (W = L D), they serve all of
          // them through the kernel that scales nothing.
          const bool prescaled = !L.spd && wc > 1 && !pl.general;
          if (prescaled) {
            const int64_t vecs = wi * (bs / (16 / (int64_t)sizeof(T)));
            const unsigned grid = (unsigned)std::min<int64_t>((vecs + 255) / 256, 4096);
            hipLaunchKernelGGL((scale_columns_kernel<T>), dim3(grid), dim3(256), 0, s0, ring[sl], bs, wi,
                               (int)bs, dk);
            MDET_HIP(fail, hipGetLastError());
            ++L.launches;
          }
          for (int64_t j = j0; j < j1 && rc == MDET_OK; ++j) {
            T* C = cols[j].base + (i - j) * bs * cols[j].ld;
            rc = L.update(s0, C, cols[j].ld, ring[sl], bs, bpool[q] + (j - j0) * bs * bs, bs, dk, wi,
                          pl.col_width(j), bs, false, true, nullptr, -1, prescaled);
          }
          if (!slot_free[sl]) slot_free[sl] = events.get();
          MDET_HIP(fail, hipEventRecord(slot_free[sl], s0));
        };
        // Factored columns 0 and 1 pass in one sweep, the rest one sweep each.  The first
        // sweep also brings in the group's original blocks, wc of them per block row beside
        // the one streamed block whose wc products pay for the transfer; with two streamed
        // blocks per row it is the products again, not the link, that set the pace.  Every
        // entry still receives its updates in the order k = 0, 1, 2, ...
        for (int64_t k = 0; k < j0 && rc == MDET_OK;) {
          const int64_t cnt = (k == 0 && j0 >= 2) ? 2 : 1;
          for (int64_t t = 0; t < cnt; ++t) upload_operands(k + t);
          if (k == 0) {
            for (int64_t i = j0; i < j1 && rc == MDET_OK; ++i) {
              upload_row(i);
              for (int64_t t = 0; t < cnt && rc == MDET_OK; ++t) update_own_row(k + t, i);
            }
          } else {
            for (int64_t t = 0; t < cnt && rc == MDET_OK; ++t) update_group_rows(k + t);
          }
          for (int64_t i = j1; i < T_ && rc == MDET_OK; ++i) {
            if (k == 0) upload_row(i);
            for (int64_t t = 0; t < cnt && rc == MDET_OK; ++t) stream_block(k + t, i);
          }
          for (int64_t t = 0; t < cnt; ++t) {
            const int q = (int)((k + t) & 1);
            if (!b_free[q]) b_free[q] = events.get();
            MDET_HIP(fail, hipEventRecord(b_free[q], s0));
          }
          k += cnt;
        }
        if (rc == MDET_OK) {
          ResidentHooks hooks;
          hooks.column_final = mark_final;
          hooks.column_flush = write_back;
          // the last group need not be written back: nothing will stream it again
          if (j1 == T_) hooks.column_final = hooks.column_flush = nullptr;
          rc = factor_resident(L, pl, cols, j0, j1, false, lookahead, s0, s1, events, &hooks);
        }
      }
      ev_arena_free = events.get();
      MDET_HIP(fail, hipEventRecord(ev_arena_free, s0));   // s1 was joined into s0
    }
  }

  if (rc == MDET_OK) L.reduce(s0, n, bs, T_, partial, out, running);
  DeviceOut o;
  std::memset(&o, 0, sizeof(o));
  if (rc == MDET_OK) {
    MDET_HIP(fail, hipMemcpyAsync(o.out, out, sizeof(o.out), hipMemcpyDeviceToHost, s0));
    MDET_HIP(fail, hipMemcpyAsync(&o.flags, L.flags, sizeof(DevFlags), hipMemcpyDeviceToHost, s0));
    if (diag_host && n > 0)
      MDET_HIP(fail, hipMemcpyAsync(diag_host, L.dvec, n * sizeof(T), hipMemcpyDeviceToHost, s0));
    if (L.perm && p.perm && n > 0)
      MDET_HIP(fail, hipMemcpyAsync(p.perm, L.perm, n * sizeof(int), hipMemcpyDeviceToHost, s0));
  }
  MDET_HIP(fail, hipStreamSynchronize(sh));
  MDET_HIP(fail, hipStreamSynchronize(s1));
  MDET_HIP(fail, hipStreamSynchronize(s0));
  MDET_HIP(fail, hipStreamSynchronize(sd));
  res->flops = 2.0 * L.fma;
  res->kernel_launches = L.launches;
  L.collect_profile(res);
  res->bytes_h2d = h2d_bytes;
  res->bytes_d2h = d2h_bytes;
  res->t_h2d = cprof.collect(0);
  res->t_d2h = cprof.collect(1);
  res->dev_bytes_high_water = sa.total + pl.pb_bytes + pl.stage_bytes + (pl.general ? pl.arena_half : 0) + arena_used;
  if (prov_rc != MDET_OK) return prov_rc;
  if (stager_in.io_failed() || stager_out.io_failed()) return MDET_EIO;
  if (!fail.ok()) { res->hip_error = fail.code; return MDET_EHIP; }
  if (rc != MDET_OK) return rc;
  rc = finish_result(o, res);
  // the permutation's sign: one factor of -1 for every leaf with an odd row order
  if (pl.general && (o.flags.odd_leaves & 1ull)) res->sign = -res->sign;
  return rc;
}

// Runs the host path in the arithmetic's type.  hA: the matrix as stored (host memory; ignored
// when `provider` is given).  The factored block columns of a streamed run go to hA itself
// (overwrite = 1 and the matrix stored in the arithmetic's type), else to the caller's
// host_scratch, else to memory the library allocates (pinned if that much can be pinned).
static int logdet_host_any(const mdet_params* p, void* hA, mdet_result* res, void* diag,
                           mdet_block_provider provider = nullptr, void* user = nullptr,
                           mdet_block_provider_device provider_dev = nullptr) {
  Plan pl;
  int rc = make_plan(*p, false, 0, pl);
  init_result(res, pl);
  if (rc != MDET_OK) return rc;
  PinnedBuf scratch;
  std::unique_ptr<char[]> plain_scratch;
  // blocks produced on the device arrive in the arithmetic's type, one triangle
  if (provider_dev && (pl.widen || pl.general)) return MDET_EINVAL;
  const bool own_store = pl.widen || provider != nullptr || provider_dev != nullptr;   // the factors cannot go where the matrix is
  void* hOut = own_store ? nullptr : hA;
  const uint64_t store_bytes = (pl.general ? 2 : 1) * pl.layout_bytes;
  if (pl.out_of_core && (!p->overwrite || own_store)) {
    if (p->host_scratch) {
      if (p->host_scratch_bytes < store_bytes) return MDET_ENOMEM_HOST;
      hOut = p->host_scratch;
    } else if (scratch.alloc(store_bytes) == MDET_OK) {
      hOut = scratch.p;
    } else {
      // more than can be pinned: ordinary memory, which the host path stages itself
      plain_scratch.reset(new (std::nothrow) char[store_bytes ? store_bytes : 1]);
      if (!plain_scratch) return MDET_ENOMEM_HOST;
      hOut = plain_scratch.get();
    }
  }
  HostSource src;
  src.narrow = pl.widen ? (const char*)hA : nullptr;
  src.dtype = p->dtype;
  src.provider = provider;
  src.provider_dev = provider_dev;
  src.user = user;
  const HostSource* sp = (pl.widen || provider || provider_dev) ? &src : nullptr;
  auto t0 = std::chrono::steady_clock::now();
  if (p->dtype == MDET_F64 || pl.widen)
    rc = logdet_host_t<double>(*p, pl, own_store ? nullptr : (double*)hA, (double*)hOut, res, (double*)diag, -1, -1, sp);
  else
    rc = logdet_host_t<float>(*p, pl, own_store ? nullptr : (float*)hA, (float*)hOut, res, (float*)diag, -1, -1, sp);
  res->t_total = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  return rc;
}

// The matrix in a file (packed layout at the start of it), optionally a second file for
// the factors.
static int logdet_file_any(const mdet_params* p, const char* matrix_path, const char* scratch_path,
                           mdet_result* res, void* diag) {
  Plan pl;
  int rc = make_plan(*p, false, 0, pl);
  init_result(res, pl);
  if (rc != MDET_OK) return rc;
  struct Fd {
    int fd = -1;
    ~Fd() { if (fd >= 0) ::close(fd); }
  } in, out;
  const bool writes = pl.out_of_core;              // factored columns are stored only when they stream
  const bool in_place = writes && p->overwrite && !pl.widen;
  in.fd = ::open(matrix_path, in_place ? O_RDWR : O_RDONLY);
  if (in.fd < 0) return MDET_EIO;
  struct stat sb;
  const uint64_t arrays = pl.general ? 2 : 1;
  if (::fstat(in.fd, &sb) != 0 || (uint64_t)sb.st_size < arrays * (pl.layout_bytes / pl.beta * pl.src_beta))
    return MDET_EIO;
  int fd_out = in.fd;
  if (writes && !in_place) {
    if (!scratch_path) return MDET_EINVAL;
    out.fd = ::open(scratch_path, O_RDWR | O_CREAT, 0600);
    if (out.fd < 0) return MDET_EIO;
    if (::ftruncate(out.fd, (off_t)(arrays * pl.layout_bytes)) != 0) return MDET_EIO;
    fd_out = out.fd;
  }
  HostSource src;
  src.narrow = nullptr;          // byte offset 0 of the matrix file
  src.dtype = p->dtype;
  const HostSource* sp = pl.widen ? &src : nullptr;
  auto t0 = std::chrono::steady_clock::now();
  if (p->dtype == MDET_F64 || pl.widen)
    rc = logdet_host_t<double>(*p, pl, (double*)nullptr, (double*)nullptr, res, (double*)diag, in.fd, fd_out, sp);
  else
    rc = logdet_host_t<float>(*p, pl, (float*)nullptr, (float*)nullptr, res, (float*)diag, in.fd, fd_out, sp);
  res->t_total = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  return rc;
}

}  // namespace mdet

// ===========================================================================
// extern "C"
// ===========================================================================
using namespace mdet;

static bool params_ok(const mdet_params* p) {
  return p && p->struct_size == sizeof(mdet_params) && p->n >= 0 && p->block_size >= 0 &&
         (p->dtype == MDET_F32 || p->dtype == MDET_F64 || p->dtype == MDET_F16 || p->dtype == MDET_BF16);
}

extern "C" {

const char* mdet_strerror(int s) {
  switch (s) {
    case MDET_OK: return "ok";
    case MDET_EINVAL: return "invalid argument";
    case MDET_EBUDGET: return "memory budget below the minimum working set";
    case MDET_ENOMEM_DEVICE: return "device memory allocation failed or workspace too small";
    case MDET_ENOMEM_HOST: return "host memory allocation failed";
    case MDET_EHIP: return "HIP runtime error (see result.hip_error)";
    case MDET_ESINGULAR: return "matrix is singular: exact zero pivot";
    case MDET_ENONFINITE: return "non-finite pivot";
    case MDET_EPROVIDER: return "block provider failed";
    case MDET_ENOTPOSDEF: return "matrix is not positive definite: a pivot is negative";
    case MDET_EIO: return "file could not be opened, is too short, or a read or write failed";
    default: return "unknown status";
  }
}

const char* mdet_version(void) { return "memdet-mi355x 0.1 (gfx950)"; }

int mdet_paper_block_rule(int64_t m, int32_t beta, uint64_t c, int64_t* n_b, int64_t* b) {
  if (m <= 0 || beta <= 0 || c == 0 || !n_b || !b) return MDET_EINVAL;
  long double r = (long double)m * sqrtl((long double)beta / (long double)c);
  int64_t nb;
  if (r <= 1.0L) nb = 1;
  else if (r <= 2.0L / sqrtl(3.0L)) nb = 2;
  else nb = (int64_t)ceill(2.0L * r);
  *n_b = nb;
  *b = 1 + (m - 1) / nb;
  return MDET_OK;
}

double mdet_paper_fma_count(int64_t m) {
  double x = (double)m;
  return x * x * x / 6.0 - x * x / 4.0 + x / 12.0;
}

int64_t mdet_host_layout_offset(int64_t n, int64_t b, int64_t j) {
  if (n < 0 || b <= 0 || b % 64 != 0 || j < 0) return -1;
  Plan pl;
  pl.n = n; pl.bs = b; pl.T = n > 0 ? (n + b - 1) / b : 0;
  if (j > pl.T) return -1;
  if (pl.T == 0) return 0;
  return pl.col_offset(j);
}

int mdet_plan(const mdet_params* p, int for_device_input, mdet_plan_info* info) {
  if (!params_ok(p) || !info) return MDET_EINVAL;
  Plan pl;
  int rc = make_plan(*p, for_device_input != 0, round_up(p->n > 0 ? p->n : 1, 4), pl);
  std::memset(info, 0, sizeof(*info));
  info->block_size_used = pl.bs;
  info->num_blocks = pl.T;
  if (rc != MDET_OK) return rc;
  info->out_of_core = pl.out_of_core;
  info->num_superpanels = (int32_t)pl.panels.size();
  info->dev_bytes_needed = pl.dev_bytes;
  info->host_bytes_needed = pl.host_bytes;
  info->host_matrix_bytes = pl.layout_bytes;
  info->stream_bytes_h2d = pl.h2d;
  info->stream_bytes_d2h = pl.d2h;
  paper_work_split(pl.T, (double)pl.bs, &info->fma_decomp, &info->fma_solve, &info->fma_gemm,
                   &info->fma_syrk);
  return MDET_OK;
}

int mdet_workspace_query(const mdet_params* p, int for_device_input, uint64_t* dev_bytes,
                         uint64_t* host_bytes) {
  mdet_plan_info info;
  int rc = mdet_plan(p, for_device_input, &info);
  if (rc != MDET_OK) return rc;
  if (dev_bytes) *dev_bytes = info.dev_bytes_needed;
  if (host_bytes) *host_bytes = info.host_bytes_needed;
  return MDET_OK;
}

int mdet_logdet_device(const mdet_params* p, void* dA, int64_t ld, mdet_result* res, void* diag) {
  if (!params_ok(p) || !res) return MDET_EINVAL;
  if (p->n > 0 && (!dA || ld < p->n)) return MDET_EINVAL;
  Plan pl;
  int rc = make_plan(*p, true, ld, pl);
  init_result(res, pl);
  if (rc != MDET_OK) return rc;
  if (p->n > 0 && ((uintptr_t)dA & 15u)) return MDET_EINVAL;
  auto t0 = std::chrono::steady_clock::now();
  if (p->dtype == MDET_F64) rc = logdet_device_t<double>(*p, pl, (double*)dA, ld, res, (double*)diag);
  else if (p->flags & MDET_FLAG_COMPUTE_F64)
    rc = logdet_device_t<double>(*p, pl, nullptr, ld, res, (double*)diag, (const void*)dA);
  else rc = logdet_device_t<float>(*p, pl, (float*)dA, ld, res, (float*)diag);
  res->t_total = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  return rc;
}

int mdet_logdet_device_noalloc(const mdet_params* p, void* dA, int64_t ld, double* out, void* diag) {
  if (!params_ok(p) || !out) return MDET_EINVAL;
  if (p->n > 0 && (!dA || ld < p->n || ((uintptr_t)dA & 15u))) return MDET_EINVAL;
  if (p->dtype != MDET_F64 && p->dtype != MDET_F32) return MDET_EINVAL;
  // in place only (a copy would be workspace of the matrix's size), plain symmetric forms only
  if (!p->overwrite || (p->flags & ~(uint32_t)(MDET_FLAG_NO_LOOKAHEAD | MDET_FLAG_ASSUME_SPD | MDET_FLAG_PIVOT)))
    return MDET_EINVAL;
  mdet_params q = *p;
  q.flags |= MDET_FLAG_NO_LOOKAHEAD;
  q.mem_budget_bytes = 0;
  q.dev_workspace = nullptr;
  Plan pl;
  int rc = make_plan(q, true, ld, pl);
  if (rc != MDET_OK) return rc;
  if (pl.need_copy) return MDET_EINVAL;            // rows not 16-byte aligned
  // the fixed array must hold the whole small area; the optional pivot-scaled copies are not used
  pl.wcopy_bytes = 0;
  if (small_area(pl.n, pl.T, pl.beta, pl.pivot).total > NOALLOC_SCRATCH_BYTES) return MDET_ENOMEM_DEVICE;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return MDET_EHIP; }
  char* base = nullptr;
  if (scratch_address(dev, &base) != hipSuccess) { (void)hipGetLastError(); return MDET_EHIP; }
  if (p->dtype == MDET_F64)
    return logdet_device_noalloc_t<double>(q, pl, base, (double*)dA, ld, out, (double*)diag);
  return logdet_device_noalloc_t<float>(q, pl, base, (float*)dA, ld, out, (float*)diag);
}

int mdet_step_schur_update(int32_t dtype, void* C, int64_t ldc, const void* A, int64_t lda,
                           const void* B, int64_t ldb, const void* d, int64_t M, int64_t N,
                           int64_t K, int32_t lower, void* stream) {
  if (!C || !A || !B || M < 0 || N < 0 || K < 0) return MDET_EINVAL;
  HipFail fail;
  int rc;
  // d == NULL: the positive-definite form, C -= A B^T (the operand pointer stands in for the
  // pivots the launcher's alignment check looks at; the kernel never reads them)
  if (dtype == MDET_F64) {
    Launcher<double> L; L.fail = &fail; L.spd = d == nullptr;
    rc = L.update((hipStream_t)stream, (double*)C, ldc, (const double*)A, lda, (const double*)B, ldb,
                  (const double*)(d ? d : A), M, N, K, lower != 0, true);
  } else if (dtype == MDET_F32) {
    Launcher<float> L; L.fail = &fail; L.spd = d == nullptr;
    rc = L.update((hipStream_t)stream, (float*)C, ldc, (const float*)A, lda, (const float*)B, ldb,
                  (const float*)(d ? d : A), M, N, K, lower != 0, true);
  } else return MDET_EINVAL;
  if (!fail.ok()) return MDET_EHIP;
  return rc;
}

static int step_panel_factor(int32_t dtype, void* P, int64_t ld, int64_t m, int64_t w, void* d,
                             void* dinv, int32_t* perm, int64_t pivot_index0, void* flags, void* stream) {
  if (!P || !d || !dinv || !flags || m < 0 || w < 0 || w > m || ld < w) return MDET_EINVAL;
  if (perm && pivot_index0 + w > INT32_MAX) return MDET_EINVAL;
  HipFail fail;
  int rc;
  if (dtype == MDET_F64) {
    if (ld % 2 || ((uintptr_t)P & 15u)) return MDET_EINVAL;
    Launcher<double> L; L.fail = &fail;
    // the launcher indexes dvec/dinv/perm by global pivot index
    L.dvec = (double*)d - pivot_index0; L.dinv = (double*)dinv - pivot_index0; L.flags = (DevFlags*)flags;
    L.linv = (double*)((char*)flags + 16);
    L.perm = perm ? perm - pivot_index0 : nullptr;
    rc = L.factor_cols((hipStream_t)stream, (double*)P, ld, m, w, pivot_index0);
  } else if (dtype == MDET_F32) {
    if (ld % 4 || ((uintptr_t)P & 15u)) return MDET_EINVAL;
    Launcher<float> L; L.fail = &fail;
    L.dvec = (float*)d - pivot_index0; L.dinv = (float*)dinv - pivot_index0; L.flags = (DevFlags*)flags;
    L.linv = (float*)((char*)flags + 16);
    L.perm = perm ? perm - pivot_index0 : nullptr;
    rc = L.factor_cols((hipStream_t)stream, (float*)P, ld, m, w, pivot_index0);
  } else return MDET_EINVAL;
  if (!fail.ok()) return MDET_EHIP;
  return rc;
}

int mdet_step_panel_factor(int32_t dtype, void* P, int64_t ld, int64_t m, int64_t w, void* d,
                           void* dinv, int64_t pivot_index0, void* flags, void* stream) {
  return step_panel_factor(dtype, P, ld, m, w, d, dinv, nullptr, pivot_index0, flags, stream);
}

int mdet_step_panel_factor_pivoted(int32_t dtype, void* P, int64_t ld, int64_t m, int64_t w, void* d,
                                   void* dinv, int32_t* perm, int64_t pivot_index0, void* flags,
                                   void* stream) {
  if (!perm) return MDET_EINVAL;
  return step_panel_factor(dtype, P, ld, m, w, d, dinv, perm, pivot_index0, flags, stream);
}

extern "C++" {
template <typename T>
static int step_panel_factor_general(T* P, T* Q, int64_t ld, int64_t m, int64_t w, T* d, T* dinv, int32_t* perm,
                                     int64_t pivot_index0, void* flags, hipStream_t st) {
  constexpr int vec = 16 / (int)sizeof(T);
  const ptrdiff_t bytes = (const char*)Q - (const char*)P;
  if (ld % vec || ((uintptr_t)P & 15u) || bytes % 16 != 0 || bytes == 0) return MDET_EINVAL;
  HipFail fail;
  Launcher<T> L;
  L.fail = &fail;
  L.dvec = d - pivot_index0;
  L.dinv = dinv - pivot_index0;
  L.perm = perm - pivot_index0;
  L.flags = (DevFlags*)flags;
  L.linv = (T*)((char*)flags + 32);
  L.linv_u = L.linv + LEAF * SUB;
  L.qoff = bytes / (ptrdiff_t)sizeof(T);
  const int rc = L.factor_cols(st, P, ld, m, w, pivot_index0);
  if (!fail.ok()) return MDET_EHIP;
  return rc;
}
}  // extern "C++"

int mdet_step_panel_factor_general(int32_t dtype, void* P, void* Q, int64_t ld, int64_t m, int64_t w, void* d,
                                   void* dinv, int32_t* perm, int64_t pivot_index0, void* flags,
                                   void* stream) {
  if (!P || !Q || !d || !dinv || !perm || !flags || m < 0 || w < 0 || w > m || ld < w) return MDET_EINVAL;
  if (pivot_index0 < 0 || pivot_index0 + w > INT32_MAX) return MDET_EINVAL;
  if (dtype == MDET_F64)
    return step_panel_factor_general<double>((double*)P, (double*)Q, ld, m, w, (double*)d, (double*)dinv, perm,
                                             pivot_index0, flags, (hipStream_t)stream);
  if (dtype == MDET_F32)
    return step_panel_factor_general<float>((float*)P, (float*)Q, ld, m, w, (float*)d, (float*)dinv, perm,
                                            pivot_index0, flags, (hipStream_t)stream);
  return MDET_EINVAL;
}

int mdet_step_logdet_reduce(int32_t dtype, const void* d, int64_t n, double* out, void* stream) {
  if (!d || !out || n < 0) return MDET_EINVAL;
  HipFail fail;
  // single block column: partial terms live right behind the three outputs
  double* partial = out + 3;
  if (dtype == MDET_F64) {
    Launcher<double> L; L.fail = &fail; L.dvec = (double*)d;
    L.reduce((hipStream_t)stream, n, n > 0 ? n : 1, n > 0 ? 1 : 0, partial, out, nullptr);
  } else if (dtype == MDET_F32) {
    Launcher<float> L; L.fail = &fail; L.dvec = (float*)d;
    L.reduce((hipStream_t)stream, n, n > 0 ? n : 1, n > 0 ? 1 : 0, partial, out, nullptr);
  } else return MDET_EINVAL;
  return fail.ok() ? MDET_OK : MDET_EHIP;
}

}  // extern "C"

extern "C" int mdet_logdet_host(const mdet_params* p, void* hA, mdet_result* res, void* diag) {
  if (!params_ok(p) || !res) return MDET_EINVAL;
  if (p->n > 0 && !hA) return MDET_EINVAL;
  return logdet_host_any(p, hA, res, diag);
}

extern "C" int mdet_logdet_file(const mdet_params* p, const char* matrix_path, const char* scratch_path,
                                mdet_result* res, void* diag) {
  if (!params_ok(p) || !res || !matrix_path) return MDET_EINVAL;
  return logdet_file_any(p, matrix_path, scratch_path, res, diag);
}

extern "C" int mdet_logdet_provider(const mdet_params* p, mdet_block_provider provider, void* user,
                                    mdet_result* res, void* diag) {
  if (!params_ok(p) || !res || !provider) return MDET_EINVAL;
  // The blocks are fetched when the schedule first needs them, each into a pinned buffer and
  // from there to the device: host memory holds no copy of the matrix.  Only a run that
  // streams keeps its factored block columns in host memory (the caller's host_scratch or the
  // library's own).
  return logdet_host_any(p, nullptr, res, diag, provider, user);
}

// The same with blocks that the caller's function produces in device memory, with work it queues on
// the stream it is handed: nothing of the matrix crosses the host link.
extern "C" int mdet_logdet_provider_device(const mdet_params* p, mdet_block_provider_device provider,
                                           void* user, mdet_result* res, void* diag) {
  if (!params_ok(p) || !res || !provider) return MDET_EINVAL;
  return logdet_host_any(p, nullptr, res, diag, nullptr, user, provider);
}
