// Leaf kernels of the block-column factorisation (LEAF = 64 columns at a time).
//
// leaf_factor_kernel : in-place A = L D L^T of one <= 64 x 64 diagonal leaf
//                      (Sec. 2.2: "in-place ... decomposition" of the diagonal block,
//                      symmetric case: unit-lower L, diagonal D, no pivoting).
// leaf_factor_pivoted_kernel : the same with the pivot taken from the diagonal inside the
//                      leaf, P A P^T = L D L^T (Sec. 2.2: the symmetric form handles
//                      permutations; pivoting inside a block, none between blocks).
// leaf_lu_kernel     : a leaf of a general matrix, P A = L D U with unit-lower L, diagonal D
//                      and unit-upper U, the pivot of each column taken among the leaf's
//                      rows (Sec. 2.2, Eq. 1 and Alg. 1: M = P L U for generic matrices;
//                      pivoting inside a block, none between blocks).
// leaf_solve_kernel  : rows below the leaf, X = A_rows L^-T D^-1
//                      (Sec. 2.2: in-place triangular solve of the off-diagonal
//                      blocks; App. E.1 "solve lower triangular system"; the
//                      D^-1 is the LDL^T "diagonal scaling").  On request also
//                      W = X D into a second array, for the rows from `wfrom` on:
//                      the operand of the Schur updates with the scaling applied,
//                      rounded as the update kernels round l * d.
// leaf_solve_general_kernel : the same for both triangles of a general matrix in one
//                      launch (rows of the lower one against U^T, rows of the transposed
//                      upper one against L with the leaf's row order as column gather).
// transpose_strict_kernel : the entries above the diagonal of a general matrix into their
//                      transposed store, and back.
//
// leaf_factor_kernel and leaf_solve_kernel work on 16-column sub-blocks: the sequential part (elimination inside a
// 16 x 16 diagonal sub-block) runs on the vector ALUs with one matrix row per lane,
// everything else (updates inside the leaf, the substitution against already
// solved sub-blocks) is 16 x 16 x 16 products on the matrix cores.  The loops over
// sub-blocks are real loops, so the code stays small enough for the instruction
// cache.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma.h"

namespace mdet {

constexpr int LEAF = 64;
constexpr int SUB = 16;               // sub-block order = MFMA tile order
constexpr int NSUB = LEAF / SUB;
constexpr int LEAF_PAD = LEAF + 1;    // LDS row stride of a leaf tile
constexpr int SUB_PAD = SUB + 1;

// Device-side status words shared by all kernels of one call.
struct DevFlags {
  unsigned long long first_bad;   // global index of the first zero / non-finite pivot; ~0 = none
  unsigned long long bad_kind;    // 1 = zero, 2 = non-finite
  unsigned long long odd_leaves;  // general matrices: leaves whose row order is an odd permutation
};

// Value of `v` in lane `src` (uniform lane index), delivered in scalar registers.
__device__ __forceinline__ double lane_value(double v, int src) {
  int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ float lane_value(float v, int src) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}

// Coalesced movement of a rows x cols tile (<= 64 x 64) from global memory into an
// LDS array with row stride `stride`, by one wavefront, in two halves of 32 rows.
// tile_fetch issues the 32 independent loads of one half (so their latencies
// overlap, and the loads of two different tiles can be in flight together);
// tile_put writes them to LDS.  Missing rows/columns read as 0 (diagonal entries
// of the padding as 1 when unit_pad is set).  With TRANSPOSE the element (r, c)
// lands at lds[c * stride + r].
constexpr int TILE_HALF = 32;   // rows per half = loads per lane per half

template <typename T, bool STRICT_LOWER>
__device__ __forceinline__ void tile_fetch(T (&v)[TILE_HALF], int half, const T* g, int64_t ld,
                                           int rows, int cols, bool unit_pad, int lane) {
#pragma unroll
  for (int q = 0; q < TILE_HALF; ++q) {
    const int r = half * TILE_HALF + q, c = lane;
    const bool in = r < rows && c < cols && (!STRICT_LOWER || c < r);
    v[q] = in ? g[(int64_t)r * ld + c] : ((unit_pad && r == c) ? T(1) : T(0));
  }
}
template <typename T, bool TRANSPOSE>
__device__ __forceinline__ void tile_put(const T (&v)[TILE_HALF], int half, T* lds, int stride,
                                         int lane) {
#pragma unroll
  for (int q = 0; q < TILE_HALF; ++q) {
    const int r = half * TILE_HALF + q, c = lane;
    lds[TRANSPOSE ? c * stride + r : r * stride + c] = v[q];
  }
}

// ---------------------------------------------------------------------------
// leaf factor
// ---------------------------------------------------------------------------
// 1/d to within a couple of ulp: hardware estimate refined by two Newton steps
// (the sequence an exact division expands to, minus its final correction and
// range scaling; pivots that would need scaling are far outside what a
// factorisation without pivoting can use anyway).
__device__ __forceinline__ double fast_rcp(double d) {
  double r = __builtin_amdgcn_rcp(d);
  r = fma(fma(-d, r, 1.0), r, r);
  r = fma(fma(-d, r, 1.0), r, r);
  return r;
}
__device__ __forceinline__ float fast_rcp(float d) {
  float r = __builtin_amdgcn_rcpf(d);
  r = fmaf(fmaf(-d, r, 1.0f), r, r);
  return r;
}

// Elimination of one 16-column panel held one row per lane (a[q] = entry (lane, c0+q)),
// column by column.  Column J first receives the updates of the columns before it,
//   a_iJ -= w_ik l_Jk,  k = 0 .. J-1,   w_ik = d_k l_ik (entry (i, k) before its division),
// then lane c0+J owns the pivot d_J and the lanes below it get l_iJ = a_iJ / d_J.
// The l_Jk are the same for every lane.  A value broadcast from a lane's register
// costs two v_readlane per double (10 to 15 clocks of the wavefront's own issue time);
// a same-address LDS read costs a third of that and the LDS works beside the vector
// ALU.  So every finished column goes to the tile in LDS in its final form (l below
// the diagonal, d on it) and row J+1 of the finished columns is fetched one step
// ahead.  Only the newest column's entry comes by v_readlane, before its division
// (an LDS round trip would sit on the chain of dependent steps); that one term is
// formed as l_i,J-1 w_J,J-1.  Column J-1 is written at the top of step J, after the
// reads of the older columns of row J+1 have been issued: LDS operations finish in
// order, and this way nothing that step J waits for is younger than a whole step.
// Rows above the panel's diagonal block (lanes < c0) compute on unused entries.
// On return the tile holds the panel's final columns.
template <typename T>
__device__ __forceinline__ void panel16_eliminate(T (&a)[SUB], T* tile, const int c0,
                                                  const int lane) {
  T* mine = tile + lane * LEAF_PAD + c0;
  T w[SUB];          // this row's entries before their division
  T row[SUB];        // l_Jk, k < J-1, for the current step
  T newest = T(0);   // w_J,J-1
#pragma unroll
  for (int J = 0; J < SUB; ++J) {
    T ahead[SUB];
    const T* next_row = tile + (c0 + J + 1) * LEAF_PAD + c0;
    if (J + 1 < SUB) {
#pragma unroll
      for (int k = 0; k + 1 < J; ++k) ahead[k] = next_row[k];
    }
    if (J > 0) mine[J - 1] = a[J - 1];
    if (J > 0 && J + 1 < SUB) ahead[J - 1] = next_row[J - 1];
    // keep the LDS traffic up here and its uses in the next step: moved next to each
    // other, every step would wait out the LDS latency
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k + 1 < J; ++k) a[J] -= w[k] * row[k];
    if (J > 0) a[J] -= a[J - 1] * newest;
    const T wj = a[J];
    w[J] = wj;
    const T dj = lane_value(wj, c0 + J);
    if (J + 1 < SUB) newest = lane_value(wj, c0 + J + 1);
    const T lj = wj * fast_rcp(dj);
    a[J] = lane > c0 + J ? lj : wj;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < J; ++k) row[k] = ahead[k];
  }
  mine[SUB - 1] = a[SUB - 1];
}

// Inverse of the unit-lower diagonal sub-block b of the leaf in `tile` -> linv.
// Lane (l16, g) computes column l16: x_i = delta_{i,l16} - sum_{k<i} L[i][k] x_k, the
// terms in the order k = 0, 1, ...; the entries of L are same-address LDS reads,
// requested a group of rows ahead of the group being computed.  Left to itself the
// compiler either puts each read next to its use, so that the latency of every one
// shows, or issues all 120 at once and needs 300 registers: each group therefore
// reads through an index the compiler cannot see through (a zero that has passed an
// empty asm statement), which ties the reads to the place where they are written.
__device__ __forceinline__ int opaque_zero() {
  int z = 0;
  asm volatile("" : "+v"(z));
  return z;
}
template <typename T, int I0, int I1>
__device__ __forceinline__ void invert_fetch(const T* Lb, T (&l)[SUB * (SUB - 1) / 2]) {
  const T* p = Lb + opaque_zero();
#pragma unroll
  for (int i = I0; i < I1; ++i)
#pragma unroll
    for (int k = 0; k < i; ++k) l[i * (i - 1) / 2 + k] = p[i * LEAF_PAD + k];
}
template <typename T, int I0, int I1>
__device__ __forceinline__ void invert_rows(const T (&l)[SUB * (SUB - 1) / 2], T (&x)[SUB],
                                            const int l16) {
#pragma unroll
  for (int i = I0; i < I1; ++i) {
    T v = i == l16 ? T(1) : T(0);
#pragma unroll
    for (int k = 0; k < i; ++k) v -= l[i * (i - 1) / 2 + k] * x[k];
    x[i] = v;
  }
}
template <typename T>
__device__ __forceinline__ void leaf_invert_sub(const T* tile, T* __restrict__ linv, const int b,
                                                const int l16) {
  const T* Lb = tile + (b * SUB) * LEAF_PAD + b * SUB;
  T l[SUB * (SUB - 1) / 2], x[SUB];
  // groups of rows with about 20 entries each; two groups are in flight at a time
  invert_fetch<T, 1, 6>(Lb, l);
  invert_fetch<T, 6, 9>(Lb, l);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 0, 6>(l, x, l16);
  invert_fetch<T, 9, 11>(Lb, l);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 6, 9>(l, x, l16);
  invert_fetch<T, 11, 13>(Lb, l);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 9, 11>(l, x, l16);
  invert_fetch<T, 13, 14>(Lb, l);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 11, 13>(l, x, l16);
  invert_fetch<T, 14, 15>(Lb, l);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 13, 14>(l, x, l16);
  invert_fetch<T, 15, 16>(Lb, l);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 14, 15>(l, x, l16);
  __builtin_amdgcn_sched_barrier(0);
  invert_rows<T, 15, 16>(l, x, l16);
  // all four groups of 16 lanes hold the same columns and store the same values (a
  // store by one group only would let the compiler move the arithmetic into that
  // branch, behind all the reads)
#pragma unroll
  for (int i = 0; i < SUB; ++i) linv[(b * SUB + i) * SUB + l16] = x[i];
}

// Four wavefronts factor one leaf held in LDS, 16 columns at a time:
//   wavefront 0: panel (rows from its diagonal down) -> registers (one row per
//                lane), eliminated, written back;
//   then all:    every sub-block right of / below the panel updated with 16x16x16
//                MFMA products, shared round-robin;
//   wavefront 3: while wavefront 0 eliminates panel b, inverts panel b-1's
//                unit-lower diagonal sub-block into `linv` (used by the solve kernel).
constexpr int FACTOR_THREADS = 256;

// LDS the factorisation needs, in elements: the leaf.
constexpr int FACTOR_LDS_ELEMS = LEAF * LEAF_PAD;

// The work of all FACTOR_THREADS threads of one workgroup; `lds` points at
// FACTOR_LDS_ELEMS elements of shared memory nobody else uses.  The update
// kernels call it too: the workgroup that has just reduced the top-left 64 x 64
// block of its launch factors that block straight away, which takes one kernel
// (and its launch-to-launch latency) off the chain of dependent launches.
//
// With IN_LDS the caller has put the leaf into `lds` already, entry by entry with
// leaf_tile_put and a barrier after the last one (an update kernel hands over its
// accumulators: writing the block to memory and reading it back would cost a memory
// round trip on the chain of dependent launches); A is then only written.
template <typename T>
__device__ __forceinline__ void leaf_tile_put(T* __restrict__ lds, int row, int col, int w, T v) {
  if (row < LEAF && col < LEAF)
    lds[row * LEAF_PAD + col] = (row < w && col < w) ? v : (row == col ? T(1) : T(0));
}

//
// spd != 0: the positive-definite form.  The leaf is still factored as L D L^T, but
// every pivot must be positive (the first that is not is reported with kind 4) and
// dinv receives d^(-1/2) instead of 1/d: the rows below the leaf, solved with that
// scaling, are then rows of the Cholesky factor L D^(1/2), and the updates that use
// them need no pivots.
template <typename T, bool IN_LDS = false>
__device__ __forceinline__ void leaf_factor_body(
    T* __restrict__ A, int64_t ld, int w, T* __restrict__ dvec, T* __restrict__ dinv,
    T* __restrict__ linv, long long pivot0, DevFlags* flags, T* __restrict__ lds, int spd = 0) {
  using X = Mfma<T>;
  using acc_t = typename X::acc_t;
  T* tile = lds;
  // The elimination is one long chain of dependent instructions; beside a
  // workgroup of the trailing update on the same SIMDs it would otherwise get an
  // issue slot only now and then.
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in all lanes: scalar branches
  const int l16 = lane & 15, g = lane >> 4;
  if constexpr (!IN_LDS) {
    // 64 x 64 tile, 16 entries per thread, all requests in flight together
    T v[LEAF * LEAF / FACTOR_THREADS];
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / FACTOR_THREADS; ++q) {
      const int e = q * FACTOR_THREADS + tid, r = e >> 6, c = e & 63;
      v[q] = (r < w && c < w) ? A[(int64_t)r * ld + c] : (r == c ? T(1) : T(0));
    }
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / FACTOR_THREADS; ++q) {
      const int e = q * FACTOR_THREADS + tid, r = e >> 6, c = e & 63;
      tile[r * LEAF_PAD + c] = v[q];
    }
    __syncthreads();
  }

#pragma unroll 1
  for (int b = 0; b < NSUB; ++b) {
    const int c0 = b * SUB;
    if (wave == 0) {
      T a[SUB];
#pragma unroll
      for (int q = 0; q < SUB; ++q) a[q] = tile[lane * LEAF_PAD + c0 + q];
      panel16_eliminate<T>(a, tile, c0, lane);
    } else if (wave == 3 && b > 0) {
      // meanwhile: inverse of the previous panel's diagonal sub-block
      leaf_invert_sub<T>(tile, linv, b - 1, l16);
    } else if (b == NSUB - 1) {
      // wavefronts 1 and 2 have no part in the last panel: they write back the
      // columns that are final already (all but the last panel's)
      constexpr int DONE = (NSUB - 1) * SUB;
      for (int e = tid - 64; e < LEAF * DONE; e += 128) {
        const int r = e / DONE, c = e % DONE;
        if (r < w && c <= r) A[(int64_t)r * ld + c] = tile[r * LEAF_PAD + c];
      }
    }
    __syncthreads();
    // trailing sub-blocks (ti, tj), b < tj <= ti:  S -= L[ti, b] D_b L[tj, b]^T
    {
      const int nt = NSUB - 1 - b;               // sub-block rows/columns left
      const int ntiles = nt * (nt + 1) / 2;
#pragma unroll 1
      for (int t = wave; t < ntiles; t += 4) {
        int ti = 0;
        while ((ti + 1) * (ti + 2) / 2 <= t) ++ti;
        const int tj = t - ti * (ti + 1) / 2;
        const int R = (b + 1 + ti) * SUB, Cc = (b + 1 + tj) * SUB;
        acc_t acc;
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = tile[(R + X::acc_row(lane, r)) * LEAF_PAD + Cc + l16];
        T aop[4], bop[4];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const int k = c0 + 4 * s4 + g;
          aop[s4] = -(tile[(R + l16) * LEAF_PAD + k] * tile[k * LEAF_PAD + k]);   // -(l d)
          bop[s4] = tile[(Cc + l16) * LEAF_PAD + k];
        }
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) acc = X::mfma(aop[s4], bop[s4], acc);
#pragma unroll
        for (int r = 0; r < 4; ++r) tile[(R + X::acc_row(lane, r)) * LEAF_PAD + Cc + l16] = acc[r];
      }
    }
    __syncthreads();
  }
  if (wave == 3) leaf_invert_sub<T>(tile, linv, NSUB - 1, l16);

  // pivots out; first zero / non-finite pivot reported through the flags
  if (wave == 0) {
    const T myd = tile[lane * LEAF_PAD + lane];
    const bool zero = myd == T(0);
    const bool finite = fabs((double)myd) <= 1.7976931348623157e308;
    const bool bad = lane < w && (zero || !finite || (spd != 0 && myd < T(0)));
    if (lane < w) {
      dvec[lane] = myd;
      dinv[lane] = spd != 0 ? T(1) / sqrt(myd) : fast_rcp(myd);
    }
    const unsigned long long mask = __ballot(bad);
    if (mask != 0ull) {
      const int first = __ffsll((long long)mask) - 1;
      if (lane == first) {
        unsigned long long idx = (unsigned long long)(pivot0 + first);
        unsigned long long old = atomicMin(&flags->first_bad, idx);
        if (idx <= old) atomicExch(&flags->bad_kind, zero ? 1ull : (!finite ? 2ull : 4ull));
      }
    }
  }
  // write back the last panel's columns (L below the diagonal, D on it); wavefront 3
  // is busy with the last inverse
  if (wave < 3) {
    constexpr int DONE = (NSUB - 1) * SUB;
    for (int e = tid; e < LEAF * SUB; e += 192) {
      const int r = e / SUB, c = DONE + e % SUB;
      if (r < w && c <= r) A[(int64_t)r * ld + c] = tile[r * LEAF_PAD + c];
    }
  }
  __builtin_amdgcn_s_setprio(0);
}

template <typename T>
__global__ __launch_bounds__(FACTOR_THREADS) void leaf_factor_kernel(
    T* __restrict__ A, int64_t ld, int w, T* __restrict__ dvec, T* __restrict__ dinv,
    T* __restrict__ linv, long long pivot0, DevFlags* flags, int spd) {
  __shared__ T lds[FACTOR_LDS_ELEMS];
  leaf_factor_body<T>(A, ld, w, dvec, dinv, linv, pivot0, flags, lds, spd);
}

// ---------------------------------------------------------------------------
// leaf factor with pivoting
// ---------------------------------------------------------------------------
// Maximum of x over the 64 lanes, delivered in a scalar register: four exchanges inside
// each row of 16 lanes on the data-parallel-primitive path, then the last lane of a row
// handed to the next row, and the last lane of the first two rows to the last two; lane
// 63 then holds the maximum.  Must be reached by all 64 lanes.
__device__ __forceinline__ unsigned wave_max_u32(unsigned x) {
  int m = (int)x;
  auto take = [&](int other) { m = (int)max((unsigned)m, (unsigned)other); };
  take(__builtin_amdgcn_update_dpp(0, m, 0xB1, 0xF, 0xF, false));    // lanes 1 0 3 2 of each four
  take(__builtin_amdgcn_update_dpp(0, m, 0x4E, 0xF, 0xF, false));    // lanes 2 3 0 1
  take(__builtin_amdgcn_update_dpp(0, m, 0x141, 0xF, 0xF, false));   // mirror inside each eight
  take(__builtin_amdgcn_update_dpp(0, m, 0x140, 0xF, 0xF, false));   // mirror inside each sixteen
  take(__builtin_amdgcn_update_dpp(m, m, 0x142, 0xA, 0xF, false));   // lane 15 -> rows 1 and 3
  take(__builtin_amdgcn_update_dpp(m, m, 0x143, 0xC, 0xF, false));   // lane 31 -> rows 2 and 3
  return (unsigned)__builtin_amdgcn_readlane(m, 63);
}

// The pivot rule: among the lanes with `candidate` set, the one whose `diag` is largest in
// magnitude (the lowest lane on ties; a NaN counts as the largest, so that it is taken
// and reported).  Magnitudes of IEEE numbers order like their bit patterns.  Returns 0 if
// there is no candidate.  Must be reached by all 64 lanes.
__device__ __forceinline__ int pick_pivot(double diag, bool candidate) {
  unsigned long long key = (unsigned long long)__double_as_longlong(fabs(diag));
  if (!(diag == diag)) key = 0x7ff0000000000000ull;
  if (!candidate) key = 0ull;
  const unsigned hi = (unsigned)(key >> 32), lo = (unsigned)key;
  const unsigned top_hi = wave_max_u32(hi);
  unsigned long long hit = __ballot(candidate && hi == top_hi);
  // the upper words (exponent, 20 bits of the fraction) nearly always decide
  if (hit & (hit - 1ull)) {
    const unsigned top_lo = wave_max_u32(hi == top_hi ? lo : 0u);
    hit = __ballot(candidate && hi == top_hi && lo == top_lo);
  }
  return hit ? __ffsll((long long)hit) - 1 : 0;
}
__device__ __forceinline__ int pick_pivot(float diag, bool candidate) {
  unsigned key = (unsigned)__float_as_int(fabsf(diag));
  if (!(diag == diag)) key = 0x7f800000u;
  if (!candidate) key = 0u;
  const unsigned top = wave_max_u32(key);
  const unsigned long long hit = __ballot(candidate && key == top);
  return hit ? __ffsll((long long)hit) - 1 : 0;
}

// a[idx] for an index that is the same in all lanes, without a memory round trip: four
// levels of two-way selects on the bits of idx.  Written as C++ conditionals the
// compiler recognises an indexed array, moves the array to scratch memory and stores
// all of it every time it changes; the select instruction itself keeps the 16 values
// in the registers they live in.
__device__ __forceinline__ int select_word(int x0, int x1, unsigned long long take1) {
  int r;
  asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(x0), "v"(x1), "s"(take1));
  return r;
}
__device__ __forceinline__ double select_value(double x0, double x1, unsigned long long take1) {
  return __hiloint2double(select_word(__double2hiint(x0), __double2hiint(x1), take1),
                          select_word(__double2loint(x0), __double2loint(x1), take1));
}
__device__ __forceinline__ float select_value(float x0, float x1, unsigned long long take1) {
  return __int_as_float(select_word(__float_as_int(x0), __float_as_int(x1), take1));
}
template <typename T>
__device__ __forceinline__ T select16(const T (&a)[SUB], int idx) {
  const unsigned long long b0 = (idx & 1) ? ~0ull : 0ull, b1 = (idx & 2) ? ~0ull : 0ull;
  const unsigned long long b2 = (idx & 4) ? ~0ull : 0ull, b3 = (idx & 8) ? ~0ull : 0ull;
  T t8[8], t4[4], t2[2];
#pragma unroll
  for (int k = 0; k < 8; ++k) t8[k] = select_value(a[2 * k], a[2 * k + 1], b0);
#pragma unroll
  for (int k = 0; k < 4; ++k) t4[k] = select_value(t8[2 * k], t8[2 * k + 1], b1);
#pragma unroll
  for (int k = 0; k < 2; ++k) t2[k] = select_value(t4[2 * k], t4[2 * k + 1], b2);
  return select_value(t2[0], t2[1], b3);
}

// One leaf, P A P^T = L D L^T with P chosen inside the leaf: at every step the largest
// remaining diagonal entry of the Schur complement is the pivot.  Nothing is swapped
// while the elimination runs.  The leaf is held as a full symmetric matrix, column c in
// lane c of each of the four wavefronts, wavefront q holding rows 16 q .. 16 q + 15 in
// registers.  Step j, pivot p: row p is one register of wavefront p / 16, a value per
// lane, and goes to LDS in one store; from there every lane reads w_c, its own column's
// entry, and the entries w_r of its wavefront's 16 rows (row p is column p, by symmetry);
// l_r = w_r / d; a_rc -= l_r w_c.  The chain from one step to the next is short: the pivot
// d itself comes from the owner lane's register before the exchange, so its reciprocal
// is ready when w_c arrives; then one product and one fused multiply-add give the lane's
// new diagonal entry, which every wavefront keeps with the same arithmetic as the
// entry in the matrix, so that each finds the next pivot by itself and no decision is
// exchanged.  The multipliers are collected by original row; once every row knows the
// step at which it was taken they move to that row of the result.  Rows and columns of
// pivots already taken keep being updated with values that nothing reads.
// Outputs as leaf_factor_kernel (L and D in pivot order into A, pivots, reciprocals,
// inverses of the diagonal sub-blocks of L), and perm[j] = pivot0 + (row taken at step j).
template <typename T>
__global__ __launch_bounds__(FACTOR_THREADS) void leaf_factor_pivoted_kernel(
    T* __restrict__ A, int64_t ld, int w, T* __restrict__ dvec, T* __restrict__ dinv,
    T* __restrict__ linv, int* __restrict__ perm, long long pivot0, DevFlags* flags) {
  __shared__ T tile[FACTOR_LDS_ELEMS];
  __shared__ T prow[2][LEAF];     // the pivot row, two steps alternating
  __shared__ T dl[LEAF];          // pivots in the order taken
  __shared__ int pos[LEAF];       // step at which a row was taken
  __shared__ int src[LEAF];       // row taken at a step
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15;
  constexpr int PER = LEAF * LEAF / FACTOR_THREADS;
  {
    T v[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = q * FACTOR_THREADS + tid, r = e >> 6, c = e & 63;
      v[q] = (r < w && c <= r) ? A[(int64_t)r * ld + c] : T(0);
    }
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = q * FACTOR_THREADS + tid, r = e >> 6, c = e & 63;
      tile[r * LEAF_PAD + c] = v[q];
    }
  }
  __syncthreads();
  T a[SUB];        // a[k] = entry (16 wave + k, lane)
#pragma unroll
  for (int k = 0; k < SUB; ++k) {
    const int r = wave * SUB + k;
    a[k] = lane <= r ? tile[r * LEAF_PAD + lane] : tile[lane * LEAF_PAD + r];
  }
  T diag = tile[lane * LEAF_PAD + lane];
  __syncthreads();
  for (int e = tid; e < FACTOR_LDS_ELEMS; e += FACTOR_THREADS) tile[e] = T(0);
  if (wave == 0) {
    pos[lane] = lane;      // rows of the padding (w < 64) stay where they are
    src[lane] = lane;
    dl[lane] = T(1);
  }
  bool taken = lane >= w;
  int p = pick_pivot(diag, !taken);
#pragma unroll 1
  for (int j = 0; j < w; ++j) {
    T* pr = prow[j & 1];
    if (wave == (p >> 4)) pr[lane] = select16<T>(a, p & 15);
    const T d = lane_value(diag, p);
    const T rd = fast_rcp(d);
    // also orders the clearing of the tile before the first multiplier written to it
    __syncthreads();
    const T wc = pr[lane];
    T wr[SUB];
#pragma unroll
    for (int k = 0; k < SUB; ++k) wr[k] = pr[wave * SUB + k];
    const bool live = !taken && lane != p;
    const T lc = live ? wc * rd : T(0);
    diag = fma(-lc, wc, diag);      // the same operands as this column's diagonal entry in a[]
    if (wave == 0) {
      if (live) tile[lane * LEAF_PAD + j] = lc;
      if (lane == p) {
        pos[lane] = j;
        src[j] = lane;
        dl[j] = d;
      }
    }
    if (lane == p) taken = true;
    p = pick_pivot(diag, !taken);
#pragma unroll
    for (int k = 0; k < SUB; ++k) a[k] = fma(-(wr[k] * rd), wc, a[k]);
  }
  __syncthreads();
  // rows into the order in which they were taken; row r has multipliers in columns < pos[r]
  {
    T v[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) v[q] = tile[((q * FACTOR_THREADS + tid) >> 6) * LEAF_PAD + (tid & 63)];
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int r = (q * FACTOR_THREADS + tid) >> 6, c = tid & 63, to = pos[r];
      tile[to * LEAF_PAD + c] = c == to ? dl[to] : v[q];
    }
  }
  __syncthreads();
  for (int e = tid; e < LEAF * LEAF; e += FACTOR_THREADS) {
    const int r = e >> 6, c = e & 63;
    if (r < w && c <= r) A[(int64_t)r * ld + c] = tile[r * LEAF_PAD + c];
  }
  leaf_invert_sub<T>(tile, linv, wave, l16);
  if (wave == 0) {
    const T myd = dl[lane];
    const bool zero = myd == T(0);
    const bool finite = fabs((double)myd) <= 1.7976931348623157e308;
    const bool bad = lane < w && (zero || !finite);
    if (lane < w) {
      dvec[lane] = myd;
      dinv[lane] = fast_rcp(myd);
      perm[lane] = (int)pivot0 + src[lane];
    }
    const unsigned long long mask = __ballot(bad);
    if (mask != 0ull) {
      const int first = __ffsll((long long)mask) - 1;
      if (lane == first) {
        unsigned long long idx = (unsigned long long)(pivot0 + first);
        unsigned long long old = atomicMin(&flags->first_bad, idx);
        if (idx <= old) atomicExch(&flags->bad_kind, zero ? 1ull : 2ull);
      }
    }
  }
  __builtin_amdgcn_s_setprio(0);
}

// ---------------------------------------------------------------------------
// leaf factor, general matrix
// ---------------------------------------------------------------------------
// The library keeps a general matrix as two lower-triangular arrays of the same shape:
// Pl holds the entries on and below the diagonal, Qu the entries above it, transposed
// (Qu[i][j] = M[j][i], i > j), so that both halves of every block row and column are read
// along rows, as the update and solve kernels want their operands.  This kernel factors
// one <= 64 x 64 diagonal leaf, given as its two halves: P A = L D U by Gaussian
// elimination with the pivot of column j taken among the leaf's rows not taken before
// (largest magnitude; the lowest row of the input on ties).  Rows stay where they are
// while the elimination runs: lane r of every wavefront holds row r, wavefront q its
// columns 16q .. 16q+15, in registers.  At step j the wavefront that owns column j picks
// the pivot row and hands the multipliers and the row's number to the others through LDS
// (one barrier per step); each wavefront then reads the pivot row's entries of its own
// columns from the pivot lane's registers.  The rows are put into the order of their
// choice at the end.  On return Pl holds L below the diagonal and D on it, Qu holds U^T
// (strictly lower, unit diagonal implied), dvec / dinv the pivots and their reciprocals,
// linvL / linvU the inverses of the 16 x 16 diagonal sub-blocks of L and of U^T (for
// leaf_solve_kernel: rows below in Pl are solved against U^T, rows below in Qu against L
// with the leaf's row order as their column gather), perm[j] = pivot0 + (row of the leaf
// taken at step j); flags->odd_leaves is raised by one if that order is an odd permutation.
// NW wavefronts (4, 8 or 16): wavefront q holds columns q CW .. q CW + CW - 1, CW = 64 / NW.
// A step costs its wavefront about 60 clocks per column held (two v_readlane of about 20
// clocks each, the multiply-add and the live-row select), which is most of the step with
// 16 columns; 16 wavefronts of 4 columns each spread that over the compute unit's SIMDs.
constexpr int LU_WAVES = 16;   // n = 8192 as a general matrix: 15.02 ms with 4, 13.97 with 8, 13.56 with 16
template <typename T, int NW>
__global__ __launch_bounds__(64 * NW) void leaf_lu_kernel(
    T* __restrict__ Pl, T* __restrict__ Qu, int64_t ld, int w, T* __restrict__ dvec,
    T* __restrict__ dinv, T* __restrict__ linvL, T* __restrict__ linvU, int* __restrict__ perm,
    long long pivot0, DevFlags* flags) {
  constexpr int CW = LEAF / NW;          // columns per wavefront
  constexpr int NT = 64 * NW;            // threads
  __shared__ T S[FACTOR_LDS_ELEMS];      // the rows in their final order: L below, D U on and above
  __shared__ T Lm[FACTOR_LDS_ELEMS];     // multipliers by input row; afterwards U^T
  __shared__ T lbuf[2][LEAF];            // a step's multipliers, for the other wavefronts
  __shared__ int pbuf[2];                // and its pivot row
  __shared__ int ord[LEAF];
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15;
  const int c0 = wave * CW;
  constexpr int PER = LEAF * LEAF / NT;
  T a[CW];
#pragma unroll
  for (int k = 0; k < CW; ++k) {
    // (r, c) of the lower half and (c, r) of the upper half come from the same place of
    // the two arrays: row max(r, c), column min(r, c)
    const int r = lane, c = c0 + k;
    const int hi = r > c ? r : c, lo = r > c ? c : r;
    a[k] = (r < w && c < w) ? (c <= r ? Pl[(int64_t)hi * ld + lo] : Qu[(int64_t)hi * ld + lo])
                            : (r == c ? T(1) : T(0));
  }
#pragma unroll
  for (int q = 0; q < PER; ++q) Lm[((q * NT + tid) >> 6) * LEAF_PAD + (tid & 63)] = T(0);
  if (tid < LEAF) ord[tid] = tid;
  __syncthreads();                            // Lm is clear before the first multiplier lands in it
  unsigned long long taken = 0ull;            // the same in every lane and wavefront
  int mypos = lane;                           // where this lane's row ends
#pragma unroll 1
  for (int jb = 0; jb < NW; ++jb) {
#pragma unroll
    for (int jj = 0; jj < CW; ++jj) {
      const int j = jb * CW + jj;
      if (j < w) {
        if (wave == jb) {
          const T cj = a[jj];
          const bool cand = lane < w && !((taken >> lane) & 1ull);
          const int pp = pick_pivot(cj, cand);
          const T rd = fast_rcp(lane_value(cj, pp));
          const T lj = (cand && lane != pp) ? cj * rd : T(0);
          lbuf[j & 1][lane] = lj;
          Lm[lane * LEAF_PAD + j] = lj;
          if (lane == 0) {
            pbuf[j & 1] = pp;
            ord[j] = pp;
          }
        }
        __syncthreads();
        const T l = lbuf[j & 1][lane];
        const int p = __builtin_amdgcn_readfirstlane(pbuf[j & 1]);
        taken |= 1ull << p;
        if (lane == p) mypos = j;
        const bool live = lane < w && !((taken >> lane) & 1ull);
        if (wave >= jb) {
#pragma unroll
          for (int k = 0; k < CW; ++k) {
            if (wave > jb || k > jj) {
              const T pv = lane_value(a[k], p);
              a[k] = live ? fma(-l, pv, a[k]) : a[k];
            }
          }
        }
      }
    }
  }
  // every row to the place of its turn; its entries left of the diagonal are replaced below
#pragma unroll
  for (int k = 0; k < CW; ++k) S[mypos * LEAF_PAD + c0 + k] = a[k];
  __syncthreads();
  {
    T v[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = q * NT + tid, r = e >> 6, c = e & 63;
      const int from = r < w ? ord[r] : r;
      v[q] = c < r ? Lm[from * LEAF_PAD + c] : S[r * LEAF_PAD + c];
    }
    __syncthreads();
    // L into place; U = D U~: rows of the upper part divided by their pivot, and its
    // transpose with a unit diagonal
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = q * NT + tid, r = e >> 6, c = e & 63;
      if (c < r) S[r * LEAF_PAD + c] = v[q];
      T u = r == c ? T(1) : T(0);
      if (c > r && c < w) u = v[q] * fast_rcp(S[r * LEAF_PAD + r]);
      if (c >= r) Lm[c * LEAF_PAD + r] = u;
    }
  }
  __syncthreads();
  for (int e = tid; e < LEAF * LEAF; e += NT) {
    const int r = e >> 6, c = e & 63;
    if (r < w && c <= r) Pl[(int64_t)r * ld + c] = S[r * LEAF_PAD + c];
    if (r < w && c < r) Qu[(int64_t)r * ld + c] = Lm[r * LEAF_PAD + c];
  }
  if (wave < NSUB) {
    leaf_invert_sub<T>(S, linvL, wave, l16);
    leaf_invert_sub<T>(Lm, linvU, wave, l16);
  }
  if (wave == 0) {
    const T myd = S[lane * LEAF_PAD + lane];
    const bool zero = myd == T(0);
    const bool finite = fabs((double)myd) <= 1.7976931348623157e308;
    const bool bad = lane < w && (zero || !finite);
    const int mine = ord[lane];
    if (lane < w) {
      dvec[lane] = myd;
      dinv[lane] = fast_rcp(myd);
      perm[lane] = (int)pivot0 + mine;
    }
    // sign of the order: parity of the number of pairs that stand the wrong way round
    int inv = 0;
    for (int k = 0; k < LEAF; ++k) inv += (k > lane && ord[k] < mine) ? 1 : 0;
    const unsigned long long odd_lanes = __ballot(inv & 1);
    if (lane == 0 && (__popcll(odd_lanes) & 1)) atomicAdd(&flags->odd_leaves, 1ull);
    const unsigned long long mask = __ballot(bad);
    if (mask != 0ull) {
      const int first = __ffsll((long long)mask) - 1;
      if (lane == first) {
        unsigned long long idx = (unsigned long long)(pivot0 + first);
        unsigned long long old = atomicMin(&flags->first_bad, idx);
        if (idx <= old) atomicExch(&flags->bad_kind, zero ? 1ull : 2ull);
      }
    }
  }
  __builtin_amdgcn_s_setprio(0);
}

// Moves the strict upper triangle of a general matrix into its transposed store, or back,
// by 64 x 64 blocks through LDS (both arrays n x n with leading dimension ld).
// back = 0: dst[i][j] = src[j][i] for i > j;  back = 1: dst[j][i] = src[i][j] for i > j.
// Workgroup b handles the block pair (bi, bj), bi >= bj, of the lower triangle.
template <typename T>
__global__ __launch_bounds__(256) void transpose_strict_kernel(const T* __restrict__ src,
                                                               T* __restrict__ dst, int64_t ld,
                                                               int64_t n, int nb, int back) {
  __shared__ T t[LEAF * LEAF_PAD];
  const int64_t b = blockIdx.x;
  int64_t bi = (int64_t)((sqrt(8.0 * (double)b + 1.0) - 1.0) * 0.5);
  while (bi * (bi + 1) / 2 > b) --bi;
  while ((bi + 1) * (bi + 2) / 2 <= b) ++bi;
  const int64_t bj = b - bi * (bi + 1) / 2;
  if (bi >= nb) return;
  // the block that is read and the block that is written: (row block, column block)
  const int64_t sr = back ? bi : bj, sc = back ? bj : bi;
  const int tid = threadIdx.x;
  for (int e = tid; e < LEAF * LEAF; e += 256) {
    const int r = e >> 6, c = e & 63;
    const int64_t gr = sr * LEAF + r, gc = sc * LEAF + c;
    t[r * LEAF_PAD + c] = (gr < n && gc < n) ? src[gr * ld + gc] : T(0);
  }
  __syncthreads();
  for (int e = tid; e < LEAF * LEAF; e += 256) {
    const int r = e >> 6, c = e & 63;                       // of the block written, (sc, sr)
    const int64_t gr = sc * LEAF + r, gc = sr * LEAF + c;
    const bool strict = back ? gc > gr : gr > gc;
    if (gr < n && gc < n && strict) dst[gr * ld + gc] = t[c * LEAF_PAD + r];
  }
}

// ---------------------------------------------------------------------------
// leaf solve
// ---------------------------------------------------------------------------
// Rows below a factored leaf: X (m x w, in place) <- X L^-T D^-1.
// 256 threads = 4 wavefronts, each owning 16 rows as four 16 x 16 sub-blocks held
// in MFMA accumulator layout.  Sub-block b:  T_b = X_b - sum_{p<b} W_p L[b,p]^T
// (products on the matrix cores, terms in the order p = 0, 1, ...), then
// W_b = T_b L_bb^-T with the inverse of the unit-lower diagonal sub-block prepared
// by the factor kernel, then L_b = W_b D_b^-1 goes back to memory.
// perm (or null): the leaf was factored with pivoting; perm[j] - perm0 is the column of
// the panel that belongs at position j.  A wavefront reads all 64 columns of its rows
// before it writes any of them.
// fix_src (or null): the launch has one workgroup more than its rows need, and that one
// copies the 64 x 64 row-major block at fix_src to fix_dst (leading dimension fix_ld), a
// block outside this launch's own rows and columns.
constexpr int SOLVE_ROWS = 64;   // rows per workgroup

template <typename T>
__device__ __forceinline__ void leaf_solve_body(
    T* __restrict__ Xg, int64_t ld, int m, int w, const T* __restrict__ Lleaf, int64_t ldl,
    const T* __restrict__ dinv, const T* __restrict__ linv, T* __restrict__ Wg, int64_t ldw,
    const T* __restrict__ dvec, int wfrom, const int* __restrict__ perm, int perm0,
    const T* __restrict__ fix_src, T* __restrict__ fix_dst, int64_t fix_ld) {
  using X = Mfma<T>;
  using acc_t = typename X::acc_t;
  // Only the sub-blocks L[b, p], p < b, and the solved W_p, p < NSUB - 1, are ever
  // multiplied: rows 16.. and columns ..47 of the leaf.  Keeping just those holds the
  // workgroup's LDS (60 KB in fp64) below that of a trailing-update workgroup, so
  // that it fits whichever half of a compute unit such a workgroup has just left.
  constexpr int LW = LEAF - SUB;                // rows of L kept = columns of L and W kept
  constexpr int LW_PAD = LW + 1;
  __shared__ T Ls[LW * LW_PAD];                 // L[16.., ..47], strictly lower part
  __shared__ T Li[NSUB * SUB * SUB_PAD];        // inverses of its diagonal sub-blocks
  __shared__ T rinv[LEAF];
  __shared__ T dsc[LEAF];                       // pivots (only read when Wg is given)
  __shared__ T wsc[4][SUB * LW_PAD];            // per wavefront: solved W, row-major
  __shared__ T tsc[4][SUB * SUB_PAD];           // per wavefront: layout change of T_b
  __builtin_amdgcn_s_setprio(2);                // on the chain of dependent launches
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;

  // a 64 x 64 block that an earlier launch left beside its place (leaf_pair_kernel): the
  // launch then has one workgroup more, which does only this
  if (fix_src != nullptr && blockIdx.x == gridDim.x - 1) {
    T v[LEAF * LEAF / 256];
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / 256; ++q) v[q] = fix_src[q * 256 + tid];
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / 256; ++q) {
      const int e = q * 256 + tid;
      fix_dst[(int64_t)(e >> 6) * fix_ld + (e & 63)] = v[q];
    }
    return;
  }
  // this wavefront's rows, straight into accumulator layout (16 lanes = 128 bytes of a row)
  const int64_t r0 = ((int64_t)blockIdx.x * 4 + wave) * SUB;
  acc_t xb[NSUB];
#pragma unroll
  for (int b = 0; b < NSUB; ++b)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t row = r0 + X::acc_row(lane, r);
      const int col = b * SUB + l16;
      // with a permutation of the leaf, column `col` of the result is the column that
      // was taken at that step
      const int from = (perm != nullptr && col < w) ? perm[col] - perm0 : col;
      xb[b][r] = (row < m && col < w) ? Xg[row * ld + from] : T(0);
    }
  // leaf data shared by the four wavefronts
  {
    T v[LEAF * LEAF / 256];
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / 256; ++q) {
      const int e = q * 256 + tid, r = e >> 6, c = e & 63;
      v[q] = (r < w && c < r) ? Lleaf[(int64_t)r * ldl + c] : T(0);
    }
    T u[NSUB * SUB * SUB / 256];
#pragma unroll
    for (int q = 0; q < NSUB * SUB * SUB / 256; ++q) u[q] = linv[q * 256 + tid];
    const T myr = (tid < LEAF && tid < w) ? dinv[tid < LEAF ? tid : 0] : T(0);
    const T myd = (Wg != nullptr && tid < LEAF && tid < w) ? dvec[tid < LEAF ? tid : 0] : T(0);
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / 256; ++q) {
      const int e = q * 256 + tid, r = e >> 6, c = e & 63;
      if (r >= SUB && c < LW) Ls[(r - SUB) * LW_PAD + c] = v[q];
    }
#pragma unroll
    for (int q = 0; q < NSUB * SUB * SUB / 256; ++q) {
      const int e = q * 256 + tid, blk = e >> 8, i = (e >> 4) & 15, k = e & 15;
      Li[(blk * SUB + i) * SUB_PAD + k] = u[q];
    }
    if (tid < LEAF) { rinv[tid] = myr; dsc[tid] = myd; }
  }
  __syncthreads();
  // with a permutation a store below may hit an entry that another lane of this wavefront
  // loads above: every load has returned before the first store is issued (free here:
  // the leaf data, requested after the rows, has already arrived)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  T* ws = wsc[wave];
  T* ts = tsc[wave];
#pragma unroll
  for (int b = 0; b < NSUB; ++b) {
    acc_t acc = xb[b];
    // T_b = X_b - sum_{p<b} W_p L[b,p]^T
#pragma unroll 1
    for (int p = 0; p < b; ++p) {
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        const int k = p * SUB + 4 * s4 + g;
        const T aop = -ws[l16 * LW_PAD + k];
        const T bop = Ls[((b - 1) * SUB + l16) * LW_PAD + k];
        acc = X::mfma(aop, bop, acc);
      }
    }
    // accumulator layout -> operand layout through LDS
#pragma unroll
    for (int r = 0; r < 4; ++r) ts[X::acc_row(lane, r) * SUB_PAD + l16] = acc[r];
    // (ts and ws belong to this wavefront alone, and a wavefront's LDS operations
    // complete in the order they were issued: no barrier between these steps)
    // W_b = T_b L_bb^-T
    acc_t wb = acc_t{0, 0, 0, 0};
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const int k = 4 * s4 + g;
      wb = X::mfma(ts[l16 * SUB_PAD + k], Li[(b * SUB + l16) * SUB_PAD + k], wb);
    }
    const T rj = rinv[b * SUB + l16];
    const T dj = dsc[b * SUB + l16];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row16 = X::acc_row(lane, r);
      if (b < NSUB - 1) ws[row16 * LW_PAD + b * SUB + l16] = wb[r];
      const int64_t row = r0 + row16;
      const int col = b * SUB + l16;
      if (row < m && col < w) {
        const T lv = wb[r] * rj;
        Xg[row * ld + col] = lv;
        if (Wg != nullptr && row >= wfrom) Wg[row * ldw + col] = lv * dj;
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void leaf_solve_kernel(
    T* __restrict__ Xg, int64_t ld, int m, int w, const T* __restrict__ Lleaf, int64_t ldl,
    const T* __restrict__ dinv, const T* __restrict__ linv, T* __restrict__ Wg, int64_t ldw,
    const T* __restrict__ dvec, int wfrom, const int* __restrict__ perm, int perm0,
    const T* __restrict__ fix_src, T* __restrict__ fix_dst, int64_t fix_ld) {
  leaf_solve_body<T>(Xg, ld, m, w, Lleaf, ldl, dinv, linv, Wg, ldw, dvec, wfrom, perm, perm0, fix_src, fix_dst,
                     fix_ld);
}

// The rows below a leaf of a general matrix, both halves in one launch with two rows of
// workgroups: blockIdx.y = 0 solves the rows of the lower half (Xg) against U^T (the leaf's
// place in the second array, qoff elements on) with linvU; blockIdx.y = 1 the rows of the
// transposed upper half (Xg + qoff) against L (Lleaf) with linvL, their columns gathered
// in the leaf's row order (perm, perm0 as in leaf_solve_kernel).
template <typename T>
__global__ __launch_bounds__(256) void leaf_solve_general_kernel(
    T* Xg, int64_t ld, int m, int w, const T* Lleaf, const T* __restrict__ dinv,
    const T* __restrict__ linvL, const T* __restrict__ linvU, const T* __restrict__ dvec,
    const int* __restrict__ perm, int perm0, int64_t qoff) {
  const bool upper = blockIdx.y != 0;
  leaf_solve_body<T>(upper ? Xg + qoff : Xg, ld, m, w, upper ? Lleaf : Lleaf + qoff, ld, dinv,
                     upper ? linvL : linvU, (T*)nullptr, (int64_t)0, dvec, 0,
                     upper ? perm : (const int*)nullptr, perm0, (const T*)nullptr, (T*)nullptr, (int64_t)0);
}

}  // namespace mdet
