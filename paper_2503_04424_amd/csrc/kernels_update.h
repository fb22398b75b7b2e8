// Trailing Schur-complement update on the matrix cores.
//
// Sec. 2.2 of the paper forms S <- S - C B for every block of the trailing matrix
// (App. E.1 counts it as "full" and "Gramian" matrix multiplications); in the
// LDL^T case the product carries the diagonal scaling:
//
//      C[M x N]  -=  A[M x K] * diag(d[0..K)) * B[N x K]^T
//
// with A and B rows of the already-factored block column (unit-lower factor L)
// and d its pivots.  All three matrices are row-major, so both operands are read
// along K with unit stride.
//
// Tiling (gfx950): 256 threads = 4 wavefronts in a 2 x 2 arrangement, each
// wavefront owns a 64 x 64 piece of a 128 x 128 block of C as 4 x 4 MFMA tiles of
// 16 x 16 (v_mfma_f64_16x16x4_f64 / v_mfma_f32_16x16x4_f32).  K is walked in
// slabs of 128 bytes per row (16 doubles / 32 floats) that go from global memory
// straight into LDS, double buffered, the next slab's loads in flight while the
// current one is multiplied.  The scaling by -d is applied to the A fragments as
// they are read from LDS; the accumulators are seeded with C.
//
// Also here, because they end with the same hand-over of the next leaf:
// leaf_update_kernel (K = 64, one shot from LDS) and leaf_pair_kernel (a leaf's solve,
// the K = 64 update by it and the next leaf's factorisation in one launch).
//
// The *_general_kernel names run the same bodies for a general matrix (Sec. 2.2, Eq. 1:
// M = P L U) kept as two lower-triangular arrays, one row of workgroups per array.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "kernels_leaf.h"
#include "mfma.h"

namespace mdet {

constexpr int UPD_THREADS = 256;

// Block scheduling.  The C blocks of a launch are grouped into 8 x 8 "super-tiles"
// (64 blocks that share 8 row strips of A and 8 row strips of B) and numbered
// super-tile by super-tile; of a lower-triangular launch only the blocks on or
// below the diagonal get a number (36 of a super-tile on the diagonal).
// Workgroups are dispatched round-robin over the 8 XCDs by linear id, each XCD
// with its own L2; the map below hands every XCD a contiguous range of block
// numbers, so the 64 or so blocks an XCD runs at one time re-use each operand
// strip eight times out of its L2 instead of fetching it once per block.  Numbers
// that fall outside a ragged edge exit at once.  A launch at most four blocks wide
// (the updates inside a block column) has no use for super-tiles: its blocks are
// numbered row by row.
//
// A launch may cover only part of the numbers: workgroup id takes number
// xcd * per + k0 + (id >> 3) with xcd = id & 7, so that a sequence of launches with
// growing k0 walks every XCD's range in order (used to keep part of the device
// free for the kernels of another stream).
constexpr int UPD_SUPER = 8;
constexpr int UPD_SUPER_LOG2 = 3;
constexpr int UPD_SUPER_TRI = UPD_SUPER * (UPD_SUPER + 1) / 2;   // blocks of a diagonal super-tile

struct UpdGrid {
  int64_t per;       // block numbers per XCD; a full launch has 8 * per workgroups
  int nsn;           // super-tile columns (super-tile mode)
  int swl;           // 3: 8 x 8 super-tiles; 0..2: rows of 1 << swl blocks, no super-tiles
};
static inline UpdGrid update_grid(int64_t M, int64_t N, bool lower, int tile) {
  int64_t nbm = (M + tile - 1) / tile, nbn = (N + tile - 1) / tile;
  UpdGrid g;
  int64_t count;
  if (nbn <= 4) {
    g.swl = nbn <= 1 ? 0 : (nbn <= 2 ? 1 : 2);
    g.nsn = 1;
    count = nbm << g.swl;
  } else {
    g.swl = UPD_SUPER_LOG2;
    const int64_t nsm = (nbm + UPD_SUPER - 1) / UPD_SUPER;
    g.nsn = (int)((nbn + UPD_SUPER - 1) / UPD_SUPER);
    if (!lower) count = nsm * g.nsn * 64;
    else {
      const int64_t t = nsm < g.nsn ? nsm : g.nsn;      // super-tile rows that reach the diagonal
      count = 32 * t * t + 4 * t + (nsm - t) * g.nsn * 64;
    }
  }
  g.per = (count + 7) / 8;
  return g;
}

// (bm, bn) of block number t, or false if there is no such block.  Number 0 is
// block (0, 0).
__host__ __device__ __forceinline__ bool update_block_of_number(const bool lower, const int64_t t, int nbm,
                                                       int nbn, int nsn, int swl, int& bm, int& bn) {
  if (swl < UPD_SUPER_LOG2) {
    bm = (int)(t >> swl);
    bn = (int)(t & ((1 << swl) - 1));
    return bm < nbm && bn < nbn && (!lower || bn <= bm);
  }
  if (!lower) {
    const int64_t st = t >> 6;
    const int loc = (int)(t & 63);
    bm = (int)(st / nsn) * UPD_SUPER + (loc >> 3);
    bn = (int)(st % nsn) * UPD_SUPER + (loc & 7);
    return bm < nbm && bn < nbn;
  }
  // super-tile row r < nsn holds r full super-tiles and the diagonal one:
  // 64 r + 36 blocks, 32 r^2 + 4 r before it
  const int64_t tri_total = 32 * (int64_t)nsn * nsn + 4 * (int64_t)nsn;
  if (t < tri_total) {
    int64_t r = (int64_t)((sqrt(16.0 + 128.0 * (double)t) - 4.0) * (1.0 / 64.0));
    while (32 * r * r + 4 * r > t) --r;
    while (32 * (r + 1) * (r + 1) + 4 * (r + 1) <= t) ++r;
    const int64_t u = t - (32 * r * r + 4 * r);
    if (u < 64 * r) {
      const int loc = (int)(u & 63);
      bm = (int)r * UPD_SUPER + (loc >> 3);
      bn = (int)(u >> 6) * UPD_SUPER + (loc & 7);
    } else {
      const int v = (int)(u - 64 * r);               // 0 .. 35, row by row of the triangle
      int i = (int)((sqrtf(8.0f * (float)v + 1.0f) - 1.0f) * 0.5f);
      while (i * (i + 1) / 2 > v) --i;
      while ((i + 1) * (i + 2) / 2 <= v) ++i;
      bm = (int)r * UPD_SUPER + i;
      bn = (int)r * UPD_SUPER + (v - i * (i + 1) / 2);
    }
  } else {
    const int64_t u = t - tri_total;
    const int64_t row = u / (64 * (int64_t)nsn), w = u % (64 * (int64_t)nsn);
    const int loc = (int)(w & 63);
    bm = (nsn + (int)row) * UPD_SUPER + (loc >> 3);
    bn = (int)(w >> 6) * UPD_SUPER + (loc & 7);
  }
  return bm < nbm && bn < nbn && bn <= bm;
}

// Block of workgroup `id` in a launch that starts at the k0-th number of every
// XCD's range of `per` numbers.
__device__ __forceinline__ bool update_block_of(const bool lower, int64_t id, int64_t per, int64_t k0,
                                                int nbm, int nbn, int nsn, int swl, int& bm, int& bn) {
  const int xcd = (int)(id & 7);
  const int64_t k = k0 + (id >> 3);
  if (k >= per) return false;
  return update_block_of_number(lower, (int64_t)xcd * per + k, nbm, nbn, nsn, swl, bm, bn);
}

// Optional tail of a lower-triangular launch: the factorisation of the leaf that starts at
// C's top-left corner (w = 0: none), done by the workgroup that reduced that
// block.  Pointers as for leaf_factor_kernel.
template <typename T>
struct FusedLeaf {
  int w;
  T* dvec;
  T* dinv;
  T* linv;
  long long pivot0;
  DevFlags* flags;
  int spd;   // positive-definite form (see leaf_factor_body)
};

// TM = MFMA tiles per wavefront in each direction: 4 -> 128 x 128 block, 2 -> 64 x 64.
template <typename T, int TM>
struct UpdShape {
  using X = Mfma<T>;
  static constexpr int BK = X::BK;                                // K elements per slab: 128 bytes a row
  static constexpr int BM = 32 * TM, BN = 32 * TM;                // block of C per workgroup
  static constexpr int SLAB_ELEMS = 2 * (BM + BN) * BK;           // both operands, double buffered
  static constexpr int LDS_ELEMS = SLAB_ELEMS > FACTOR_LDS_ELEMS ? SLAB_ELEMS : FACTOR_LDS_ELEMS;
};

typedef __attribute__((address_space(1))) const void* upd_global_ptr;
typedef __attribute__((address_space(3))) void* upd_lds_ptr;

// One block (bm, bn) of C, by all threads of the workgroup; `lds` = LDS_ELEMS
// elements.  Every thread returns from it (there are barriers inside), so a
// workgroup may call it for one block after another.
//
// Staging.  A slab is 128 bytes of K per operand row.  It goes from global memory
// straight into LDS (global_load_lds_dwordx4: every lane names its own 16 global
// bytes, and lane l's land at the wavefront's LDS base + 16 l), so it needs no
// staging registers, no LDS store instructions and no wait before the end of the
// slab.  One such load fills 1 KB = 8 rows; a workgroup's four wavefronts issue
// BM/32 of them per operand and slab.  Rows are 128 bytes apart in LDS without
// padding; instead the eight 16-byte chunks of row r are stored in the order
// chunk ^ ((r >> 1) & 7), which a lane arranges by choosing what it loads.  The
// 16 lanes that fetch one MFMA operand (16 consecutive rows, same logical chunk)
// then hit 16 different bank groups.  The scaling by -d is applied to the A
// fragments as they come out of LDS (the same single rounding of a * (-d) as if
// it were applied on the way in).
//
// SCALED: C -= A B^T with operands that carry the diagonal scaling already (rows of
// the Cholesky factor, or a left operand L D): no pivots are read and no fragment is
// scaled.
// In both forms the accumulators start from -C, collect +A D B^T and are negated on
// the way out, which rounds exactly like C - A D B^T term by term and needs neither a
// negated operand nor a negated pivot.
template <typename T, int TM, bool SCALED = false>
__device__ __forceinline__ void schur_update_block(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int K,
    const bool lower, const int bm, const int bn, const FusedLeaf<T>& fl, T* __restrict__ lds) {
  using X = Mfma<T>;
  using acc_t = typename X::acc_t;
  using vec_t = typename X::vec_t;
  constexpr int BK = X::BK, VEC = X::VEC;
  static_assert(BK * sizeof(T) == 128 && VEC * sizeof(T) == 16, "a slab row is eight 16-byte chunks");
  constexpr int WT = 16 * TM;                         // rows/cols of C per wavefront
  constexpr int BM = 2 * WT, BN = 2 * WT;             // block of C per workgroup
  constexpr int NV = BM / 32;                         // 1 KB loads per wavefront, operand and slab
  constexpr int KS = BK / 4;                          // MFMA k-steps per slab (= 2 chunks a lane)
  static_assert(KS == 2 * VEC, "a lane's share of a slab row is two chunks");

  T (*As)[BM * BK] = reinterpret_cast<T (*)[BM * BK]>(lds);
  T (*Bs)[BN * BK] = reinterpret_cast<T (*)[BN * BK]>(lds + 2 * BM * BK);

  const int row0 = bm * BM, col0 = bn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // a wavefront whose 64 x 64 piece lies strictly above the diagonal has nothing to do
  const bool active = !(lower && (row0 + wm * WT + WT - 1 < col0 + wn * WT));

  // ---- global -> LDS staging --------------------------------------------
  // Load v of a wavefront covers rows 8 * (4 v + wave) .. + 7 of the block; lane l
  // brings physical chunk l & 7 of row l >> 3, i.e. logical chunk (l & 7) ^ swizzle.
  // Addresses: a base common to the workgroup (scalar registers; moves along K) plus
  // a 32-bit byte offset per lane and load that is fixed for the whole block (row
  // clamped at the ragged edge included).  The host checks that 128 rows of either
  // operand span less than 4 GiB.
  const char* Abase = reinterpret_cast<const char*>(A + (int64_t)row0 * lda);
  const char* Bbase = reinterpret_cast<const char*>(B + (int64_t)col0 * ldb);
  unsigned aoff[NV], boff[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int rt = 8 * (4 * v + wave) + (lane >> 3);          // row within the block
    const int chunk = (lane & 7) ^ ((rt >> 1) & 7);           // logical 16-byte chunk this lane brings
    int ar = rt; if (row0 + ar > M - 1) ar = M - 1 - row0;
    int br = rt; if (col0 + br > N - 1) br = N - 1 - col0;
    aoff[v] = (unsigned)(((int64_t)ar * lda + chunk * VEC) * (int64_t)sizeof(T));
    boff[v] = (unsigned)(((int64_t)br * ldb + chunk * VEC) * (int64_t)sizeof(T));
  }
  // Two nudges keep these loads in the "scalar base + 32-bit vector offset" form
  // inside the K loop, instead of one 64-bit induction pointer per lane and load:
  // the slab's byte offset goes through readfirstlane (it is uniform anyway), and
  // the per-lane offset through an empty asm, so that its widening is not hoisted
  // out of the loop.
  auto pinned = [](unsigned o) { asm volatile("" : "+v"(o)); return o; };
  auto gload = [&](int kt, int buf) {
    const unsigned kb = __builtin_amdgcn_readfirstlane((unsigned)kt * (unsigned)(BK * sizeof(T)));
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int blk = __builtin_amdgcn_readfirstlane(4 * v + wave);
      __builtin_amdgcn_global_load_lds((upd_global_ptr)(Abase + kb + pinned(aoff[v])),
                                       (upd_lds_ptr)(&As[buf][blk * 8 * BK]), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((upd_global_ptr)(Bbase + kb + pinned(boff[v])),
                                       (upd_lds_ptr)(&Bs[buf][blk * 8 * BK]), 16, 0, 0);
    }
  };
  // all of this wavefront's loads have landed (the barrier that follows publishes them)
  auto landed = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

  const int r16 = lane & 15, g = lane >> 4;

  // The accumulators start from (minus) C and the products are added to them in
  // K order, so every entry is reduced term by term exactly as in the unblocked
  // recurrence a_ij - sum_k l_ik d_k l_jk; when the Schur complement is much
  // smaller than a_ij (low-rank Gram matrix plus a small shift) the late roundings
  // are then relative to the small running value, not to the full sum.
  acc_t acc[TM][TM];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j) acc[i][j] = acc_t{0, 0, 0, 0};
  if (active) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int grow = row0 + wm * WT + i * 16 + X::acc_row(lane, r);
        if (grow >= M) continue;
        const T* crow = C + (int64_t)grow * ldc;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          const int gcol = col0 + wn * WT + j * 16 + r16;
          if (gcol < N && (!lower || gcol <= grow)) acc[i][j][r] = crow[gcol];
        }
      }
    }
  }

  const int nk = K / BK;

  // lane group g owns the KS consecutive k's [g*KS, (g+1)*KS) of a slab, i.e. its
  // logical chunks 2g and 2g+1; MFMA step s multiplies the s-th of them from every
  // group (any assignment of the slab's k's to steps is valid as long as A and B
  // use the same one).  Where those chunks sit in a row depends only on the lane
  // (rows 16 apart share the swizzle).
  const int sw = (r16 >> 1) & 7;
  const int c0 = ((2 * g) ^ sw) * VEC, c1 = ((2 * g + 1) ^ sw) * VEC;
  const T* dlane = d + g * KS;
  vec_t dcur[2], dnext[2];                            // d of this lane's k's: current slab, next slab
  auto load_d = [&](vec_t (&dst)[2], int kt) {
    dst[0] = *reinterpret_cast<const vec_t*>(dlane + (int64_t)kt * BK);
    dst[1] = *reinterpret_cast<const vec_t*>(dlane + (int64_t)kt * BK + VEC);
  };

  gload(0, 0);
  if (!SCALED && active) load_d(dcur, 0);
  landed();
  __syncthreads();
  {
    // -C, in one go now that the loads have landed (negating each entry as it is
    // loaded would make every load wait for itself)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][j][r] = -acc[i][j][r];
  }

  // One slab; MORE: another one follows (decided at compile time, so that the
  // stages of a slab form one straight run of instructions).  The next slab's loads
  // go out first, into the buffer nobody reads during this slab.
  auto slab = [&](const int kt, auto more_tag) {
    constexpr bool MORE = decltype(more_tag)::value;
    const int buf = kt & 1;
    if (MORE) gload(kt + 1, buf ^ 1);
    if (active) {
      if (!SCALED && MORE) load_d(dnext, kt + 1);
      T nd[KS];                                         // d, this lane's k's
      if constexpr (!SCALED) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { nd[e] = dcur[0][e]; nd[VEC + e] = dcur[1][e]; }
      }
      const T* as = &As[buf][(wm * WT + r16) * BK];
      const T* bs = &Bs[buf][(wn * WT + r16) * BK];
      // Fragments are fetched one 16-row strip at a time, each fetch issued one
      // stage ahead of its first use, so that LDS latency hides behind the chain
      // of MFMAs of the stage before.  Stage (i, j): all KS products of
      // accumulator (i, j) back to back.
      T fa[2][KS], fb[TM][KS];
      auto fetch = [&](T (&f)[KS], const T* base) {
        const vec_t v0 = *reinterpret_cast<const vec_t*>(base + c0);
        const vec_t v1 = *reinterpret_cast<const vec_t*>(base + c1);
#pragma unroll
        for (int e = 0; e < VEC; ++e) { f[e] = v0[e]; f[VEC + e] = v1[e]; }
      };
      auto scale = [&](T (&f)[KS]) {
        if constexpr (!SCALED) {
#pragma unroll
          for (int e = 0; e < KS; ++e) f[e] *= nd[e];
        }
      };
      fetch(fa[0], as);
      fetch(fb[0], bs);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          if (i == 0 && j + 1 < TM) fetch(fb[j + 1], bs + (j + 1) * 16 * BK);
          if (j == TM - 1 && i + 1 < TM) fetch(fa[(i + 1) & 1], as + (i + 1) * 16 * BK);
          if (j == 0) scale(fa[i & 1]);
          __builtin_amdgcn_sched_barrier(0);   // all of the above goes out before this stage's products
#pragma unroll
          for (int e = 0; e < KS; ++e) acc[i][j] = X::mfma(fa[i & 1][e], fb[j][e], acc[i][j]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (MORE) {
      landed();
      if constexpr (!SCALED) {
        dcur[0] = dnext[0];
        dcur[1] = dnext[1];
      }
    }
    __syncthreads();
  };
  for (int kt = 0; kt + 1 < nk; ++kt) slab(kt, std::true_type{});
  slab(nk - 1, std::false_type{});

  // ---- epilogue: store the reduced block ----------------------------------
  // The workgroup that goes on to factor the leaf at the block's top left hands that
  // part over in LDS (the operand buffers are free after the last slab's barrier)
  // and leaves its write-back to the factorisation.
  const bool fuse = lower && fl.w > 0 && bm == 0 && bn == 0;
  const int wleaf = fuse ? fl.w : 0;
  if (fuse) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          leaf_tile_put<T>(lds, wm * WT + i * 16 + X::acc_row(lane, r), wn * WT + j * 16 + r16,
                           wleaf, -acc[i][j][r]);
  }
  if (active) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int grow = row0 + wm * WT + i * 16 + X::acc_row(lane, r);
        if (grow >= M) continue;
        T* crow = C + (int64_t)grow * ldc;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          const int gcol = col0 + wn * WT + j * 16 + r16;
          if (gcol < N && (!lower || gcol <= grow) && !(grow < wleaf && gcol < wleaf))
            crow[gcol] = -acc[i][j][r];
        }
      }
    }
  }
  if (fuse) {
    __syncthreads();
    leaf_factor_body<T, true>(C, ldc, fl.w, fl.dvec, fl.dinv, fl.linv, fl.pivot0, fl.flags, lds,
                              fl.spd);
  }
}

// One block per workgroup.
template <typename T, int TM, bool SCALED = false>
__device__ __forceinline__ void schur_update_body(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int K,
    int nsn, int swl, const bool lower, int per, int k0, const FusedLeaf<T>& fl) {
  using Sh = UpdShape<T, TM>;
  __shared__ __attribute__((aligned(16))) T lds[Sh::LDS_ELEMS];
  int bm, bn;
  if (!update_block_of(lower, blockIdx.x, per, k0, (M + Sh::BM - 1) / Sh::BM,
                       (N + Sh::BN - 1) / Sh::BN, nsn, swl, bm, bn))
    return;
  schur_update_block<T, TM, SCALED>(C, ldc, A, lda, B, ldb, d, M, N, K, lower, bm, bn, fl, lds);
}

// Names for the same body: the update of the trailing matrix by a finished block
// column (the bulk of all work), and the updates inside a block column's own
// recursive factorisation (128- and 64-wide blocks; the small one spreads short
// launches over more compute units).  The latter sit on the chain of dependent
// launches and often share SIMDs with a workgroup of the former: they run at a
// raised wave priority.
template <typename T, bool SCALED = false>
__global__ __launch_bounds__(UPD_THREADS, 2) void trailing_update_kernel(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int K, int nsn,
    int swl, int lower, int per, int k0, FusedLeaf<T> fl) {
  schur_update_body<T, 4, SCALED>(C, ldc, A, lda, B, ldb, d, M, N, K, nsn, swl, lower != 0, per, k0, fl);
}
// The trailing update of a short block column: with 128 x 128 blocks it would have
// fewer workgroups than the device has compute units and last as long as one
// workgroup's walk along K; 64 x 64 blocks quarter that walk.
template <typename T, bool SCALED = false>
__global__ __launch_bounds__(UPD_THREADS) void trailing_update64_kernel(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int K, int nsn,
    int swl, int lower, int per, int k0, FusedLeaf<T> fl) {
  schur_update_body<T, 2, SCALED>(C, ldc, A, lda, B, ldb, d, M, N, K, nsn, swl, lower != 0, per, k0, fl);
}
template <typename T, bool SCALED = false>
__global__ __launch_bounds__(UPD_THREADS, 2) void panel_update_kernel(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int K, int nsn,
    int swl, int lower, int per, int k0, FusedLeaf<T> fl) {
  __builtin_amdgcn_s_setprio(2);
  schur_update_body<T, 4, SCALED>(C, ldc, A, lda, B, ldb, d, M, N, K, nsn, swl, lower != 0, per, k0, fl);
}
template <typename T, bool SCALED = false>
__global__ __launch_bounds__(UPD_THREADS) void panel_update64_kernel(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int K, int nsn,
    int swl, int lower, int per, int k0, FusedLeaf<T> fl) {
  __builtin_amdgcn_s_setprio(2);
  schur_update_body<T, 2, SCALED>(C, ldc, A, lda, B, ldb, d, M, N, K, nsn, swl, lower != 0, per, k0, fl);
}

// K = 64 exactly (the update of the columns right of a leaf by that leaf): both
// operands, the pivots and the C block are requested in one go and the whole
// product runs from LDS, so the launch costs one memory round trip instead of one
// per slab.  64 x 64 block of C per workgroup, 2 x 2 MFMA tiles per wavefront.
template <typename T, bool SCALED>
__device__ __forceinline__ void leaf_update_body(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int nsn, int swl,
    int lower_, int per, const FusedLeaf<T>& fl) {
  __builtin_amdgcn_s_setprio(2);
  const bool lower = lower_ != 0;
  using X = Mfma<T>;
  using acc_t = typename X::acc_t;
  using vec_t = typename X::vec_t;
  constexpr int VEC = X::VEC, BK = X::BK, KS = BK / 4;
  constexpr int KT = 64;                                    // K
  constexpr int S = (KT * (int)sizeof(T) + 16) / (int)sizeof(T);   // padded LDS row, elements
  constexpr int VPR = KT / VEC;                             // 16-byte vectors per row
  constexpr int NV = VPR / 4;                               // per thread (4 threads per row)
  __shared__ __attribute__((aligned(16))) T lds[2 * 64 * S];
  static_assert(2 * 64 * S >= FACTOR_LDS_ELEMS, "the fused leaf needs the operand buffers");
  T* As = lds;
  T* Bs = lds + 64 * S;

  int bm, bn;
  if (!update_block_of(lower, blockIdx.x, per, 0, (M + 63) / 64, (N + 63) / 64, nsn, swl, bm, bn))
    return;
  const int row0 = bm * 64, col0 = bn * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r16 = lane & 15, g = lane >> 4;
  const bool active = !(lower && (row0 + wm * 32 + 31 < col0 + wn * 32));

  const int srow = tid >> 2, sq = tid & 3;
  int ar = row0 + srow; if (ar > M - 1) ar = M - 1;
  int br = col0 + srow; if (br > N - 1) br = N - 1;
  const T* Ap = A + (int64_t)ar * lda + sq * NV * VEC;
  const T* Bp = B + (int64_t)br * ldb + sq * NV * VEC;
  const T* dp = d + sq * NV * VEC;
  vec_t ra[NV], rb[NV], rd[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    ra[v] = *reinterpret_cast<const vec_t*>(Ap + v * VEC);
    rb[v] = *reinterpret_cast<const vec_t*>(Bp + v * VEC);
    if constexpr (!SCALED) rd[v] = *reinterpret_cast<const vec_t*>(dp + v * VEC);
  }
  acc_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = acc_t{0, 0, 0, 0};
  if (active) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int grow = row0 + wm * 32 + i * 16 + X::acc_row(lane, r);
        if (grow >= M) continue;
        const T* crow = C + (int64_t)grow * ldc;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int gcol = col0 + wn * 32 + j * 16 + r16;
          if (gcol < N && (!lower || gcol <= grow)) acc[i][j][r] = crow[gcol];
        }
      }
  }
  {
    T* as = &As[srow * S + sq * NV * VEC];
    T* bs = &Bs[srow * S + sq * NV * VEC];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if constexpr (SCALED) *reinterpret_cast<vec_t*>(as + v * VEC) = -ra[v];
      else *reinterpret_cast<vec_t*>(as + v * VEC) = -(ra[v] * rd[v]);
      *reinterpret_cast<vec_t*>(bs + v * VEC) = rb[v];
    }
  }
  __syncthreads();
  if (active) {
#pragma unroll
    for (int slab = 0; slab < KT / BK; ++slab) {
      const T* as = &As[(wm * 32 + r16) * S + slab * BK + g * KS];
      const T* bs = &Bs[(wn * 32 + r16) * S + slab * BK + g * KS];
#pragma unroll
      for (int h = 0; h < KS / VEC; ++h) {
        vec_t fa[2], fb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          fa[t] = *reinterpret_cast<const vec_t*>(as + t * 16 * S + h * VEC);
          fb[t] = *reinterpret_cast<const vec_t*>(bs + t * 16 * S + h * VEC);
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e)
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = X::mfma(fa[i][e], fb[j][e], acc[i][j]);
      }
    }
  }
  // the workgroup that factors the leaf at C's top left hands it over in LDS
  const bool fuse = lower && fl.w > 0 && bm == 0 && bn == 0;
  const int wleaf = fuse ? fl.w : 0;
  if (fuse) {
    __syncthreads();   // everybody is done with the operands
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          leaf_tile_put<T>(lds, wm * 32 + i * 16 + X::acc_row(lane, r), wn * 32 + j * 16 + r16,
                           wleaf, acc[i][j][r]);
  }
  if (active) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int grow = row0 + wm * 32 + i * 16 + X::acc_row(lane, r);
        if (grow >= M) continue;
        T* crow = C + (int64_t)grow * ldc;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int gcol = col0 + wn * 32 + j * 16 + r16;
          if (gcol < N && (!lower || gcol <= grow) && !(grow < wleaf && gcol < wleaf))
            crow[gcol] = acc[i][j][r];
        }
      }
  }
  if (fuse) {
    __syncthreads();
    leaf_factor_body<T, true>(C, ldc, fl.w, fl.dvec, fl.dinv, fl.linv, fl.pivot0, fl.flags, lds,
                              fl.spd);
  }
}

template <typename T, bool SCALED = false>
__global__ __launch_bounds__(UPD_THREADS) void leaf_update_kernel(
    T* __restrict__ C, int64_t ldc, const T* __restrict__ A, int64_t lda,
    const T* __restrict__ B, int64_t ldb, const T* __restrict__ d, int M, int N, int nsn, int swl,
    int lower_, int per, FusedLeaf<T> fl) {
  leaf_update_body<T, SCALED>(C, ldc, A, lda, B, ldb, d, M, N, nsn, swl, lower_, per, fl);
}

// General matrices (Sec. 2.2, Eq. 1: M = P L U): the matrix is two lower-triangular arrays
// qoff elements apart, the entries on and below the diagonal and the transposed entries
// above it.  The same update runs on both in one launch with two rows of workgroups
// (blockIdx.y): the first array takes A's rows there and B's rows in the second array,
// the second array the other way round.  C, A and B all point into the first array.
template <typename T>
struct GeneralOperands {
  T* C;
  const T* A;
  const T* B;
};
template <typename T>
__device__ __forceinline__ GeneralOperands<T> general_operands(T* C, const T* A, const T* B, int64_t qoff) {
  if (blockIdx.y != 0) return {C + qoff, A + qoff, B};
  return {C, A, B + qoff};
}
template <typename T>
__global__ __launch_bounds__(UPD_THREADS) void leaf_update_general_kernel(
    T* C, int64_t ldc, const T* A, int64_t lda, const T* B, int64_t ldb, const T* __restrict__ d,
    int M, int N, int nsn, int swl, int lower_, int per, int64_t qoff) {
  const GeneralOperands<T> o = general_operands<T>(C, A, B, qoff);
  const FusedLeaf<T> none{0, nullptr, nullptr, nullptr, 0, nullptr, 0};
  leaf_update_body<T, false>(o.C, ldc, o.A, lda, o.B, ldb, d, M, N, nsn, swl, lower_, per, none);
}
#define MDET_GENERAL_UPDATE_KERNEL(NAME, TM, OCC, PRIO)                                              \
  template <typename T>                                                                             \
  __global__ __launch_bounds__(UPD_THREADS, OCC) void NAME(                                         \
      T* C, int64_t ldc, const T* A, int64_t lda, const T* B, int64_t ldb, const T* __restrict__ d, \
      int M, int N, int K, int nsn, int swl, int lower, int per, int k0, int64_t qoff) {            \
    if (PRIO) __builtin_amdgcn_s_setprio(2);                                                        \
    const GeneralOperands<T> o = general_operands<T>(C, A, B, qoff);                                \
    const FusedLeaf<T> none{0, nullptr, nullptr, nullptr, 0, nullptr, 0};                           \
    schur_update_body<T, TM, false>(o.C, ldc, o.A, lda, o.B, ldb, d, M, N, K, nsn, swl, lower != 0, \
                                    per, k0, none);                                                 \
  }
MDET_GENERAL_UPDATE_KERNEL(trailing_update_general_kernel, 4, 2, 0)
MDET_GENERAL_UPDATE_KERNEL(trailing_update64_general_kernel, 2, 1, 0)
MDET_GENERAL_UPDATE_KERNEL(panel_update_general_kernel, 4, 2, 1)
MDET_GENERAL_UPDATE_KERNEL(panel_update64_general_kernel, 2, 1, 1)
#undef MDET_GENERAL_UPDATE_KERNEL

// Two leaves side by side (a 128-column strip of a block column), the first one
// factored: one launch solves the rows below the first leaf against it, updates the
// second leaf's columns of those rows with the result (K = 64), and factors the second
// leaf.  Separately these are a leaf_solve_kernel and a leaf_update_kernel, the second
// waiting for all of the first; here a workgroup needs nothing from the others: it
// solves its own 64 rows and, once more, the 64 rows of the second leaf (rows 0 .. 63
// below the first), whose solved form is the right operand of everybody's update.
// Those 64 rows therefore stay as they are in memory during this launch (every
// workgroup reads them unsolved); workgroup 0, which owns them, puts their solved form
// into `l10` (64 x 64, row-major) and the solve launch of the second leaf copies it
// into place (leaf_solve_kernel, fix_src).
//   Xg    row 0 of the region below the first leaf, column 0 of the strip; m rows
//   Lleaf the first leaf, factored; dinv, dvec, linv: its reciprocal pivots, pivots and
//         the inverses of its diagonal sub-blocks (linv must not be the array that the
//         fused factorisation of the second leaf writes, fl.linv: workgroups start at
//         different times)
//   Wg    as in leaf_solve_kernel
// The update's left operand is the solved row before its division by the pivots,
// w = l d, which the solve keeps in LDS anyway; its right operand the second leaf's rows
// l (SCALED, the positive-definite form, where dinv holds d^(-1/2) and l stands for the
// row of the Cholesky factor: l d^(-1/2), so that the product is again w (1/d) w^T).
// LDS: 94 KB in fp64, which fits beside one workgroup of the trailing update on a
// compute unit, so that the launch need not wait for whole units to drain.
template <typename T, bool SCALED = false>
__global__ __launch_bounds__(256) void leaf_pair_kernel(
    T* __restrict__ Xg, int64_t ld, int m, const T* __restrict__ Lleaf, int64_t ldl,
    const T* __restrict__ dinv, const T* __restrict__ linv, const T* __restrict__ dvec,
    T* __restrict__ Wg, int64_t ldw, int wfrom, T* __restrict__ l10, FusedLeaf<T> fl) {
  using X = Mfma<T>;
  using acc_t = typename X::acc_t;
  using vec_t = typename X::vec_t;
  constexpr int VEC = X::VEC, BK = X::BK, KS = BK / 4;
  constexpr int KT = 64;
  constexpr int S = (KT * (int)sizeof(T) + 16) / (int)sizeof(T);   // padded LDS row of an operand
  constexpr int LW = LEAF - SUB;
  constexpr int LW_PAD = LW + 1;
  __shared__ T Ls[LW * LW_PAD];                 // first leaf: L[16.., ..47], strictly lower part
  __shared__ T Li[NSUB * SUB * SUB_PAD];        // inverses of its diagonal sub-blocks
  __shared__ T rinv[LEAF];
  __shared__ T dsc[LEAF];
  // As: the solved rows w of the workgroup, 16 per wavefront (while a wavefront solves the
  // second leaf's rows, theirs); Bs: the second leaf's rows l; later the second leaf itself
  __shared__ __attribute__((aligned(16))) T ops[2 * 64 * S];
  static_assert(2 * 64 * S >= FACTOR_LDS_ELEMS, "the fused leaf needs the operand buffers");
  T* As = ops;
  T* Bs = ops + 64 * S;
  __builtin_amdgcn_s_setprio(2);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int blk = blockIdx.x;
  const bool first = blk == 0;                  // this workgroup's rows are the second leaf's

  // the block of C: rows 64 blk .. of the region, columns 64 .. 127 of the strip; its
  // (0, 0) for blk = 0 is on the matrix diagonal
  T* C = Xg + LEAF;
  const int row0 = blk * 64;
  const int wm = wave >> 1, wn = wave & 1;
  const bool active = !(row0 + wm * 32 + 31 < wn * 32);
  acc_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = acc_t{0, 0, 0, 0};
  if (active) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int grow = row0 + wm * 32 + i * 16 + X::acc_row(lane, r);
        if (grow >= m) continue;
        const T* crow = C + (int64_t)grow * ld;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int gcol = wn * 32 + j * 16 + l16;
          if (gcol <= grow) acc[i][j][r] = crow[gcol];
        }
      }
  }
  // rows to solve, in accumulator layout: this wavefront's 16 of the workgroup's own
  // rows and its 16 of the second leaf's
  const int64_t r_own = ((int64_t)blk * 4 + wave) * SUB, r_leaf = (int64_t)wave * SUB;
  acc_t x_own[NSUB], x_leaf[NSUB];
#pragma unroll
  for (int b = 0; b < NSUB; ++b)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = b * SUB + l16;
      const int64_t ro = r_own + X::acc_row(lane, r), rl = r_leaf + X::acc_row(lane, r);
      x_own[b][r] = ro < m ? Xg[ro * ld + col] : T(0);
      x_leaf[b][r] = (!first && rl < m) ? Xg[rl * ld + col] : T(0);
    }
  {
    T v[LEAF * LEAF / 256];
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / 256; ++q) {
      const int e = q * 256 + tid, r = e >> 6, c = e & 63;
      v[q] = c < r ? Lleaf[(int64_t)r * ldl + c] : T(0);
    }
    T u[NSUB * SUB * SUB / 256];
#pragma unroll
    for (int q = 0; q < NSUB * SUB * SUB / 256; ++q) u[q] = linv[q * 256 + tid];
    const T myr = tid < LEAF ? dinv[tid < LEAF ? tid : 0] : T(0);
    const T myd = tid < LEAF ? dvec[tid < LEAF ? tid : 0] : T(0);
#pragma unroll
    for (int q = 0; q < LEAF * LEAF / 256; ++q) {
      const int e = q * 256 + tid, r = e >> 6, c = e & 63;
      if (r >= SUB && c < LW) Ls[(r - SUB) * LW_PAD + c] = v[q];
    }
#pragma unroll
    for (int q = 0; q < NSUB * SUB * SUB / 256; ++q) {
      const int e = q * 256 + tid, bq = e >> 8, i = (e >> 4) & 15, k = e & 15;
      Li[(bq * SUB + i) * SUB_PAD + k] = u[q];
    }
    if (tid < LEAF) { rinv[tid] = myr; dsc[tid] = myd; }
  }
  __syncthreads();

  // X L^-T D^-1 for 16 rows, as leaf_solve_kernel; the wavefront's 16 rows of As hold the
  // solved sub-blocks, and sub-block b's columns of them also serve for the change of
  // layout of T_b (a wavefront's LDS operations complete in order).  own: the
  // workgroup's rows (stored, As keeps them as the left operand); otherwise the second
  // leaf's rows (right operand only).
  T* ws = As + wave * SUB * S;
  auto solve16 = [&](acc_t (&x)[NSUB], const int64_t r0, const bool own) {
#pragma unroll
    for (int b = 0; b < NSUB; ++b) {
      acc_t a = x[b];
#pragma unroll 1
      for (int p = 0; p < b; ++p) {
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const int k = p * SUB + 4 * s4 + g;
          a = X::mfma(-ws[l16 * S + k], Ls[((b - 1) * SUB + l16) * LW_PAD + k], a);
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) ws[X::acc_row(lane, r) * S + b * SUB + l16] = a[r];
      acc_t wb = acc_t{0, 0, 0, 0};
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        const int k = 4 * s4 + g;
        wb = X::mfma(ws[l16 * S + b * SUB + k], Li[(b * SUB + l16) * SUB_PAD + k], wb);
      }
      const T rj = rinv[b * SUB + l16];
      const T dj = dsc[b * SUB + l16];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row16 = X::acc_row(lane, r);
        ws[row16 * S + b * SUB + l16] = wb[r];
        const int64_t row = r0 + row16;
        const int col = b * SUB + l16;
        const T lv = wb[r] * rj;
        if (own && row < m) {
          if (first) l10[(int)row * LEAF + col] = lv;
          else Xg[row * ld + col] = lv;
          if (Wg != nullptr && row >= wfrom) Wg[row * ldw + col] = lv * dj;
        }
        if (!own || first) Bs[(wave * SUB + row16) * S + col] = SCALED ? lv * rj : lv;
      }
    }
  };
  if (!first) solve16(x_leaf, r_leaf, false);
  solve16(x_own, r_own, true);
  __syncthreads();

  if (active) {
#pragma unroll
    for (int slab = 0; slab < KT / BK; ++slab) {
      const T* as = &As[(wm * 32 + l16) * S + slab * BK + g * KS];
      const T* bs = &Bs[(wn * 32 + l16) * S + slab * BK + g * KS];
#pragma unroll
      for (int h = 0; h < KS / VEC; ++h) {
        vec_t fa[2], fb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          fa[t] = -*reinterpret_cast<const vec_t*>(as + t * 16 * S + h * VEC);
          fb[t] = *reinterpret_cast<const vec_t*>(bs + t * 16 * S + h * VEC);
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e)
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = X::mfma(fa[i][e], fb[j][e], acc[i][j]);
      }
    }
  }
  const bool fuse = first && fl.w > 0;
  const int wleaf = fuse ? fl.w : 0;
  if (fuse) {
    __syncthreads();   // everybody is done with the operands
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          leaf_tile_put<T>(ops, wm * 32 + i * 16 + X::acc_row(lane, r), wn * 32 + j * 16 + l16, wleaf,
                           acc[i][j][r]);
  }
  if (active) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int grow = row0 + wm * 32 + i * 16 + X::acc_row(lane, r);
        if (grow >= m) continue;
        T* crow = C + (int64_t)grow * ld;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int gcol = wn * 32 + j * 16 + l16;
          if (gcol <= grow && !(grow < wleaf && gcol < wleaf)) crow[gcol] = acc[i][j][r];
        }
      }
  }
  if (fuse) {
    __syncthreads();
    leaf_factor_body<T, true>(C, ld, fl.w, fl.dvec, fl.dinv, fl.linv, fl.pivot0, fl.flags, ops, fl.spd);
  }
}

}  // namespace mdet
