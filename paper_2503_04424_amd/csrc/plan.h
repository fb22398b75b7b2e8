// Host-side planner: block grid, residency plan and traffic prediction.
//
// The paper picks the number of blocks n_b from a memory cap c with
// r = m sqrt(beta/c) (App. D) and keeps 3-4 equal blocks in memory.  On a GPU with
// a host link far slower than HBM, four equal blocks would leave the matrix cores
// waiting; this planner instead keeps a *group of whole block columns* ("super
// panel") resident and streams the already-factored block columns past it, so
// that each streamed block is used for as many products as the group has columns.
// The budget is still a hard cap: everything the call allocates on the device is
// accounted for here.  Pure C++, no HIP.
#pragma once
#include <stdint.h>
#include <vector>

#include "../../include/memdet.h"

namespace mdet {

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

struct SuperPanel {
  int64_t j0, j1;            // block columns [j0, j1)
  uint64_t resident_bytes;   // bytes of those columns (rows from their diagonal down)
};

struct Plan {
  int64_t n = 0, bs = 0, T = 0;
  int beta = 8;                    // bytes per element on the device (the arithmetic's type)
  int src_beta = 8;                // bytes per element of the caller's matrix (differs with MDET_FLAG_COMPUTE_F64)
  bool widen = false;              // MDET_FLAG_COMPUTE_F64: stored narrow, widened exactly on the device
  uint64_t stage_bytes = 0;        // host entry points with widen: device staging for the narrow uploads
  bool device_input = false;
  bool out_of_core = false;
  bool need_copy = false;          // device input: work on a copy (overwrite = 0)
  bool pivot = false;              // MDET_FLAG_PIVOT or MDET_FLAG_PIVOT_BLOCK: a permutation is kept
  bool pivot_block = false;        // MDET_FLAG_PIVOT_BLOCK: candidates = the whole diagonal block
  uint64_t pb_bytes = 0;           // its workspace (pivot_block_area), right behind the small area
  bool general = false;            // MDET_FLAG_GENERAL: P A = L D U, two triangular arrays
  uint64_t q_bytes = 0;            // the second of them (device input)
  uint64_t arena_half = 0;         // host input: bytes of block columns and streamed blocks of ONE array
                                   // (a general matrix has two, the second arena_half bytes after the first)
  uint64_t small_bytes = 0;        // pivots, reciprocals, flags, reduction scratch
  uint64_t layout_bytes = 0;       // packed lower block-column layout
  uint64_t copy_bytes = 0;
  uint64_t wcopy_bytes = 0;        // two pivot-scaled copies of a block column (MDET_FLAG_SCALED_COPY)
  bool wcopy_optional = false;     // taken without being asked for: dropped if memory is short
  uint64_t ring_tiles = 3;         // streamed row blocks in flight (out-of-core)
  uint64_t tile_bytes = 0;
  uint64_t dev_bytes = 0;          // total device bytes the call uses
  uint64_t host_bytes = 0;
  uint64_t h2d = 0, d2h = 0;
  std::vector<SuperPanel> panels;

  int64_t col_width(int64_t j) const { int64_t w = n - j * bs; return w < bs ? w : bs; }
  int64_t col_rows(int64_t j) const { return n - j * bs; }
  // element offset of block column j in the packed layout
  int64_t col_offset(int64_t j) const {
    // sum_{t<j} (n - t bs) * w_t ; all t < j <= T-1 have w_t = bs unless j == T
    int64_t full = j < T ? j : T - 1;
    int64_t off = full * n * bs - bs * bs * (full * (full - 1) / 2);
    if (j == T && T > 0) off += col_rows(T - 1) * col_width(T - 1);
    return off;
  }
  uint64_t col_bytes(int64_t j) const { return (uint64_t)col_rows(j) * col_width(j) * beta; }
  // on the device a block column keeps a leading dimension that is a multiple of 4
  // elements (16-byte rows); only a ragged last column differs from the host layout
  int64_t col_ld(int64_t j) const { return round_up(col_width(j), 4); }
  uint64_t dev_col_bytes(int64_t j) const { return (uint64_t)col_rows(j) * col_ld(j) * beta; }
  uint64_t block_bytes(int64_t i, int64_t k) const {   // block (i, k), i >= k
    return (uint64_t)col_width(i) * col_width(k) * beta;   // rows of block row i = w_i
  }
};

inline int64_t default_block_size(int64_t n) {
  int64_t b = round_up(n / 16 > 0 ? n / 16 : 1, 64);
  if (b < 256) b = 256;
  if (b > 4096) b = 4096;
  return b;
}

inline uint64_t align256(uint64_t x) { return (x + 255) / 256 * 256; }

// Layout of the small scratch area (offsets in bytes from its start).
struct SmallArea {
  uint64_t dvec, dinv, linv, l10, flags, partial, out, running, perm, total;
};
// pivot: room for the permutation (n 32-bit indices) of MDET_FLAG_PIVOT
inline SmallArea small_area(int64_t n, int64_t T, int beta, bool pivot) {
  SmallArea a;
  uint64_t o = 0;
  a.dvec = o; o += align256((uint64_t)(n > 0 ? n : 1) * beta);
  a.dinv = o; o += align256((uint64_t)(n > 0 ? n : 1) * beta);
  a.linv = o; o += 2 * align256((uint64_t)64 * 16 * beta);   // inverse diagonal sub-blocks of two leaves
  a.l10 = o; o += align256((uint64_t)64 * 64 * beta);        // a 64 x 64 block on its way into place
  a.flags = o; o += 256;
  a.partial = o; o += align256((uint64_t)(T > 0 ? T : 1) * 3 * 8);
  a.out = o; o += 256;
  a.running = o; o += align256((uint64_t)(T > 0 ? T : 1) * 8);
  a.perm = o; if (pivot) o += align256((uint64_t)(n > 0 ? n : 1) * 4);
  a.total = o;
  return a;
}

// Workspace of MDET_FLAG_PIVOT_BLOCK (offsets in bytes from its start): the diagonal block as
// a full symmetric matrix, the block's multipliers with rows in input order and columns in
// pivot order, the rows below the block with their columns in pivot order, and small arrays.
struct PivotBlockArea {
  uint64_t S, Lfull, Y, Bg, leaf, linv, dg, active, piv, part, total;
  int64_t ldl;                 // leading dimension of S, Lfull, Y and Bg: bs rounded up to 64
};
inline PivotBlockArea pivot_block_area(int64_t n, int64_t bs, int beta) {
  PivotBlockArea a;
  a.ldl = round_up(bs > 0 ? bs : 64, 64);
  const uint64_t rows_below = (uint64_t)(n > bs ? n - bs : 0);
  uint64_t o = 0;
  a.S = o; o += align256((uint64_t)bs * a.ldl * beta);
  a.Lfull = o; o += align256((uint64_t)bs * a.ldl * beta);
  a.Y = o; o += align256((rows_below + 64) * a.ldl * beta);
  a.Bg = o; o += align256((uint64_t)64 * a.ldl * beta);
  a.leaf = o; o += align256((uint64_t)64 * 64 * beta);
  a.linv = o; o += align256((uint64_t)64 * 16 * beta);
  a.dg = o; o += align256((uint64_t)bs * beta);
  a.active = o; o += align256((uint64_t)bs * 4);
  a.piv = o; o += align256((uint64_t)bs * 4);
  a.part = o; o += align256((uint64_t)2 * 64 * 16);
  a.total = o;
  return a;
}

// Returns an mdet_status.
inline int make_plan(const mdet_params& p, bool device_input, int64_t ld, Plan& pl) {
  if (p.n < 0 || p.block_size < 0) return MDET_EINVAL;
  const bool narrow16 = p.dtype == MDET_F16 || p.dtype == MDET_BF16;
  if (p.dtype != MDET_F32 && p.dtype != MDET_F64 && !narrow16) return MDET_EINVAL;
  // fp32 or 16-bit storage with fp64 arithmetic: everything on the device is fp64
  const bool widen = p.dtype != MDET_F64 && (p.flags & MDET_FLAG_COMPUTE_F64) != 0;
  if (narrow16 && !widen) return MDET_EINVAL;      // 16-bit types are storage formats only
  pl.n = p.n;
  pl.beta = (p.dtype == MDET_F64 || widen) ? 8 : 4;
  pl.widen = widen;
  pl.src_beta = p.dtype == MDET_F64 ? 8 : (p.dtype == MDET_F32 ? 4 : 2);
  pl.bs = round_up(p.block_size > 0 ? p.block_size : default_block_size(p.n), 64);
  pl.T = p.n > 0 ? (p.n + pl.bs - 1) / pl.bs : 0;
  pl.device_input = device_input;
  pl.tile_bytes = (uint64_t)pl.bs * pl.bs * pl.beta;
  pl.pivot_block = (p.flags & MDET_FLAG_PIVOT_BLOCK) != 0;
  if (pl.pivot_block && (p.flags & (MDET_FLAG_PIVOT | MDET_FLAG_GENERAL))) return MDET_EINVAL;
  pl.pivot = (p.flags & (MDET_FLAG_PIVOT | MDET_FLAG_PIVOT_BLOCK)) != 0;
  // general matrix: in the arithmetic of its own type; the row order inside each leaf is
  // always recorded.  From host memory both triangles travel: twice the arrays, twice the traffic
  pl.general = (p.flags & MDET_FLAG_GENERAL) != 0;
  if (pl.general && (widen || (p.flags & MDET_FLAG_PIVOT))) return MDET_EINVAL;
  if (pl.general && (p.flags & MDET_FLAG_ASSUME_SPD)) return MDET_EINVAL;
  if (pl.general) pl.pivot = true;
  if (pl.pivot && (p.flags & MDET_FLAG_ASSUME_SPD)) return MDET_EINVAL;   // nothing to choose from
  if (pl.pivot && p.n > INT32_MAX) return MDET_EINVAL;
  pl.pb_bytes = pl.pivot_block ? pivot_block_area(pl.n, pl.bs, pl.beta).total : 0;
  // counted with the fixed part of the workspace, which it follows
  pl.small_bytes = small_area(pl.n, pl.T, pl.beta, pl.pivot).total + pl.pb_bytes;
  pl.layout_bytes = pl.T > 0 ? (uint64_t)pl.col_offset(pl.T) * pl.beta : 0;
  pl.panels.clear();
  pl.h2d = pl.d2h = 0;
  pl.host_bytes = 0;
  const uint64_t budget = p.mem_budget_bytes;
  // optional: room for W = L D of the block column being factored and of the one whose
  // bulk update is still running; taken only where everything is resident and it fits
  pl.wcopy_bytes = 0;
  // asked for, or taken unasked where nothing caps the memory and the matrix is large
  // enough for it to pay (measured cross-over between n = 16384 and 24576); the unasked
  // one is given up again if the workspace cannot be had (wcopy_optional)
  const bool wcopy_auto = !(p.flags & MDET_FLAG_SCALED_COPY) && budget == 0 && p.n >= 24576;
  const uint64_t wcopy = (((p.flags & MDET_FLAG_SCALED_COPY) || wcopy_auto) &&
                          !(p.flags & MDET_FLAG_ASSUME_SPD) && !pl.general && !pl.pivot_block && pl.T >= 2)
                             ? 2 * align256((uint64_t)pl.n * pl.bs * pl.beta) : 0;
  pl.wcopy_optional = wcopy_auto && wcopy != 0;
  pl.arena_half = 0;

  if (device_input) {
    const int vec = 16 / pl.beta;
    const bool aligned = ld % vec == 0;
    pl.need_copy = widen || !p.overwrite || !aligned;
    if (pl.need_copy) {
      int64_t ldp = round_up(p.n > 0 ? p.n : 1, vec);
      pl.copy_bytes = align256((uint64_t)p.n * ldp * pl.beta);
    }
    pl.q_bytes = 0;
    if (pl.general) {
      // the transposed upper triangle: an array shaped like the one the driver works on
      const int64_t ldq = pl.need_copy ? round_up(p.n > 0 ? p.n : 1, vec) : ld;
      pl.q_bytes = align256((uint64_t)p.n * ldq * pl.beta);
    }
    pl.dev_bytes = pl.small_bytes + pl.copy_bytes + pl.q_bytes;
    pl.out_of_core = false;
    if (budget && pl.dev_bytes > budget) return MDET_EBUDGET;
    if (wcopy && (!budget || pl.dev_bytes + wcopy <= budget)) {
      pl.wcopy_bytes = wcopy;
      pl.dev_bytes += wcopy;
    }
    return MDET_OK;
  }

  const bool force_ooc = (p.flags & MDET_FLAG_FORCE_OUT_OF_CORE) != 0;
  uint64_t dev_layout = 0;
  for (int64_t j = 0; j < pl.T; ++j) dev_layout += align256(pl.dev_col_bytes(j));
  // narrow storage: the originals arrive in the stored width in a staging buffer of at most
  // 64 MiB (one block row of a block column at a time, cut further if need be) and are
  // widened from there into their block column.  A general matrix has the buffer too: blocks
  // of its upper triangle that a block provider hands over are transposed from there.
  pl.stage_bytes = 0;
  if ((widen || pl.general) && pl.T > 0) {
    const uint64_t piece = (uint64_t)pl.bs * pl.bs * pl.src_beta;
    const uint64_t one_row = (uint64_t)pl.bs * pl.src_beta;
    uint64_t st = piece < (64ull << 20) ? piece : (64ull << 20);
    if (st < one_row) st = one_row;
    pl.stage_bytes = align256(st);
  }
  pl.small_bytes += pl.stage_bytes;      // counted with the fixed part of the workspace
  const uint64_t arrays = pl.general ? 2 : 1;
  const uint64_t incore = pl.small_bytes + arrays * dev_layout;
  if (!force_ooc && (budget == 0 || incore <= budget)) {
    pl.out_of_core = false;
    pl.dev_bytes = incore;
    pl.arena_half = dev_layout;
    if (wcopy && (!budget || incore + wcopy <= budget)) {
      pl.wcopy_bytes = wcopy;
      pl.dev_bytes += wcopy;
    }
    pl.h2d = arrays * (pl.layout_bytes / pl.beta * pl.src_beta);
    pl.panels.push_back({0, pl.T, pl.layout_bytes});
    return MDET_OK;
  }

  // ---- out-of-core: greedy groups of block columns ------------------------
  pl.out_of_core = true;
  // with no cap at all (forced streaming) behave as if a quarter of the layout were allowed
  uint64_t cap = budget ? budget : (pl.small_bytes + arrays * (pl.layout_bytes / 4 + 8 * pl.tile_bytes));
  uint64_t peak = 0;
  int64_t j0 = 0;
  while (j0 < pl.T) {
    uint64_t resident = 0;
    int64_t j1 = j0;
    while (j1 < pl.T) {
      uint64_t cand = resident + align256(pl.dev_col_bytes(j1));
      uint64_t wc = (uint64_t)(j1 + 1 - j0);
      // streamed factor blocks: two sets of wc row blocks of the group's own rows
      // (operands reused by every streamed block) plus the ring
      uint64_t stream = (j0 > 0) ? (2 * wc + pl.ring_tiles) * align256(pl.tile_bytes) : 0;
      if (pl.small_bytes + arrays * (cand + stream) > cap) break;
      resident = cand;
      ++j1;
    }
    if (j1 == j0) return MDET_EBUDGET;   // not even one block column fits
    uint64_t wc = (uint64_t)(j1 - j0);
    uint64_t stream = (j0 > 0) ? (2 * wc + pl.ring_tiles) * align256(pl.tile_bytes) : 0;
    uint64_t use = pl.small_bytes + arrays * (resident + stream);
    if (use > peak) peak = use;
    if (resident + stream > pl.arena_half) pl.arena_half = resident + stream;
    pl.panels.push_back({j0, j1, resident});
    // traffic: originals in, factors out, and every earlier column's rows from j0 down
    for (int64_t j = j0; j < j1; ++j) {
      pl.h2d += arrays * (pl.col_bytes(j) / pl.beta * pl.src_beta);
      pl.d2h += arrays * pl.col_bytes(j);
    }
    for (int64_t k = 0; k < j0; ++k)
      pl.h2d += arrays * ((uint64_t)pl.col_rows(j0) * pl.col_width(k) * pl.beta);
    j0 = j1;
  }
  pl.dev_bytes = peak;
  // the factors are always in the arithmetic's type: a matrix stored narrower cannot take them
  pl.host_bytes = (p.overwrite && !widen) ? 0 : arrays * pl.layout_bytes;
  return MDET_OK;
}

// App. E.1 operation counts (fused multiply-adds) for n_b blocks of order b.
inline void paper_work_split(int64_t nb, double b, double* decomp, double* solve, double* gemm,
                             double* syrk) {
  double N = (double)nb;
  *decomp = N * (b * b * b / 6 - b * b / 4 + b / 12);
  *solve = (N * N / 2 - N / 2) * (b * b * b / 2 - b * b / 2);
  *gemm = (N * N * N / 6 - N * N / 2 + N / 3) * b * b * b;
  *syrk = (N * N / 2 - N / 2) * (b * b * b / 2);
}

}  // namespace mdet
