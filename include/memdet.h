/*
 * memdet.h - C ABI of the MI355X (gfx950) log-determinant library.
 *
 * The library computes  log|det A|  and  sign(det A)  of a large symmetric
 * matrix by a hierarchical block-wise LDL^T decomposition under a device-memory
 * budget: the symmetric case ("case II") of the paper's memory-constrained
 * algorithm (Sec. 2.2: block Schur-complement recursion of Eq. 1, stored-triangle
 * processing and diagonal scaling for LDL^T; App. D: inputs "matrix, maximum
 * memory c", outputs "l = log|det|, sigma = sign").  By default no pivoting is done: D is
 * diagonal, L unit lower triangular, and
 *
 *      logabsdet = sum_j log|d_j| ,   sign = prod_j sgn(d_j) .
 *
 * Flags select the other forms of the method: pivoting on the diagonal inside a block
 * (MDET_FLAG_PIVOT), the Cholesky form for positive-definite matrices
 * (MDET_FLAG_ASSUME_SPD), the LU form for general matrices (MDET_FLAG_GENERAL), and
 * storage narrower than the arithmetic (MDET_FLAG_COMPUTE_F64).
 *
 * Conventions common to every entry point
 *  - Only the LOWER triangle of the matrix is read.  Element (i, j), i >= j.
 *  - All sizes are in elements unless a name says bytes.  n may be any value
 *    >= 0; it need not be a multiple of block_size (the last block row/column is
 *    smaller, as in App. D where blocks are "at most b x b").
 *  - block_size is the order b of the square blocks the matrix is cut into (the
 *    paper's b = m / n_b).  It is rounded up to a multiple of 64 internally
 *    (result->block_size_used); the result does not depend on it beyond rounding.
 *  - Functions return an mdet_status; they never throw, abort or exit.  `result`
 *    is fully written on MDET_OK and MDET_ESINGULAR, and its hip_error /
 *    bad_pivot_index fields on the corresponding failures.
 *  - Calls are synchronous: on return all device work of the call has finished.
 *  - The library uses the HIP device that is current in the calling thread.
 *  - Thread safety: calls that use distinct workspaces may run concurrently.
 */
#ifndef MEMDET_H
#define MEMDET_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* MDET_F16 (IEEE binary16) and MDET_BF16 are storage formats only: accepted together with
 * MDET_FLAG_COMPUTE_F64, not without it. */
typedef enum { MDET_F32 = 0, MDET_F64 = 1, MDET_F16 = 2, MDET_BF16 = 3 } mdet_dtype;

typedef enum {
  MDET_OK = 0,
  MDET_EINVAL = 1,        /* bad argument (null pointer, negative size, ld < n, ...) */
  MDET_EBUDGET = 2,       /* mem_budget_bytes below the minimum working set        */
  MDET_ENOMEM_DEVICE = 3, /* device allocation failed / workspace too small        */
  MDET_ENOMEM_HOST = 4,   /* host allocation failed                                */
  MDET_EHIP = 5,          /* a HIP call failed; raw code in result->hip_error      */
  MDET_ESINGULAR = 6,     /* exact zero pivot: sign = 0, logabsdet = -inf          */
  MDET_ENONFINITE = 7,    /* NaN/Inf pivot met (input not finite or overflow)      */
  MDET_EPROVIDER = 8,     /* the block provider returned non-zero                  */
  MDET_ENOTPOSDEF = 9,    /* MDET_FLAG_ASSUME_SPD and a negative pivot was met      */
  MDET_EIO = 10           /* mdet_logdet_file: open, read or write failed, or the
                             file is shorter than the matrix                        */
} mdet_status;

/* Parameters of one log-determinant call.  Zero-initialise, then set fields. */
typedef struct mdet_params {
  uint32_t struct_size;      /* = sizeof(mdet_params); guards ABI drift            */
  int32_t dtype;             /* mdet_dtype: type of the matrix AND of the arithmetic
                                (but see MDET_FLAG_COMPUTE_F64)                     */
  int64_t n;                 /* matrix order (the paper's m)                        */
  int64_t block_size;        /* b; 0 = let the library choose                       */
  uint64_t mem_budget_bytes; /* cap on device bytes this call may allocate or use as
                                workspace (the paper's c, App. D).  0 = no cap.
                                For mdet_logdet_device the caller's matrix itself is
                                not counted; for the host/provider entry points every
                                device byte is.                                     */
  int32_t overwrite;         /* 1: the input may be destroyed (it then holds the
                                factor: unit-lower L below the diagonal, D on it).
                                0: the input is preserved (paper's overwrite=False:
                                Schur-updated blocks go to scratch space instead).  */
  int32_t reserved0;         /* must be 0                                           */
  uint32_t flags;            /* MDET_FLAG_* bits                                    */
  void* stream;              /* hipStream_t to order the work after (borrowed, e.g.
                                from PyTorch); NULL = the default stream.  The call
                                still synchronises before returning.               */
  void* dev_workspace;       /* optional caller-owned device scratch (e.g. a
                                torch.empty buffer); NULL = the library hipMallocs
                                what it needs (within the budget) and frees it.     */
  uint64_t dev_workspace_bytes;
  void* host_scratch;        /* out-of-core with overwrite=0 only: pinned host
                                memory of at least mdet_workspace_query()'s
                                host_bytes that receives the updated blocks; NULL =
                                the library allocates pinned memory itself.        */
  uint64_t host_scratch_bytes;
  void* perm;                /* MDET_FLAG_PIVOT, MDET_FLAG_GENERAL: n int32 that receive
                                the permutation (a DEVICE pointer for mdet_logdet_device,
                                a HOST pointer for the host and provider entry points);
                                NULL = not wanted.  Ignored without those flags.     */
} mdet_params;

#define MDET_FLAG_NO_LOOKAHEAD 1u /* run every step on one stream, strictly in order
                                     (results are bit-identical either way)        */
#define MDET_FLAG_FORCE_OUT_OF_CORE 2u /* host entry points: stream blocks even if the
                                     whole triangle would fit in the budget         */
#define MDET_FLAG_COMPUTE_F64 8u  /* dtype = MDET_F32, MDET_F16 or MDET_BF16: the matrix is
                                     STORED in that format and every arithmetic step
                                     runs in fp64 on the exactly widened values (App. C,
                                     data-precision pipeline, stage 3: whatever precision
                                     the matrix was stored in, the log-determinant is
                                     computed in 64 bit).  diag receives n DOUBLES.
                                     mdet_logdet_device works on an fp64 copy in its
                                     workspace (n * ld_padded * 8 bytes, counted against
                                     the budget; the input is never modified).  The host,
                                     provider and file entry points move the original
                                     blocks over the host link in the stored width and
                                     widen them on the device (a staging buffer of at most
                                     64 MiB, counted against the budget); the factored
                                     block columns of a streamed run are fp64 and never go
                                     back into the matrix: they go to host_scratch (or the
                                     scratch file), whatever `overwrite` says, and
                                     mdet_workspace_query reports the fp64 layout's size
                                     as host_bytes.                                    */
#define MDET_FLAG_PROFILE 4u      /* bracket every launch of the two trailing-update
                                     kernels (128 x 128 blocks for the bulk of the work,
                                     64 x 64 blocks for updates too small to fill the
                                     device) with HIP events on its own stream and
                                     report, per kernel, launches, summed durations and
                                     flops, and the union of all the intervals, in
                                     result->t_trailing_update etc.                 */
#define MDET_FLAG_SCALED_COPY 32u /* speed for memory: 2 n block_size further elements of
                                     device workspace hold, for the block column being
                                     factored, its rows scaled by the pivots (W = L D),
                                     so that the Schur updates read their left operand
                                     ready-made instead of scaling it on the fly.  Same
                                     bits in the result.  Used where the whole matrix is
                                     resident and the budget allows; ignored otherwise
                                     and with MDET_FLAG_ASSUME_SPD (nothing to scale).
                                     Without the flag the library does the same by itself
                                     when mem_budget_bytes == 0 and n >= 24576 (where it
                                     pays; mdet_plan and mdet_workspace_query count it),
                                     and goes without if that memory cannot be had.      */
#define MDET_FLAG_ASSUME_SPD 16u  /* the matrix is symmetric positive definite: use the
                                     Cholesky form of the method (the paper's algorithm
                                     for positive-definite matrices, App. D; block
                                     columns hold rows of L D^(1/2), the Schur updates
                                     are plain A B^T products without the diagonal
                                     scaling).  A negative pivot ends the call with
                                     MDET_ENOTPOSDEF and its index in bad_pivot_index;
                                     `diag` still receives the pivots d_j = L_jj^2.    */

#define MDET_FLAG_PIVOT 64u       /* symmetric pivoting inside each group of 64 consecutive
                                     rows/columns (Sec. 2.2: the symmetric form handles
                                     permutations; pivoting stays inside a block, there is
                                     none between blocks): at every step the pivot is the
                                     entry of largest magnitude left on the diagonal of the
                                     current Schur complement within the group (the first
                                     on ties), P A P^T = L D L^T.  perm[j] = index of the
                                     input row/column that stands at position j, so
                                     A[perm][:, perm] = L D L^T; `diag` receives the
                                     pivots in that order.  log|det| and sign are those of
                                     A.  An exact zero left as the largest candidate ends
                                     the call with MDET_ESINGULAR (a matrix like
                                     [[0, 1], [1, 0]] would need a 2 x 2 pivot, which is
                                     not provided).  The stored factor S (overwrite = 1)
                                     holds L with the rows of every group left in input
                                     order for the columns before the group: A = M D M^T
                                     with M = S except that row perm[j] of each diagonal
                                     64 x 64 block of M is row j of that block of S.
                                     Costs one more launch per 64 columns; n < 2^31; not
                                     with MDET_FLAG_ASSUME_SPD (MDET_EINVAL).  The group of
                                     64 is this library's unit of factorisation, smaller
                                     than the paper's block: MDET_FLAG_PIVOT_BLOCK searches
                                     the whole diagonal block instead, at a price.       */

#define MDET_FLAG_PIVOT_BLOCK 256u /* symmetric pivoting over the whole diagonal block (Sec. 2.2:
                                     pivoting within each block, none between blocks): as
                                     MDET_FLAG_PIVOT, but at every step the candidates are ALL
                                     entries left on the diagonal of the current Schur
                                     complement inside the block column's own b x b diagonal
                                     block (b = block_size_used), not only those of a group
                                     of 64.  perm, diag, sign, log|det| as for MDET_FLAG_PIVOT;
                                     the stored factor (overwrite = 1) holds, in each diagonal
                                     b x b block, L and D of that block in pivot order, the
                                     rows left of it in input order.  1 x 1 pivots only: a
                                     block whose diagonal is exhausted by zeros ([[0, 1],
                                     [1, 0]]) ends the call with MDET_ESINGULAR.  Costs one
                                     small launch per elimination step (about 0.3 ms per 64
                                     columns) and workspace for two b x b arrays and one
                                     (n - b) x b array, counted by mdet_plan; every entry
                                     point takes it; not with MDET_FLAG_PIVOT,
                                     MDET_FLAG_ASSUME_SPD or MDET_FLAG_GENERAL (MDET_EINVAL),
                                     b <= 16384.                                          */

#define MDET_FLAG_GENERAL 128u    /* the matrix is not symmetric (Sec. 2.2, Eq. 1 and Alg. 1:
                                     M = P L U for generic matrices, with pivoting inside a
                                     block and none between blocks), fp32 or fp64 in their
                                     own arithmetic; MDET_FLAG_ASSUME_SPD, MDET_FLAG_PIVOT and
                                     MDET_FLAG_COMPUTE_F64 with it give MDET_EINVAL.  All
                                     n x n entries of the input are read.  Gaussian elimination in the order of the symmetric
                                     path (block columns, leaves of 64); in column j the pivot
                                     is the entry of largest magnitude among the rows j .. end
                                     of j's group of 64 consecutive rows (the first on ties),
                                     and the two rows change places.  The factors are kept
                                     as P A = L D U, L unit lower and U unit upper
                                     triangular; log|det| = sum log|d_j|, sign = the
                                     permutation's sign times the pivots' signs.
                                     `diag` receives d; perm (as for MDET_FLAG_PIVOT, n
                                     int32) the row order: perm[j] = row of
                                     the input that stands at position j inside its group.
                                     As in the symmetric pivoted form the exchanges are not
                                     applied to the columns left of a group, so with
                                     overwrite = 1 the array returns S = L below the
                                     diagonal with the rows of every group in input order
                                     left of the group, d on the diagonal and U above it:
                                     A[perm] = L' D U with L' = S's lower part, rows of each
                                     diagonal 64-block's columns already in pivot order.
                                     mdet_logdet_device: one more array of the matrix's shape
                                     in the workspace (the entries above the diagonal are
                                     kept transposed, so that both triangles are read along
                                     rows), counted by mdet_plan and mdet_workspace_query.
                                     mdet_logdet_host and mdet_logdet_file (the
                                     memory-constrained generic case of Alg. 1): the caller
                                     supplies both triangles in that form, the packed lower
                                     block-column layout of M followed by the packed lower
                                     block-column layout of M^T (diagonal blocks complete in
                                     the first, only their strictly lower part read in the
                                     second); block columns of both are resident, streamed
                                     and written back together, so every figure of the plan
                                     (device bytes, traffic, host scratch) is twice the
                                     symmetric one; with overwrite = 1 a streamed run leaves
                                     L and D in the first layout and U^T (unit) in the second.
                                     mdet_logdet_provider: the callback is asked for the
                                     blocks of both triangles (see mdet_block_provider), plus
                                     a staging buffer of at most 64 MiB on the device.
                                     A column whose candidates are all zero ends the call with
                                     MDET_ESINGULAR.                                     */

typedef struct mdet_result {
  double logabsdet;            /* log|det A|; -inf when sign == 0                    */
  int32_t sign;                /* -1, 0, +1 (numpy.linalg.slogdet convention)        */
  int32_t hip_error;           /* raw hipError_t of the failing call, else 0         */
  int64_t bad_pivot_index;     /* first zero / non-finite pivot, else -1             */
  int64_t negative_pivots;     /* number of d_j < 0 (not an error: Sec. 2.2 explains
                                  why LDL^T is preferred to Cholesky)                */
  int64_t block_size_used;     /* b after rounding                                   */
  int64_t num_blocks;          /* n_b = ceil(n / b)                                  */
  int32_t out_of_core;         /* 1 if blocks were streamed from host memory         */
  int32_t num_superpanels;     /* out-of-core: number of resident column groups      */
  double flops;                /* fused multiply-adds x 2 actually launched          */
  double t_total;              /* seconds, wall clock of the call                    */
  uint64_t bytes_h2d;          /* host -> device bytes moved                         */
  uint64_t bytes_d2h;          /* device -> host bytes moved                         */
  uint64_t dev_bytes_high_water; /* highest workspace offset the call used, in bytes
                                    (the arena is carved group by group; <= budget and
                                    <= mdet_plan's dev_bytes_needed)                  */
  uint64_t kernel_launches;
  /* filled when MDET_FLAG_PROFILE is set: the Schur updates of the trailing matrix */
  uint64_t trailing_update_launches;
  double t_trailing_update;      /* seconds, sum of the launches' event-timed durations */
  double trailing_update_flops;  /* 2 x multiply-adds those launches performed          */
  /* filled by the host entry points when MDET_FLAG_PROFILE is set: time the host link
     was busy in each direction (sum of the copies' event-timed durations, seconds) */
  double t_h2d;
  double t_d2h;
  /* MDET_FLAG_PROFILE, continued: the same three figures for the 64 x 64-block variant of
     the trailing-update kernel (updates too small to fill the device with 128 x 128
     blocks), and the time during which at least one trailing-update launch of either
     kernel was running (the union of the launches' intervals: launches on the library's
     two compute streams overlap, so the sums above count some time twice) */
  uint64_t trailing_update64_launches;
  double t_trailing_update64;
  double trailing_update64_flops;
  double t_trailing_update_busy;
} mdet_result;

/*
 * Block provider (the paper's "matrix stored on disk, may not be loaded on
 * memory", App. D): called by mdet_logdet_provider from the calling thread to fetch
 * the stored-triangle block with block coordinates (bi, bj), bi >= bj, i.e. rows
 * [bi*b, bi*b+rows) x columns [bj*b, bj*b+cols) with b = block_size_used.  It must
 * write the block row-major with leading dimension `ld` elements into the HOST
 * buffer `dst` (pinned memory owned by the library) and return 0; any other
 * return value aborts the call with MDET_EPROVIDER.  For diagonal blocks only the
 * lower triangle need be filled.  Every block is asked for exactly once, block columns in
 * ascending order within a resident group, elements of params->dtype.
 * With MDET_FLAG_GENERAL (Sec. 2.2, Eq. 1: generic matrices) the blocks of both triangles
 * are asked for, bi < bj included and diagonal blocks in full, each still exactly once:
 * block (bj, bi) right after block (bi, bj); the library transposes the upper ones on the
 * device.
 */
typedef int (*mdet_block_provider)(void* user, int64_t bi, int64_t bj, int64_t rows,
                                   int64_t cols, void* dst, int64_t ld);

/* Host planner (no GPU needed): what a call with these parameters would do. */
typedef struct mdet_plan_info {
  int64_t block_size_used;
  int64_t num_blocks;           /* n_b                                              */
  int32_t out_of_core;          /* host entry points: 0 in-core, 1 streamed          */
  int32_t num_superpanels;      /* groups of block columns resident at a time        */
  uint64_t dev_bytes_needed;    /* device workspace the call will use (<= budget)    */
  uint64_t host_bytes_needed;   /* pinned scratch needed when overwrite == 0         */
  uint64_t host_matrix_bytes;   /* size of the packed lower block-column layout      */
  uint64_t stream_bytes_h2d;    /* predicted host->device traffic                    */
  uint64_t stream_bytes_d2h;    /* predicted device->host traffic                    */
  double fma_decomp, fma_solve, fma_gemm, fma_syrk; /* App. E.1, Table "complexity"  */
} mdet_plan_info;

/*
 * mdet_plan: computes the block grid and residency plan for an n x n matrix in the
 * packed host layout (see mdet_logdet_host) under params->mem_budget_bytes, and
 * the work split of App. E.1.  `for_device_input` != 0 plans mdet_logdet_device
 * instead (matrix already in HBM).  Pure host code.  Returns MDET_EBUDGET when the
 * budget cannot hold the minimum working set.
 */
int mdet_plan(const mdet_params* params, int for_device_input, mdet_plan_info* info);

/* Device / pinned-host scratch sizes a call needs (subset of mdet_plan). */
int mdet_workspace_query(const mdet_params* params, int for_device_input,
                         uint64_t* dev_bytes, uint64_t* host_bytes);

/*
 * mdet_logdet_device: matrix resident in HBM.
 *   dA    DEVICE pointer, n x n row-major with leading dimension ld >= n elements
 *         of params->dtype; only the lower triangle is read.  With overwrite = 1
 *         it is factored in place; with overwrite = 0 the library works on a copy
 *         in its workspace (n*ld_padded elements are then part of the workspace).
 *   diag  optional DEVICE pointer to n elements of params->dtype receiving the
 *         pivots d_j (cumulative sums of log|d_j| are the log-determinants of the
 *         leading principal sub-matrices, App. D); NULL to skip.
 * Caller owns every buffer.  Errors: see mdet_status.
 */
int mdet_logdet_device(const mdet_params* params, void* dA, int64_t ld,
                       mdet_result* result, void* diag);

/*
 * mdet_logdet_device_noalloc: mdet_logdet_device for callers that cannot allocate device
 * memory or wait: code that records its work into a HIP graph, tight serving loops, harnesses
 * that forbid hipMalloc.  The call allocates and frees nothing on the device or through the
 * runtime (no stream, no event) and does not synchronise: it only queues kernels and two
 * device-to-device copies on params->stream, all in order on that one stream (the schedule of
 * MDET_FLAG_NO_LOOKAHEAD, whose results are bit-identical to the two-stream schedule).  The
 * small workspace of the path (pivots, their reciprocals, leaf inverses, flags, partial sums,
 * permutation) lives in a fixed array of MDET_NOALLOC_SCRATCH_BYTES in device memory that
 * belongs to the library; each GPU the library runs on holds its own copy until the process
 * ends.  Hence:
 *   - n is limited by that array: about 16 n + 64 KiB bytes in fp64 (8 n in fp32, 4 n more
 *     with MDET_FLAG_PIVOT), i.e. n <= ~250 000; beyond it MDET_ENOMEM_DEVICE.
 *   - overwrite must be 1 (the matrix is factored in place; rows 16-byte aligned), and of the
 *     flags only MDET_FLAG_ASSUME_SPD and MDET_FLAG_PIVOT are taken; mem_budget_bytes,
 *     dev_workspace and host_scratch are ignored.  Anything else: MDET_EINVAL.
 *   - all calls on one GPU share the array, which keeps the last call's contents (what must
 *     start clean is cleared by the call itself): calls that overlap on one GPU, on whatever
 *     streams, race.  Calls on different GPUs do not.
 *   dA, ld, diag (DEVICE, n elements of dtype or NULL), params->perm (DEVICE): as for
 *   mdet_logdet_device.
 *   out   DEVICE pointer to 5 doubles, valid once the stream has run the work: [0] log|det A|,
 *         [1] sign, [2] number of negative pivots, [3] index of the first zero or non-finite
 *         pivot (-1: none), [4] the mdet_status the synchronous entry point would have
 *         returned (MDET_OK, MDET_ESINGULAR, MDET_ENONFINITE, MDET_ENOTPOSDEF), with [0], [1]
 *         set as that entry point sets logabsdet and sign.
 * Returns MDET_OK when everything was queued.
 */
#define MDET_NOALLOC_SCRATCH_BYTES (4ull << 20)
int mdet_logdet_device_noalloc(const mdet_params* params, void* dA, int64_t ld, double* out,
                               void* diag);

/*
 * mdet_logdet_host: matrix in HOST memory (pinned or not: memory that is not pinned
 * is moved through pinned chunks of the library's own, by a few threads that live for
 * the length of the call), in the packed lower block-column layout:
 * with b = block_size rounded up to a multiple of 64 and n_b = ceil(n/b), block
 * column j (columns [j*b, min(n, (j+1)*b)), width w_j) stores rows [j*b, n)
 * row-major with leading dimension w_j, and block columns follow each other:
 *      offset_j = sum_{t<j} (n - t*b) * w_t      (elements)
 * (use mdet_host_layout_offset).  Entries above the diagonal inside the diagonal
 * blocks are never read.  If the whole layout plus workspace fits in
 * mem_budget_bytes the factorisation runs in-core; otherwise block columns are
 * processed in resident groups while already-factored blocks stream in from the
 * host over side streams, and factored groups are written back (to hA when
 * overwrite = 1, to host scratch otherwise).
 *   diag  optional HOST pointer to n elements of params->dtype.
 */
int mdet_logdet_host(const mdet_params* params, void* hA, mdet_result* result,
                     void* diag);

/* As mdet_logdet_host, but the original blocks are fetched through `provider` (e.g. from
 * disk), each when the schedule first needs it, into one of two pinned buffers of one block
 * and from there to the device: host memory holds no copy of the matrix.  Only a run that
 * streams keeps its factored block columns in host memory (params->host_scratch, or memory the
 * library allocates: mdet_workspace_query's host_bytes with overwrite = 0).  overwrite is
 * ignored. */
int mdet_logdet_provider(const mdet_params* params, mdet_block_provider provider,
                         void* user, mdet_result* result, void* diag);

/* The block provider for blocks that are PRODUCED ON THE DEVICE (a kernel matrix or a Gram
 * matrix formed block by block, App. D: the matrix need never exist in one piece): the callback
 * is handed `dst`, a DEVICE pointer into the library's workspace where block (bi, bj), bi >= bj,
 * belongs (rows x cols, row-major, leading dimension ld elements of params->dtype; for diagonal
 * blocks only the lower triangle need be filled), and `stream`, a hipStream_t: it must queue on
 * that stream the kernels or copies that fill the block and return 0 without waiting for them;
 * any other return value ends the call with MDET_EPROVIDER.  Every block is asked for exactly
 * once, when the schedule first needs it, as for mdet_block_provider.  Nothing of the matrix
 * crosses the host link; a run that streams still keeps its factored block columns in host
 * memory (params->host_scratch or the library's own).  MDET_FLAG_COMPUTE_F64 and
 * MDET_FLAG_GENERAL are not taken (MDET_EINVAL); `diag` is a HOST pointer. */
typedef int (*mdet_block_provider_device)(void* user, int64_t bi, int64_t bj, int64_t rows,
                                          int64_t cols, void* dst, int64_t ld, void* stream);
int mdet_logdet_provider_device(const mdet_params* params, mdet_block_provider_device provider,
                                void* user, mdet_result* result, void* diag);

/* As mdet_logdet_host, with the matrix in a FILE (the paper's third tier, Sec. 2.2: the
 * matrix lives on disk, blocks are loaded as needed, a scratchpad on disk takes the
 * updated blocks; the software appendix: scratch_dir, parallel_io): `matrix_path` holds
 * the packed lower block-column layout, elements of params->dtype, from byte 0.  Blocks
 * are read (and, when the run streams, factored block columns written and read again)
 * with pread/pwrite by a few threads at a time, through pinned chunks; host memory use
 * does not grow with the matrix.
 *   overwrite = 1  the factored block columns go back into matrix_path (when the whole
 *                  matrix fits the budget nothing is written at all);
 *   overwrite = 0  matrix_path is opened read-only and, if the run streams, the factored
 *                  block columns go to `scratch_path`, which is created or overwritten
 *                  (MDET_EINVAL if it is NULL then); host_scratch is ignored.
 *   diag, params->perm  HOST pointers as for mdet_logdet_host.
 * MDET_EIO if a file cannot be opened, is too short, or a read or write fails. */
int mdet_logdet_file(const mdet_params* params, const char* matrix_path,
                     const char* scratch_path, mdet_result* result, void* diag);

/* Element offset of block column j in the packed host layout; total elements for
 * j = n_b.  b must already be a multiple of 64.  Returns -1 on bad arguments. */
int64_t mdet_host_layout_offset(int64_t n, int64_t b, int64_t j);

/* The paper's rule for the number of blocks from a memory cap (App. D: r = m
 * sqrt(beta/c); n_b = 1, 2 or ceil(2r); b = 1 + floor((m-1)/n_b)).  Provided for
 * reference and comparison; the library's own plan is mdet_plan. */
int mdet_paper_block_rule(int64_t m, int32_t beta, uint64_t c, int64_t* n_b, int64_t* b);

/* Closed-form operation count of App. E.1 for the symmetric case, in fused
 * multiply-adds: m^3/6 - m^2/4 + m/12. */
double mdet_paper_fma_count(int64_t m);

/*
 * Single steps of the path, exposed for tests and benchmarks.  All pointers are
 * DEVICE pointers to elements of `dtype`; matrices are row-major; `stream` is a
 * hipStream_t or NULL; the calls are asynchronous (enqueue only) and return
 * MDET_EINVAL on misaligned or inconsistent arguments (leading dimensions and
 * base pointers must keep rows 16-byte aligned, K must be a multiple of 64).
 */

/* Trailing Schur-complement update (Sec. 2.2, S <- S - C B with the diagonal
 * scaling of the LDL^T case):  C[M x N] -= A[M x K] diag(d[K]) B[N x K]^T.
 * lower != 0: C's (0,0) lies on the matrix diagonal and only entries with
 * column <= row are computed and stored (Gramian / lower-triangle case).
 * d == NULL: no scaling, C -= A B^T (the positive-definite form). */
int mdet_step_schur_update(int32_t dtype, void* C, int64_t ldc, const void* A,
                           int64_t lda, const void* B, int64_t ldb, const void* d,
                           int64_t M, int64_t N, int64_t K, int32_t lower, void* stream);

/* Factor one block column in place: P points at its diagonal entry; the panel has
 * m rows and w <= m columns.  On return the top w x w block holds L (strictly
 * lower) and D (diagonal), the rows below hold L_ik = A_ik L_kk^-T D_k^-1, and
 * d[w], dinv[w] hold the pivots and their reciprocals.  flags: device pointer to
 * 16 + 8192 bytes; the first two uint64 must be preset to all-ones: [0] receives
 * the smallest index (pivot_index0 + column) of a zero or non-finite pivot, [1] its
 * kind (1 zero, 2 non-finite); the remaining 8192 bytes are scratch. */
int mdet_step_panel_factor(int32_t dtype, void* P, int64_t ld, int64_t m, int64_t w,
                           void* d, void* dinv, int64_t pivot_index0, void* flags,
                           void* stream);

/* The same with pivoting inside each 64-column leaf (MDET_FLAG_PIVOT): perm receives
 * w int32, perm[j] = pivot_index0 + (row of P, counted from its first, that stands at
 * position j); on return the top w x w block holds L and D of the permuted block and the
 * rows below hold their columns in that order. */
int mdet_step_panel_factor_pivoted(int32_t dtype, void* P, int64_t ld, int64_t m, int64_t w,
                                   void* d, void* dinv, int32_t* perm, int64_t pivot_index0,
                                   void* flags, void* stream);

/* One block column of a general matrix (MDET_FLAG_GENERAL; Sec. 2.2, Eq. 1 and Alg. 1:
 * M = P L U, pivoting inside a block).  The block column is given as two panels of m rows
 * and w <= m columns with the same leading dimension, both DEVICE pointers: P points at
 * the diagonal entry of the entries on and below the diagonal, Q at the same place of the
 * transposed entries above it (Q[i][j] = M[j][i] for i > j; its diagonal and everything
 * above the diagonal of either panel is not referenced).  Q - P must be a non-zero multiple
 * of 16 bytes.  On return P holds L (unit lower, strictly below the diagonal) and D on the
 * diagonal, Q holds U^T (unit upper U, M[perm] = L D U on these columns), the rows of every
 * 64-row group left in input order for the columns left of the group; d[w], dinv[w] the
 * pivots and their reciprocals; perm[w] the row order as for
 * mdet_step_panel_factor_pivoted.  flags: DEVICE pointer to 32 + 2 * 8192 bytes; uint64
 * [0] and [1] preset to all-ones receive the first bad pivot and its kind as above, [2]
 * preset to zero receives the number of 64-row leaves whose row order is an odd
 * permutation (the sign of P is -1 if that number is odd); the rest is scratch. */
int mdet_step_panel_factor_general(int32_t dtype, void* P, void* Q, int64_t ld, int64_t m,
                                   int64_t w, void* d, void* dinv, int32_t* perm,
                                   int64_t pivot_index0, void* flags, void* stream);

/* sum log|d_j|, sign and negative count of d[0..n) -> out[0] = logabsdet (double),
 * out[1] = sign (as double), out[2] = negative count (as double).  out: DEVICE
 * pointer to at least 8 doubles (the tail is scratch). */
int mdet_step_logdet_reduce(int32_t dtype, const void* d, int64_t n, double* out,
                            void* stream);

/* ------------------------------------------------------------------------
 * Principal-minor sequence and FLODANCE (Sec. 3.2, Alg. 2)
 *
 * The pivots D_ii that the log-determinant calls return in `diag` give the
 * log-determinants of all leading principal blocks, ell_k = sum_{i<=k} log|D_ii|
 * (Sec. 2.1); Alg. 2 fits the curve of Eq. (7) to every d-th of them and
 * extrapolates it.  All pointers below are DEVICE pointers unless said otherwise;
 * the caller owns every buffer; each call only queues kernels on `stream` (the
 * results are there once the stream has run them), allocates nothing and returns
 * MDET_EINVAL for inconsistent arguments, MDET_ENOMEM_DEVICE for a workspace that is
 * too small and MDET_EHIP if a launch failed.  All arithmetic is fp64.
 * ---------------------------------------------------------------------- */

/* Device bytes that the two calls below need as workspace, for a pivot vector of
 * length n and a fit over `rows` = n_s - n_0 samples with q correction terms (pure
 * host code; pass 0 for the part that is not used). */
int mdet_sequence_workspace_query(int64_t n, int64_t rows, int32_t q, uint64_t* bytes);

/* ell[k] = sum_{i<=k} log|d[i]|, k = 0 .. n-1 (Alg. 2, first step): log|det| of the
 * (k+1) x (k+1) leading principal block.  d: n pivots of type dtype; ell: n doubles. */
int mdet_principal_logdets(int32_t dtype, const void* d, int64_t n, double* ell,
                           void* workspace, uint64_t workspace_bytes, void* stream);

/* The regression of Alg. 2 on ell[0 .. len): with L_j = ell[j d - 1] / j it uses
 * n_j = n0 + 1 .. ns (needs 1 <= n0 < ns, ns d <= len, 0 <= q <= 10 and at least
 * q + 2 samples), responses y_j = n_j (n_j-1)^-1/2 (L_{n_j} - L_{n0}) and covariates
 * (n_j-1)^1/2 and -(n_j-1)^-1/2 n_j^(1-i) logGamma(n_j+1), i = 1 .. q+1, and solves
 * the least-squares problem by Householder QR.  coef receives q + 4 doubles:
 * c_0, nu_0 .. nu_q, then L_{n0}, then the residual norm |X beta - y|_2. */
int mdet_flodance_fit(const double* ell, int64_t len, int64_t d, int64_t n0, int64_t ns,
                      int32_t q, double* coef, void* workspace, uint64_t workspace_bytes,
                      void* stream);

/* out[i] = Lhat_n at n = n_values[i] (Alg. 2, last step):
 * L_{n0} + c_0 (1 - 1/n) - sum_{i=1}^{q+1} nu_{i-1} n^-i logGamma(n+1), from the q + 4
 * doubles that mdet_flodance_fit wrote.  n_values, out: `count` doubles each. */
int mdet_flodance_eval(const double* coef, int32_t q, const double* n_values, int64_t count,
                       double* out, void* stream);

/* ------------------------------------------------------------------------
 * Measuring sticks for the benchmark (asynchronous, enqueue only; DEVICE pointers).
 * ---------------------------------------------------------------------- */

/* A plain copy of `bytes` bytes (a multiple of 16, both pointers 16-byte aligned) by one
 * kernel: reads `bytes`, writes `bytes`.  The ratio between what a profiler's memory
 * counters report for it and these known figures calibrates the same counters for the
 * kernels of the path (the traffic figures beside the roofline of the trailing update of
 * Sec. 2.2). */
int mdet_step_copy(void* dst, const void* src, uint64_t bytes, void* stream);

/* Matrix-core instructions on registers only (16 x 16 x 4 products of `dtype`, MDET_F64 or
 * MDET_F32; `accumulators` = 4 or 16 accumulator tiles used in turn, 16 / accumulators
 * dependent products in a row on each): `workgroups` workgroups of four wavefronts, `iters`
 * rounds of 16 products per wavefront.  *flop receives the flops of the launch (2048 per
 * product); `out` needs 65536 elements of dtype (receives values that keep the compiler
 * from dropping the work).  Time it with events: the rate is the matrix pipe's measured
 * ceiling for the Schur update S <- S - C B of Sec. 2.2. */
int mdet_step_mfma_peak(int32_t dtype, int32_t accumulators, int32_t workgroups, int32_t iters,
                        void* out, double* flop, void* stream);

const char* mdet_strerror(int status);
const char* mdet_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MEMDET_H */
