/*
 * tsenor.h - C ABI of the MI355X (gfx950) transposable N:M mask finder.
 *
 * The library computes, for every MxM block of a weight-importance matrix, a 0/1
 * mask with exactly N ones in every row and every column of the block that keeps
 * as much importance as possible (paper Sec. 3, Eq. 1 and Eq. 2).  Each block is
 * relaxed to an entropy-regularised capacitated transport problem (Sec. 3.2,
 * Eq. 4), solved with T Dykstra iterations (Algorithm 1) and rounded to a mask by
 * greedy selection plus swap-based local search (Sec. 3.3, Algorithm 2, Eq. 5).
 *
 * Conventions shared by every entry point
 *   - Every pointer named in a problem is a DEVICE pointer owned by the caller;
 *     the library never frees or keeps them.  The tsenor_problem structs
 *     themselves live in HOST memory and are read before the call returns.
 *   - Work is enqueued on `stream` and is NOT synchronised; outputs are valid
 *     once the stream has reached the end of the enqueued work.
 *   - Return value: TSENOR_OK (0) or a negative tsenor_status.  Every argument of
 *     every problem of a call is validated on the host before anything is enqueued:
 *     on any error but TSENOR_ERR_HIP nothing was enqueued (TSENOR_ERR_HIP reports a
 *     failing launch, after which earlier launches of the call may already be queued).
 *     Inputs must be finite; NaN/Inf weights give unspecified masks.
 *   - Matrices are row-major; element (i, j) of W is W[i * ld + j]; the mask and
 *     the optional plan use leading dimension `cols`.
 *   - rows and cols must be multiples of M (the method never pads, Sec. 3.1);
 *     M must be one of 4, 8, 16, 32, 64 and 0 <= N <= M.  N == 0 and N == M are
 *     answered with the all-zero / all-one mask without iterating (objective_out,
 *     prev_mask and iters_done_out are TSENOR_ERR_UNSUPPORTED for them: there is
 *     nothing to compare or count).
 *   - The arithmetic of the Dykstra iterations, the sort keys and the swap scores
 *     is IEEE double precision on the device (iterations after the fourth in single
 *     precision with TSENOR_FLAG_FP32_ITERATIONS).
 */
#ifndef TSENOR_H
#define TSENOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* opaque stream handle: pass a hipStream_t (NULL = the default stream) */
typedef void* tsenor_stream_t;

typedef enum tsenor_status {
  TSENOR_OK = 0,
  TSENOR_ERR_NULL = -1,        /* a required pointer is NULL */
  TSENOR_ERR_SHAPE = -2,       /* rows/cols <= 0, not multiples of M, ld < cols, or too large (more than 2^40
                                  weights in a matrix, or 2^31 or more blocks of one size in a call) */
  TSENOR_ERR_NM = -3,          /* N < 0 or N > M */
  TSENOR_ERR_UNSUPPORTED = -4, /* M not in {4, 8, 16, 32, 64}, unknown dtype, tau_mode or flag */
  TSENOR_ERR_PARAM = -5,       /* tau <= 0 or not finite, iters < 0, tau out of the supported range */
  TSENOR_ERR_WORKSPACE = -6,   /* workspace NULL, misaligned (256 B) or smaller than tsenor_workspace_bytes */
  TSENOR_ERR_HIP = -7,         /* a HIP call failed; tsenor_last_hip_error() returns the runtime's error code */
  TSENOR_ERR_TOO_LARGE = -8    /* tsenor_mask_ex_static only: the problem needs more than TSENOR_STATIC_SCRATCH_BYTES */
} tsenor_status;

enum { TSENOR_F32 = 0, TSENOR_BF16 = 1 }; /* storage type of W; bf16 is widened exactly */

/* How `tau` forms the log-kernel K of Algorithm 1 (S^(0) = exp(K)):
 *   ABSOLUTE        K_ij = tau * imp_ij, Algorithm 1 line 1 as printed.
 *   REL_MATRIX_MAX  K_ij = imp_ij / (tau * max_ij imp_ij): the entropy weight 1/tau_eff of Eq. 4 is
 *                   tau times the largest importance of this matrix (the parameter choice of
 *                   App. B.1, "0.005 max|W|", read so that it is consistent with Eq. 4).
 * In REL_MATRIX_MAX mode a call starts with a pass over W that finds the maximum; a caller that knows it can
 * pass ABSOLUTE with tau = 1 / (coefficient * maximum) instead and save that kernel (a small launch is then a
 * single kernel).
 * In REL_MATRIX_MAX mode tau must be >= 1/690 (K <= 690 natural-log units), else TSENOR_ERR_PARAM.
 * In ABSOLUTE mode K is not bounded by the call; the supported range is a spread of K of at most ~700
 * inside any one row of a block (column, with TSENOR_FLAG_COLS_FIRST): entries further below their row's
 * largest K are treated as 700 below it, which is exact to double precision unless the iteration count is
 * large enough for the row's scaling to grow by e^700 (N^iters >= e^700). */
enum { TSENOR_TAU_ABSOLUTE = 0, TSENOR_TAU_REL_MATRIX_MAX = 1 };

enum {
  /* Algorithm 2 exactly as printed: at most `local_search_steps` rounds and a swap is applied only
   * when its score is > 0; blocks may then be left with fewer than N ones in some rows/columns.
   * Without this flag local search runs until every row and column holds N ones and applies the
   * best valid swap even if its score is <= 0.  (A valid swap always exists while a row i and a
   * column j are short: greedy leaves S_ij = 1 wherever both are short, so every row with a 0 in
   * column j is full, and its N ones cannot all sit in the fewer than N columns where row i has ones.) */
  TSENOR_FLAG_STRICT_PAPER = 1u << 0,
  /* project onto the column-sum set before the row-sum set (the order of the listing in App. A.2);
   * default is rows first as in Algorithm 1 */
  TSENOR_FLAG_COLS_FIRST = 1u << 1,
  /* Run the Dykstra iterations after the fourth in single precision (single-precision multiplies and
   * adds issue 1.5-1.8 times as fast as double-precision ones on MI355X).  The potentials then carry ~1e-6 of rounding noise: the plan agrees with a
   * double-precision evaluation to ~1e-5 instead of ~1e-13, and the greedy order - hence the mask - can
   * differ from it in a block where two plan entries are closer than that (none in 8192 blocks of the
   * 16:32 test workload).  Sort keys, swap scores and all results stay in double.  Off by default.  A matrix that
   * runs on the small tiles (below) iterates in double whatever this flag says: such a launch is bound by latency,
   * not by instruction issue, and single precision would buy nothing. */
  TSENOR_FLAG_FP32_ITERATIONS = 1u << 2,
  /* Which kernel runs the greedy selection (Algorithm 2 lines 1-6).  Both give the same mask.  One takes
   * one lane per block (fewest instructions: best when tens of thousands of blocks fill the chip), the other
   * M lanes per block and decides M scan entries per step (shortest dependent chain: best for the small
   * calls of a column-by-column pruning loop).  Default: chosen by the number of blocks in the launch.
   * Setting both is an error. */
  TSENOR_FLAG_GREEDY_ONE_LANE = 1u << 3,
  TSENOR_FLAG_GREEDY_M_LANES = 1u << 4,
  /* How the Dykstra kernel spreads a block over lanes.  Same arithmetic, same results up to the order of
   * the additions inside a row or column sum (~1e-15).  LARGE tiles: 32 entries per lane (16 for M <= 8),
   * fewest instructions per entry: best for full matrices.  SMALL tiles (M <= 32, iters > 0, not with
   * TSENOR_FLAG_SIMPLE_ROUNDING; ignored otherwise): 16 entries per lane (4 for M <= 8),
   * more lanes per block, a shorter dependent chain per iteration: best while the launch cannot fill the
   * chip anyway; on them the whole path, Algorithm 2 included, runs in one kernel (the TSENOR_FLAG_GREEDY_* choice
   * does not apply).  Default: chosen by the number of blocks of the matrix (and earlier for the large tiles when
   * TSENOR_FLAG_FP32_ITERATIONS is set, which only they honour).  Setting both is an error. */
  TSENOR_FLAG_TILES_LARGE = 1u << 5,
  TSENOR_FLAG_TILES_SMALL = 1u << 6,
  /* Ablation arm "Simple" of App. B.2.1 in place of Algorithm 2: per block, keep the N largest plan entries
   * of every row, then of what is left the N largest of every column (ties to the lower index).  No local
   * search: rows may keep fewer than N entries (stats_out[3] counts what is missing). */
  TSENOR_FLAG_SIMPLE_ROUNDING = 1u << 7
};

typedef struct tsenor_problem {
  const void* W;          /* device, rows x ld elements of `dtype`; read-only */
  int32_t dtype;          /* TSENOR_F32 or TSENOR_BF16 */
  int64_t rows, cols, ld; /* ld in elements, >= cols */
  const float* col_scale; /* device, optional (NULL = none), length cols: importance = |W_ij| * col_scale[j]
                             as one float multiply (Sec. 4, Wanda-style importance); values must be >= 0 */
  int32_t N, M;           /* keep N of every M, in rows and in columns of every MxM block */
  double tau;             /* > 0, see tau_mode */
  int32_t tau_mode;       /* TSENOR_TAU_ABSOLUTE or TSENOR_TAU_REL_MATRIX_MAX */
  int32_t iters;          /* T of Algorithm 1: exactly this many iterations, no early exit; 0 = round the
                             importance itself */
  int32_t local_search_steps; /* L of Algorithm 2 (paper: 10); the round limit under STRICT_PAPER, and the
                                 threshold of stats_out[2] otherwise */
  uint32_t flags;         /* TSENOR_FLAG_* */
  uint8_t* mask;          /* device out, rows x cols bytes, 1 = keep */
  double* plan_out;       /* device out, optional (NULL = skip): rows x cols doubles, S^(T) of Algorithm 1 */
  double* tau_eff_out;    /* device out, optional: the multiplier tau_eff with K = tau_eff * imp */
  int64_t* stats_out;     /* device out, optional, 4 counters summed over blocks: [0] ones still missing after
                             greedy selection, [1] swaps applied with score <= 0, [2] blocks that needed more
                             than local_search_steps rounds, [3] ones still missing at return (STRICT_PAPER) */

  /* ---- importance transform: the scores the layer-wise pruning frameworks of Sec. 4 hand to Eq. 1.
   *      All of it is float arithmetic in this order: x = W + add_scale * add;  a = |x|;  a = a * col_scale[j];
   *      importance = a (ABS) or a * a (SQUARE).  Zero-initialised fields give importance = |W| * col_scale. */
  const void* add;        /* device, optional (NULL = none): matrix of W's dtype, shape and ld; with add_scale = 1/rho
                             this is the ALPS score (W + V/rho)^2 of Proposition 1 */
  float add_scale;        /* finite; ignored when add is NULL */
  int32_t importance;     /* TSENOR_IMPORTANCE_ABS (0) or TSENOR_IMPORTANCE_SQUARE */

  /* ---- further outputs, all optional (NULL = skip) ---- */
  uint8_t* packed_out;    /* device out, rows x cols/8 bytes: bit (j & 7) of byte j >> 3 of row i is S_ij; needs
                             cols % 8 == 0 */
  void* pruned_out;       /* device out, rows x cols elements of W's dtype, leading dimension cols: x_ij where the
                             mask keeps it, +0 elsewhere (the pruned weights of Sec. 4; the D-update of
                             Proposition 1).  bf16 output rounds x to nearest-even */
  double* objective_out;  /* device out, 2 doubles: [0] sum_ij S_ij * importance_ij of the returned mask (the
                             objective of Eq. 1), [1] the same for prev_mask (0 if none).  Summed block by block in a
                             fixed order: bitwise reproducible from run to run */
  const uint8_t* prev_mask; /* device, optional, rows x cols bytes (0/1): the safeguard of App. A.1 (Assumption 1).
                             If this mask scores strictly higher than the one just found, under the importance of
                             THIS call, it is returned instead (mask, packed_out, pruned_out follow it) */
  double tol;             /* 0 (default): exactly `iters` iterations, as Algorithm 1 is run in the paper's tables.
                             > 0: `iters` is a bound ("maximum iterations"): a block stops after a
                             TSENOR_ADAPTIVE_CHECK_EVERY-th iteration in which every row and column scaling factor
                             (N / row sum, N / column sum) was within tol of 1.  Changes the result by O(tol).
                             With TSENOR_FLAG_FP32_ITERATIONS the factors after the fourth iteration are
                             single-precision numbers: a tol below ~1e-6 is then never met */
  int32_t* iters_done_out; /* device, optional, one int per block (block-row major): iterations that block ran */
} tsenor_problem;

enum { TSENOR_ADAPTIVE_CHECK_EVERY = 4 };

enum { TSENOR_IMPORTANCE_ABS = 0, TSENOR_IMPORTANCE_SQUARE = 1 };

/* Bytes of device scratch that tsenor_mask_ex / tsenor_mask_batched need for these problems
 * (the sum over the batch).  0 on invalid arguments.  The scratch holds what passes between the kernels of
 * the path: the scan order of Algorithm 2 line 1 (two bytes per weight), the mask greedy selection leaves
 * (Algorithm 2 line 6) and per-block objective values of Eq. 1. */
size_t tsenor_workspace_bytes(const tsenor_problem* problems, int count);

/* The whole path (tile load -> Algorithm 1 -> Algorithm 2 -> mask write) for one matrix: Eq. 1 solved block
 * by block (Eq. 2) as in Sec. 3.2 and 3.3.
 * `workspace`: device memory, 256-byte aligned, at least tsenor_workspace_bytes(p, 1) bytes; its contents
 * are scratch.  Calls that overlap in time must not share a workspace. */
int tsenor_mask_ex(const tsenor_problem* p, void* workspace, size_t workspace_bytes, tsenor_stream_t stream);

/* The same for `count` matrices (for example the seven projections of a decoder layer) on one stream.  The
 * problem of Eq. 1 separates into independent blocks (Sec. 3.1, Eq. 2), and so do the blocks of different
 * matrices: problems may differ in every field, and those that share M and the kernel variant (default, fp32
 * iterations, iters == 0, tiling, ...) go through the kernels together, up to 16 matrices per launch: one
 * launch of every kernel serves the whole group.  The kernel variant of a problem is chosen from that problem
 * alone, so the results are those of `count` separate tsenor_mask_ex calls, bit for bit. */
int tsenor_mask_batched(const tsenor_problem* problems, int count, void* workspace, size_t workspace_bytes,
                        tsenor_stream_t stream);

/* Convenience form of the paper's problem statement (Eq. 1; Algorithm 1 and Algorithm 2 with their inputs as
 * printed): fp32 weights, importance |W|, ld = cols, K = tau * |W| (ABSOLUTE), default local search.
 * Allocates its scratch with hipMallocAsync on `stream` and frees it with hipFreeAsync; everything else as
 * tsenor_mask_ex. */
int tsenor_mask(const float* W, int64_t rows, int64_t cols, int N, int M, float tau, int iters, uint8_t* mask,
                tsenor_stream_t stream);

/* tsenor_mask_ex for callers that cannot allocate or pass scratch: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same problems, same kernels, same results; the scratch is a fixed
 * array of TSENOR_STATIC_SCRATCH_BYTES in device memory that belongs to the library (every GPU the library
 * runs on holds its own copy from the first call on that GPU until the process ends).  The call allocates
 * nothing, on the host or on the device, and clears what it needs with a kernel.
 *   - A problem whose tsenor_workspace_bytes exceeds TSENOR_STATIC_SCRATCH_BYTES is refused with
 *     TSENOR_ERR_TOO_LARGE before anything is enqueued (the array holds e.g. a 4096 x 4096 matrix with
 *     M >= 16, or any slab of a column-by-column pruning loop).
 *   - The array of the CURRENT device is used: `stream` must belong to the current device.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU race (also calls on
 *     different streams, and replays of graphs that captured such calls).  Order them on one stream or with
 *     events. */
#define TSENOR_STATIC_SCRATCH_BYTES (48u << 20)
int tsenor_mask_ex_static(const tsenor_problem* p, tsenor_stream_t stream);

/* The hipError_t value of the last HIP failure that a call made by THIS thread reported as TSENOR_ERR_HIP
 * (0 if there was none).  A launch fails, for example, when the pointers or the stream of a call come from
 * another copy of the HIP runtime than the one this library is linked to. */
int tsenor_last_hip_error(void);

const char* tsenor_status_string(int status);
int tsenor_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TSENOR_H */
