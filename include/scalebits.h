/*
 * libscalebits -- the data-parallel hot path of ScaleBITS' global bitwidth
 * allocation search (arXiv 2602.17698), hand-written HIP for gfx950 (MI355X).
 *
 * The calls follow the paper's statement of the problem (Sec. 2.1, Eq. 1): a
 * partition of the weights into components, a candidate precision set, a
 * budget B in bits per weight and a quantizer.  Weights, per-weight
 * sensitivity, block shape, candidate bitwidths and budget go in;
 * permutations, per-block bitwidths and packed codes with scales come out.
 *
 * General conventions
 *   - Every tensor argument is DEVICE memory owned by the caller unless the
 *     comment says HOST.  The library allocates no device memory; scratch is
 *     the caller's workspace `ws` of sbits_workspace_bytes() bytes, 256-byte
 *     aligned.  Calls that share a workspace must not overlap in time.
 *   - A context and its plans keep small host-side tables that calls fill in on
 *     first use: calls on one context (or on plans of one context) must not run
 *     concurrently from several host threads.  Different contexts are independent.
 *   - All work is enqueued on the stream given to sbits_create() and the call
 *     returns without waiting, except where stated (sbits_allocate and
 *     sbits_search wait for the stream because they return host results).
 *   - A weight matrix is rows x cols, row-major, rows = output channels,
 *     cols = input channels (paper App. D); weights are bfloat16, sensitivities
 *     are float32, non-negative and finite.  Weights are finite and max - min
 *     over a quantization group is finite in fp32 (true whenever |w| < 1.7e38).
 *     The kernels are compiled not to honour NaN: with NaN/Inf inputs, or a
 *     group range that overflows, the results are undefined.  Ranges of zero
 *     and ranges so small that qmax / range overflows are defined cases
 *     (scale = 0: every code 0, the group dequantizes to its minimum).
 *     Every call that takes matrices requires rows that start on 16-byte
 *     boundaries: w_bf16 and sens 16-byte aligned, ld_w a multiple of 8, ld_s a
 *     multiple of 4, ld >= cols (else SBITS_ERR_INVALID_ARG).
 *   - A block is block_rows x block_cols (m x n) of the REORDERED matrix and is
 *     the unit of precision (paper Sec. 4.1).  The quantization group is one
 *     block row: group size = block width (paper App. E, block size).  m and n
 *     are powers of two, 8 <= m <= 1024, 8 <= n <= 512; rows % m == 0 and
 *     cols % n == 0; rows, cols <= 32768 per matrix; at most 2^24 blocks in all.
 *   - Blocks are numbered globally: matrix after matrix in plan order, inside a
 *     matrix row-major over the block grid: id = base(mat) + I*(cols/n) + J.
 *   - Candidate bitwidths are strictly increasing integers in 0..8 (so at most
 *     9 of them, at least one above 0).  A "level" is an index into that list.
 *     0 bits means the block is pruned (paper Sec. 3: b_i = 0 removes the
 *     component): its stored value is 0 everywhere, so its cost is the sum of
 *     s * w^2 over the block, it occupies no bytes of the code stream, its scale
 *     and zero entries are written as 0, sbits_dequant returns zeros for it and
 *     sbits_mp_gemm skips it; its surrogates are s_up = sum g*w and s_down = 0.
 *   - Permutations are in gather form: reordered[i] = original[perm[i]].
 *   - Return value: 0 (SBITS_OK) or a negative sbits_status; nothing throws or
 *     aborts; outputs are undefined after an error.
 */
#ifndef SCALEBITS_H
#define SCALEBITS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SBITS_OK                   =  0,
    SBITS_ERR_INVALID_ARG      = -1,  /* null pointer, index out of range, misaligned workspace */
    SBITS_ERR_BAD_SHAPE        = -2,  /* block shape not a supported power of two, or not dividing the matrix */
    SBITS_ERR_BAD_BITWIDTHS    = -3,  /* empty, more than 9, not strictly increasing, outside 0..8, only 0 */
    SBITS_ERR_INFEASIBLE_BUDGET= -4,  /* avg_bits below the smallest candidate */
    SBITS_ERR_WORKSPACE        = -5,  /* workspace smaller than the call needs (sbits_set_workspace_size), or a
                                         plan beyond the fixed scratch of sbits_offsets_static */
    SBITS_ERR_MAX_ITERS        = -6,  /* search stopped by max_iters; levels are valid and within budget */
    SBITS_ERR_HIP              = -7,  /* a HIP call failed; sbits_last_hip_error() has its code */
    SBITS_ERR_UNIMPLEMENTED    = -8,
    SBITS_ERR_CAPACITY         = -9,  /* an output buffer (codes) is too small */
    SBITS_ERR_INTERNAL         = -10  /* a consistency check of the library's own bookkeeping failed */
} sbits_status;

typedef struct sbits_ctx  sbits_ctx;    /* device + stream; small host state only           */
typedef struct sbits_plan sbits_plan;   /* shapes, block numbering, candidate list (host)   */

/* One weight matrix and its sensitivity. ld_* are row pitches in elements.  */
typedef struct {
    const void  *w_bf16;   /* DEVICE, rows x cols bfloat16                                   */
    const float *sens;     /* DEVICE, rows x cols float32, element sensitivity (paper Eq. 3
                              evaluated by the caller; static input here)                    */
    int64_t rows, cols, ld_w, ld_s;
} sbits_matrix;

/* Hyper-parameters of the scalable greedy search (paper Algorithm 2, Sec. 5). */
typedef struct {
    double  gamma0;     /* initial update ratio, k = floor(gamma0*N); paper: 0.05            */
    double  gammaT;     /* stop when k < floor(gammaT*N); paper: 0.02                         */
    int32_t init_mode;  /* 0: warm start, every block at the largest candidate <= floor(B)
                              (Alg. 2 line 2);  1: every block at the smallest candidate
                              (Alg. 1 line 2)                                                 */
    int32_t max_iters;  /* hard cap on loop iterations (>= 1)                                 */
} sbits_params;

typedef struct {
    int32_t iters, expansions, swaps_ok, swaps_rej;
    int64_t k_final;       /* batch size when the loop ended                                 */
    int64_t bits_used;     /* sum over blocks of the chosen bitwidth                         */
    int64_t bits_budget;   /* floor(avg_bits * N)  (Eq. 1, all blocks have equal size)       */
    int64_t cost_fixed;    /* sum_i FX(cost[i][level_i]), FX(v) = rint(v * 2^cost_shift)     */
    int32_t cost_shift;
    int32_t pad_;
} sbits_stats;

/* One record per loop iteration of sbits_allocate (optional, for inspection). */
typedef struct {
    int32_t kind;          /* 0 expansion, 1 swap accepted, 2 swap rejected                  */
    int32_t pad_;
    int64_t k;
    int64_t n_up, n_dn;    /* blocks raised / lowered (0 when rejected)                      */
    int64_t p_up, p_dn;    /* sizes of the proposal                                          */
    int64_t bits_before, bits_after;
    int64_t delta_fixed;   /* swap: fixed-point cost change of the proposal                  */
} sbits_trace;

/* Result of sbits_propose. */
typedef struct {
    int32_t kind;          /* 0 nothing to propose, 1 expansion, 2 balanced swap             */
    int32_t pad_;
    int64_t n_up, n_dn;    /* blocks raised / lowered in level_out                           */
    int64_t bits_before, bits_after, bits_budget;   /* sum of bitwidths over blocks; floor(avg_bits * N) */
} sbits_proposal;

/* ---- context ---------------------------------------------------------------
 * device >= 0: HIP device ordinal; hip_stream: a hipStream_t (NULL = the null
 * stream).  device == -1 creates a host-only context: plans, sizes and argument
 * validation work, every call that would touch the GPU returns SBITS_ERR_HIP.  */
int  sbits_create (sbits_ctx **out, int device, void *hip_stream);
int  sbits_destroy(sbits_ctx *ctx);
int  sbits_last_hip_error(const sbits_ctx *ctx);
const char *sbits_strerror(int status);

/* ---- plan: the partition Pi_w (paper Sec. 2, Sec. 4.1) -----------------------
 * rows/cols: HOST arrays of n_mats entries; bitwidths: HOST array of n_bits.    */
int  sbits_plan_create(sbits_ctx *ctx, const int64_t *rows, const int64_t *cols, int n_mats,
                       int block_rows, int block_cols, const int32_t *bitwidths, int n_bits,
                       sbits_plan **out);
int  sbits_plan_destroy(sbits_plan *plan);
int64_t sbits_num_blocks(const sbits_plan *plan, int mat /* -1: all matrices */);
int64_t sbits_block_base(const sbits_plan *plan, int mat);
size_t  sbits_workspace_bytes(const sbits_plan *plan);
/* Declares how many bytes the workspace that later calls on this plan receive holds.  From
 * then on every call that "uses ws" returns SBITS_ERR_WORKSPACE (on the host, before
 * anything is enqueued) while that size is below sbits_workspace_bytes(plan); this call
 * itself returns SBITS_ERR_WORKSPACE in that case too (the size is recorded anyway).  A
 * plan whose workspace size was never declared is not checked: the pointer alone does not
 * tell its extent.                                                                       */
int  sbits_set_workspace_size(sbits_plan *plan, size_t bytes);
/* upper bound on the packed size in bytes for a budget: floor(avg_bits*N)*m*n/8 */
int64_t sbits_codes_bytes_bound(const sbits_plan *plan, double avg_bits);

/* ---- bi-directional channel reordering (paper Sec. 4.1; per matrix) ----------
 * Channel score = l1 norm of the channel's element sensitivities, summed in the
 * canonical order (runs of 8 left to right, then an adjacent-pair tree, zero
 * padded to a power of two); permutation = channels by score, descending, ties
 * to the lower index.  row_perm[rows], col_perm[cols] out.  Uses ws.            */
int  sbits_reorder(sbits_plan *plan, int mat, const sbits_matrix *M,
                   int32_t *row_perm, int32_t *col_perm, void *ws);
/* the scores alone: row_score[rows], col_score[cols] (float32).  Uses ws.       */
int  sbits_channel_scores(sbits_plan *plan, int mat, const sbits_matrix *M,
                          float *row_score, float *col_score, void *ws);
/* The same for every matrix of the plan in a few launches.  mats: HOST array of the
 * plan's n_mats matrices; row_perm / col_perm: the permutations concatenated in
 * plan order (sum of rows / sum of cols entries).  Uses ws.                       */
int  sbits_reorder_all(sbits_plan *plan, const sbits_matrix *mats,
                       int32_t *row_perm, int32_t *col_perm, void *ws);
/* Coupled reordering (paper Sec. 4.1 last paragraph and App. "Channel Reordering"):
 * matrix dimensions that carry the same activation (the residual stream; the
 * up / gate rows and down columns of one MLP; the value rows and output columns
 * of one attention block) must share ONE permutation, computed from the sum of
 * their channel scores.  row_group[i] / col_group[i] (HOST arrays, n_mats each)
 * give, for the rows / columns of matrix i, SBITS_DIM_INDEPENDENT (own scores, as
 * sbits_reorder_all), SBITS_DIM_FIXED (identity: e.g. query / key rows under rotary
 * embeddings) or a group id in [0, n_groups).  All members of a group must have
 * the group's length times their repeat, see below (else SBITS_ERR_BAD_SHAPE).
 * The group's score of channel j is the fp32 sum of the members' scores of channel j, added member after member in
 * the order: rows of matrix 0, 1, ..., then columns of matrix 0, 1, ...
 * group_segment[g] (HOST, may be NULL = all 0): 0, or a piece length dividing the
 * group's length: channels are then only permuted inside consecutive pieces of
 * that length (attention heads).  Order inside a piece: score descending, ties to
 * the lower index.  Every member receives the same permutation.
 * row_repeat[i] / col_repeat[i] (HOST, n_mats each, may be NULL = all 1): with
 * grouped-query attention one value head feeds r query heads, so the output
 * projection's columns are r times as many as the value projection's rows.
 * A member with repeat r > 1 (needs a segmented group) is r times the group's
 * length; piece p of the group stands for the member's pieces r*p .. r*p + r - 1:
 * their r scores of a channel are added one after the other (lower piece first)
 * where a member with repeat 1 adds one, and each of those pieces receives the
 * permutation of group piece p.  The first member of a group (in the order above)
 * has repeat 1 (else SBITS_ERR_INVALID_ARG); independent and fixed dimensions too.
 * Uses ws.                                                                        */
#define SBITS_DIM_INDEPENDENT (-1)
#define SBITS_DIM_FIXED       (-2)
int  sbits_reorder_coupled_all(sbits_plan *plan, const sbits_matrix *mats,
                               const int32_t *row_group, const int32_t *col_group,
                               int n_groups, const int32_t *group_segment,
                               const int32_t *row_repeat, const int32_t *col_repeat,
                               int32_t *row_perm, int32_t *col_perm, void *ws);
/* w_out[i][j] = W[row_perm[i]][col_perm[j]], s_out likewise; outputs are dense
 * (pitch = cols) and must not alias the inputs.                                 */
int  sbits_gather(sbits_plan *plan, int mat, const sbits_matrix *M,
                  const int32_t *row_perm, const int32_t *col_perm,
                  void *w_out_bf16, float *s_out);

/* All matrices: w_re / s_re receive the reordered matrices concatenated in plan
 * order, each dense (matrix i starts at element sum_{j<i} rows_j*cols_j); either
 * may be NULL.  Permutations concatenated as in sbits_reorder_all.  Uses ws.      */
int  sbits_gather_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                      const int32_t *col_perm, void *w_re_bf16, float *s_re, void *ws);

/* ---- block x bitwidth cost table (paper Sec. 5: RTN quantizer, group = block
 * row; App. E: the exact re-quantized change that the surrogates approximate) --
 * For every block of matrix `mat` and every candidate c_l:
 *   cost[(base+b)*K + l] = sum over the block of s * (w - what_l)^2
 * with what_l the asymmetric min-max round-to-nearest-even grid of 2^c_l levels
 * on each block row (scale = range/qmax, origin = row minimum).  w_re, s_re are
 * the dense reordered matrix (pitch = cols).  `cost` is the GLOBAL table [N][K];
 * the call writes this matrix's rows only.  One HBM pass over w_re and s_re.    */
int  sbits_cost_table(sbits_plan *plan, int mat, const void *w_re_bf16, const float *s_re,
                      float *cost);
/* The power of the change in the cost above is fixed when the library is built: 2 (the
 * default build, libscalebits.so) or 1 (libscalebits_l1.so, built with
 * -DSBITS_COST_POWER=1): cost = sum s * |w - what_l|, the element-wise first-order form
 * of paper Eq. 3 when s is the absolute gradient.  Everything else (grids, summation
 * order, the search on the table) is the same.  Returns the power of this build.     */
int  sbits_cost_power(void);

/* The same for every matrix of the plan in ONE launch.  w_re, s_re: the reordered
 * matrices concatenated in plan order, each dense (matrix i starts at element
 * sum_{j<i} rows_j*cols_j).  Uses ws.                                            */
int  sbits_cost_table_all(sbits_plan *plan, const void *w_re_bf16, const float *s_re,
                          float *cost, void *ws);

/* Reordering and scoring in ONE pass over the ORIGINAL matrices (paper Sec. 4.2
 * reordering followed by the Sec. 5 quantizer, as above): equivalent to
 * sbits_gather_all followed by sbits_cost_table_all, bit for bit, without writing
 * or re-reading the reordered sensitivities.  cost[N][K] is written, and w_re
 * (reordered weights, what sbits_pack_all reads) unless it is NULL:
 * sbits_gather_pack_all does not need it.  Supported for 64- and 128-column
 * blocks, on a device whose memories run with error correction (target id
 * "sramecc+", as every MI355X reports: the kernel relies on how 16-bit register
 * loads behave there); otherwise returns SBITS_ERR_UNIMPLEMENTED and writes
 * nothing: use the two calls above.  The route is chosen per matrix: rows of at
 * most 16384 elements are read once (6 bytes per weight); a matrix with wider
 * rows is reordered into a copy inside the workspace first and scored from there
 * (18 bytes per weight; sbits_workspace_bytes covers the copy of the largest such
 * matrix), with the same bits in the table.
 * sbits_gather_cost_supported: 1 if the plan's shapes qualify (the device is
 * checked by the call itself), else 0.  Uses ws.                                  */
int  sbits_gather_cost_supported(const sbits_plan *plan);
int  sbits_gather_cost_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                           const int32_t *col_perm, void *w_re_bf16, float *cost, void *ws);

/* ---- dynamic-sensitivity surrogates (paper App. "choice of sensitivity
 * statistics", the two displayed equations; Algorithm 2 line 5) ------------------
 * One pass over the ORIGINAL weights and a gradient taken at the currently
 * quantized model (mats[i].sens holds the gradient g here: fp32, any sign, same
 * layout rules as the sensitivity), reordered on the fly like
 * sbits_gather_cost_all.  For every block at its CURRENT bitwidth b =
 * bitwidths[level[i]]:
 *   s_up[i]   = sum over the block of g * (w - what)       what = fma(q, scale, min),
 *   s_down[i] = 2^-b * sum over the block of |g * what|    the dequantized weight
 * (row-group grid and code q as in sbits_pack; sums in the order of the cost
 * table).  level: DEVICE uint8[N]; s_up, s_down: DEVICE float[N].  64- and
 * 128-column blocks and rows of at most 16384 elements (same device rule as
 * sbits_gather_cost_all), else SBITS_ERR_UNIMPLEMENTED.  Uses ws.                 */
int  sbits_surrogates_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                          const int32_t *col_perm, const uint8_t *level,
                          float *s_up, float *s_down, void *ws);

/* ---- scalable greedy search (paper Algorithm 2 with the relaxed step Eq. 5) ---
 * Runs on the device over the cost table: marginal change per bit from the
 * table, radix selection of the top-k / bottom-k sets on (value, index) keys,
 * budget prefix, fixed-point acceptance test.  level[N] out (uint8 candidate
 * index).  host_stats (HOST, may be NULL) and trace (HOST, may be NULL, at most
 * trace_cap records) are filled after the stream has been waited for.
 * Returns SBITS_ERR_INFEASIBLE_BUDGET if avg_bits < smallest candidate,
 * SBITS_ERR_MAX_ITERS if the cap ended the loop.  Uses ws.                      */
int  sbits_allocate(sbits_plan *plan, const float *cost, double avg_bits,
                    const sbits_params *params, uint8_t *level,
                    sbits_stats *host_stats, sbits_trace *host_trace, int64_t trace_cap,
                    void *ws);

/* One step of Algorithm 2 (lines 6-10) on the CALLER's estimates: the paper's own
 * loop re-estimates s_up / s_down from a fresh gradient at every iteration (lines
 * 4-5; sbits_surrogates_all computes them) and tests the loss of the proposal
 * (lines 11-12), which only the caller can evaluate.  s_up[N], s_down[N]: float32,
 * finite; ranked as given (not divided by the width of the step).  level_in[N]:
 * the current levels; level_out[N] (may be level_in): the proposal.
 *   slack = floor(avg_bits * N) - bits in use.
 *   If slack > 0: expansion = the first min(k, eligible) blocks in the order
 *     (s_up descending, lower index first), cut at the first s_up <= 0 and where
 *     the cumulative step bits would exceed the slack; if that set is not empty it
 *     is raised by one candidate each (kind 1; Alg. 2 applies it without a test).
 *   Otherwise: balanced swap with h = max(1, k / 2): U = the first h by s_up,
 *     D = the first h by (s_down ascending, lower index first) outside U, U' = the
 *     longest prefix of U whose step bits fit slack + the bits D frees; if U' and D
 *     are both non-empty, U' is raised and D lowered (kind 2): the caller keeps
 *     level_out if its loss did not increase, else keeps level_in and halves k.
 *   Else kind 0 and level_out = level_in (the caller halves k).
 * The loop ends when k < floor(gammaT * N).  host_out (HOST, may be NULL): filled
 * after waiting for the stream; with NULL the call does not wait.  Uses ws.       */
int  sbits_propose(sbits_plan *plan, const float *s_up, const float *s_down,
                   const uint8_t *level_in, double avg_bits, int64_t k,
                   uint8_t *level_out, sbits_proposal *host_out, void *ws);

/* ---- storage (paper Sec. 5.3: one bitwidth per tile) --------------------------
 * byte_off[i] = sum_{i'<i} m*n*c[level[i']]/8, byte_off[N] = total.  Uses ws.   */
int  sbits_offsets(sbits_plan *plan, const uint8_t *level, int64_t *byte_off, void *ws);
/* The same without a workspace, for callers that cannot allocate device memory or
 * hand one over: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  The scan's partial sums live in a fixed array in the library's
 * device image (32 KiB per GPU, held until the process ends), enough for plans of at
 * most SBITS_OFFSETS_STATIC_MAX_BLOCKS blocks; larger plans get SBITS_ERR_WORKSPACE
 * (checked on the host before anything else, also on a host-only context).  The
 * call allocates nothing and enqueues kernels only; output identical to
 * sbits_offsets.  Every call on one GPU shares that GPU's array: calls that overlap
 * in time on one GPU (two streams, two contexts) race; calls in stream order do not
 * (each call overwrites the part of the array it reads).                          */
#define SBITS_OFFSETS_STATIC_MAX_BLOCKS 8388608
int  sbits_offsets_static(sbits_plan *plan, const uint8_t *level, int64_t *byte_off);
/* Re-quantizes matrix `mat` at the chosen bitwidths and writes, for each of its
 * blocks b (global id), the codes at codes[byte_off[b]...]: element e (row-major
 * in the block) occupies bits [e*c, (e+1)*c) of the block's little-endian bit
 * stream; scale[b*m + r], zero[b*m + r] for block row r (dequantized value =
 * code*scale + zero).  level, byte_off, codes, scale, zero are the GLOBAL arrays.*/
int  sbits_pack(sbits_plan *plan, int mat, const void *w_re_bf16, const uint8_t *level,
                const int64_t *byte_off, uint8_t *codes, float *scale, float *zero);

/* All matrices in one launch; w_re concatenated as in sbits_gather_all.  Uses ws.  */
int  sbits_pack_all(sbits_plan *plan, const void *w_re_bf16, const uint8_t *level,
                    const int64_t *byte_off, uint8_t *codes, float *scale, float *zero, void *ws);

/* The same from the ORIGINAL weights and the permutations (reordering on the fly,
 * no reordered copy needed); identical output.  mats: HOST array, only w_bf16 /
 * ld_w are read.  64- and 128-column blocks (every row length of the plan is read
 * once), any device; otherwise SBITS_ERR_UNIMPLEMENTED.  codes 8-byte, scale and
 * zero 16-byte aligned.  Uses ws.                                                 */
int  sbits_gather_pack_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                           const int32_t *col_perm, const uint8_t *level, const int64_t *byte_off,
                           uint8_t *codes, float *scale, float *zero, void *ws);

/* ---- the whole path in one call -------------------------------------------- */
typedef struct {
    int32_t *row_perm;     /* concatenated over matrices: sum(rows) entries                  */
    int32_t *col_perm;     /* concatenated: sum(cols) entries                                */
    void    *w_re_bf16;    /* reordered weights, matrices concatenated, each dense           */
    float   *s_re;         /* reordered sensitivities, same layout                           */
                           /* Both are needed by the two-pass route only.  When              */
                           /* sbits_gather_cost_supported(plan) and every matrix meets the   */
                           /* alignment rule, s_re is never written and may be NULL, and     */
                           /* w_re_bf16 is written if not NULL (costs one more HBM write).   */
    float   *cost;         /* [N][K]                                                         */
    uint8_t *level;        /* [N]                                                            */
    int64_t *byte_off;     /* [N+1]                                                          */
    uint8_t *codes;        /* codes_capacity bytes (>= sbits_codes_bytes_bound); may be NULL */
                           /* when that bound is 0 (a budget of 0 bits: every block pruned)  */
    int64_t  codes_capacity;
    float   *scale, *zero; /* [N*m] each                                                     */
} sbits_outputs;
/* mats: HOST array of the plan's n_mats matrices.  Waits for the stream.        */
int  sbits_search(sbits_plan *plan, const sbits_matrix *mats, double avg_bits,
                  const sbits_params *params, const sbits_outputs *out,
                  sbits_stats *host_stats, void *ws);
/* The same with coupled reordering (paper Sec. 4.1, App. "Channel Reordering"): the
 * permutations come from sbits_reorder_coupled_all with these groups (same arguments,
 * same errors) instead of sbits_reorder_all; everything after is unchanged.        */
int  sbits_search_coupled(sbits_plan *plan, const sbits_matrix *mats,
                          const int32_t *row_group, const int32_t *col_group, int n_groups,
                          const int32_t *group_segment, const int32_t *row_repeat,
                          const int32_t *col_repeat, double avg_bits,
                          const sbits_params *params, const sbits_outputs *out,
                          sbits_stats *host_stats, void *ws);

/* ---- the stored matrix as numbers (paper Sec. 5.3: uniform bitwidth per tile) ----
 * out[i][j] = fmaf(code, scale, zero) of matrix `mat`, from the packed stream (GLOBAL
 * arrays as written by the packing calls), in the REORDERED coordinates: row i and
 * column j of the matrix the stream was packed from.  out_bf16 = 0: float32 (the
 * format's exact value); 1: rounded to bfloat16, nearest even.  out: [rows][ld_out]
 * elements, 16-byte aligned, ld_out >= cols and a multiple of 8.  Any block shape.  */
int  sbits_dequant(sbits_plan *plan, int mat, const uint8_t *level, const int64_t *byte_off,
                   const uint8_t *codes, const float *scale, const float *zero,
                   void *out, int64_t ld_out, int out_bf16);

/* ---- inference with the stored weights (paper Sec. 5.3 "Inference Kernel") -----
 * y[b][i] = sum_j What[i][j] * x[b][j] for matrix `mat` of the plan, read from the
 * packed stream (the outputs of sbits_pack / sbits_pack_all / sbits_gather_pack_all,
 * the GLOBAL arrays): What[i][j] = code * scale + zero of the element's block row.
 * Dequantization is fused into the product, tile = precision block, one bitwidth
 * per tile.  Rows and columns are the REORDERED ones: x is indexed by the matrix's
 * permuted input channels and y by its permuted output channels (the paper stores
 * the permuted weights and keeps connected layers consistent, App. "Channel
 * Reordering").  x_bf16: [batch][ld_x] bfloat16, 16-byte aligned, ld_x >= cols and a
 * multiple of 8; y: [batch][rows] float32; batch >= 1.  The kernel is built for the
 * small batches of decoding: 32 rows of x per launch, each launch reading the whole
 * code stream of the matrix; for large batches (prefill) take sbits_dequant to bf16
 * once and an ordinary dense product instead.  Products are exact (integer codes
 * times bf16) and summed in fp32 on the matrix cores; scale and zero are applied per
 * block row in fp32.
 * SBITS_ERR_UNIMPLEMENTED unless block_cols is 64 or 128 and block_rows a multiple
 * of 32.  Uses ws.                                                               */
int  sbits_mp_gemm(sbits_plan *plan, int mat, const void *x_bf16, int64_t ld_x, int batch,
                   const uint8_t *level, const int64_t *byte_off, const uint8_t *codes,
                   const float *scale, const float *zero, float *y, void *ws);

#ifdef __cplusplus
}
#endif
#endif /* SCALEBITS_H */
