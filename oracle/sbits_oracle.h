/*
 * ScaleBITS bitwidth-allocation search -- CPU ORACLE (test infrastructure).
 *
 * A plain, slow, single-threaded C99 statement of what the search path
 * computes, written from the paper (ScaleBITS, arXiv 2602.17698).  It exists
 * only so that the GPU library can be checked against it.  It shares no code,
 * header, table or helper with the GPU library, and nothing in the product
 * path may call it: only tests, the smoke check and the benchmark's
 * "cpu_baseline" leg do.
 *
 * Conventions used everywhere below
 *   - a weight matrix W is R x C, row-major, rows = output channels, columns =
 *     input channels (paper App. D);
 *   - W holds bfloat16 values as raw uint16_t, converted exactly to float;
 *   - S is the per-weight sensitivity, float, S >= 0 and finite;
 *   - a block is an m x n sub-matrix of the reordered matrix (paper Sec. 4.1,
 *     "Block-wise Weight Partition"); the quantization group is one block row
 *     (group size = block width, paper App. E "impact of block size");
 *   - m and n are powers of two, both >= 8;
 *   - candidate bitwidths c[0] < c[1] < ... < c[K-1], each in 1..8;
 *   - a "level" is an index into the candidate list.
 *   - every floating-point operation is a single IEEE-754 binary32 operation
 *     in round-to-nearest-even; the only fused operations are the ones written
 *     as fmaf().  Build with -ffp-contract=off and without -ffast-math.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py except
 * the trajectory of orc_allocate (which blocks move at which iteration), which
 * the paper does not determine beyond Algorithm 2 itself: "parity unpinned"
 * for that trajectory; its invariants, its optimum on convex tables and its
 * agreement with Algorithm 1 are pinned.
 */
#ifndef SBITS_ORACLE_H
#define SBITS_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- canonical summation --------------------------------------------------
 * CANON8(x[0..L)): pad with +0 to 8*2^p elements; each aligned run of 8 is
 * summed left to right starting from +0; the run sums are combined by an
 * adjacent-pair binary tree.  Used for the channel scores.                   */
float orc_canon8(const float *x, int64_t L, int64_t stride);

/* ---- a1: channel scores (paper Sec. 4.1 "Bi-directional Channel Reordering":
 * each channel aggregates the element sensitivities with the l1 norm).
 * rs[i] = CANON8(|S[i][0..C)|), cs[j] = CANON8(|S[0..R)][j]|).               */
void orc_channel_scores(const float *S, int64_t R, int64_t C, int64_t ld,
                        float *rs, float *cs);

/* ---- a2: permutation = indices by score, descending, ties -> lower index
 * (sensitive channels move to the top-left, paper Sec. 4 / Fig. 3b).
 * Gather form: new[i] = old[perm[i]].                                        */
void orc_argsort_desc(const float *score, int64_t n, int32_t *perm);

/* coupled reordering (App. "Channel Reordering"): summed scores of the coupled dimensions, and the
 * descending order inside consecutive pieces (heads) */
void orc_group_scores(const float *const *member_scores, int n_members, int64_t n, float *out);
void orc_argsort_desc_pieces(const float *score, int64_t n, int64_t piece, int32_t *perm);

/* ---- a3: reorder both directions: out[i][j] = in[rp[i]][cp[j]].           */
void orc_gather_bf16(const uint16_t *W, int64_t R, int64_t C, int64_t ld,
                     const int32_t *rp, const int32_t *cp, uint16_t *out);
void orc_gather_f32(const float *S, int64_t R, int64_t C, int64_t ld,
                    const int32_t *rp, const int32_t *cp, float *out);

/* ---- quantizer: round-to-nearest uniform scalar quantizer on one group
 * (paper Sec. 5 "Implementation": RTN, group size = block width).
 * Asymmetric min-max grid with 2^bits levels:
 *     mn = min, mx = max, Rg = mx - mn, qmax = 2^bits - 1
 *     inv = qmax / Rg, scale = Rg / qmax        (both 0 if inv is not finite)
 *     x = w - mn; q = clamp(rint(x * inv), 0, qmax); what = fma(q, scale, mn)
 * bits = 0 (Sec. 3: the component is pruned): what = 0 for the whole group, stored as
 * q = 0, scale = 0, zero = 0; its change is the weight itself, d = w.
 * q_out (n ints) may be NULL.                                                */
void orc_quant_group(const float *w, int n, int bits,
                     int32_t *q_out, float *scale, float *zero);

/* ---- a5: block x bitwidth cost table on a reordered matrix.
 * cost[(I*(C/n)+J)*K + l] = sum over block (I,J) of S'*(W' - What_l)^2,
 * accumulated in the canonical order:
 *   chunk  E[r][j] : the 8 elements (r, 8j..8j+7) left to right,
 *                    a = fmaf(S', d*d, a) from a = +0, d = fmaf(-q, scale, x)
 *   octet  O[o][j] : adjacent-pair tree over rows 8o..8o+7 of E[.][j]
 *   octet sum      : adjacent-pair tree over j of O[o][.]
 *   block cost     : adjacent-pair tree over o of the octet sums             */
void orc_cost_table(const uint16_t *Wp, const float *Sp, int64_t R, int64_t C,
                    int m, int n, const int32_t *bits, int K, float *cost);
/* The same with the power of the change as an argument: power 2 is the table above, power 1
 * weighs the absolute change instead, a = fmaf(S', |d|, a): the element-wise first-order
 * form of paper Eq. 3 when S' is the absolute gradient.                                  */
void orc_cost_table_pow(const uint16_t *Wp, const float *Sp, int64_t R, int64_t C,
                        int m, int n, const int32_t *bits, int K, int power, float *cost);

/* dynamic-sensitivity surrogates s_up, s_down per block at the blocks' current bitwidths
 * (App. "choice of sensitivity statistics") */
void orc_surrogates(const uint16_t *Wp, const float *Gp, int64_t R, int64_t C, int m, int n,
                    const int32_t *bits, const uint8_t *level, float *s_up, float *s_down);

/* ---- a6-a8: scalable greedy search (paper Algorithm 2) on a cost table ---- */
typedef struct {
    double  gamma0, gammaT;   /* update ratios; paper Sec. 5: 0.05 and 0.02    */
    int32_t init_mode;        /* 0: warm start at floor(B) (Alg. 2 line 2);
                                 1: start at the lowest candidate (Alg. 1)     */
    int32_t max_iters;
} orc_params;

typedef struct {
    int32_t iters, expansions, swaps_ok, swaps_rej;
    int64_t k_final, bits_used, bits_budget;
    int64_t cost_fixed;       /* sum_i FX(cost[i][level_i])                    */
    int32_t cost_shift;       /* FX(v) = llrint(v * 2^cost_shift)              */
    int32_t pad_;
} orc_stats;

/* one record per loop iteration, for the invariant tests */
typedef struct {
    int32_t kind;             /* 0 expansion, 1 swap accepted, 2 swap rejected */
    int32_t pad_;
    int64_t k;                /* batch size in force during this iteration     */
    int64_t n_up, n_dn;       /* blocks raised / lowered (0 if rejected: the
                                 proposal's sizes are in p_up, p_dn)           */
    int64_t p_up, p_dn;       /* proposed sizes                                */
    int64_t bits_before, bits_after;
    int64_t delta_fixed;      /* swap: fixed-point cost change of the proposal */
} orc_trace;

/* returns 0 ok, -1 infeasible budget (avg_bits < c[0]), -2 max_iters hit,
 * -3 bad argument.  level[N] out.  trace may be NULL; at most trace_cap
 * records are written, *n_trace receives the number of iterations.           */
int orc_allocate(const float *cost, int64_t N, const int32_t *bits, int K,
                 double avg_bits, const orc_params *prm, uint8_t *level,
                 orc_stats *stats, orc_trace *trace, int64_t trace_cap,
                 int64_t *n_trace);

/* One step of Algorithm 2 with caller-supplied estimates (the paper's own loop: fresh
 * s_up / s_down every iteration, acceptance by the caller's loss): see the definition. */
int orc_propose(const float *s_up, const float *s_down, const uint8_t *level_in, int64_t N,
                const int32_t *bits, int K, double avg_bits, int64_t k, uint8_t *level_out,
                int64_t *n_up, int64_t *n_dn, int64_t *bits_before, int64_t *bits_after);

/* fixed-point helpers exposed for the tests */
int32_t orc_cost_shift(const float *cost, int64_t N, int K);
int64_t orc_fx(float v, int32_t shift);

/* ---- cross-checks for a6-a8 (tiny instances only) ------------------------- */
/* paper Algorithm 1 on a cost table: start at the lowest candidate, add one
 * candidate step at a time to the block with the largest gain per bit that
 * still fits the budget.                                                     */
void orc_classic_greedy(const float *cost, int64_t N, const int32_t *bits,
                        int K, double avg_bits, uint8_t *level);
/* exhaustive optimum of paper Eq. 1 on a cost table: minimise sum cost subject
 * to sum bits <= floor(avg_bits*N).  Returns the optimal cost (double sum).  */
double orc_brute_force(const float *cost, int N, const int32_t *bits, int K,
                       double avg_bits, uint8_t *best_level);

/* ---- a9: byte offsets and bit-packing -------------------------------------
 * byte_off[i] = sum_{i' < i} m*n*c[level[i']]/8, byte_off[N] = total.        */
void orc_offsets(const uint8_t *level, int64_t N, int m, int n,
                 const int32_t *bits, int64_t *byte_off);
/* One matrix.  level/byte_off/scale/zero/codes are the GLOBAL arrays; this
 * matrix's blocks are block_base .. block_base + (R/m)*(C/n) - 1.
 * Block i's codes start at codes[byte_off[i]]; element e (row-major inside the
 * block) occupies bits [e*c, (e+1)*c) of the block's little-endian bit stream.
 * scale/zero are [block][row in block].                                      */
void orc_pack(const uint16_t *Wp, int64_t R, int64_t C, int m, int n,
              const int32_t *bits, int K, const uint8_t *level,
              const int64_t *byte_off, int64_t block_base,
              uint8_t *codes, float *scale, float *zero);

/* ---- inference with the stored weights (paper Sec. 5.3 "Inference Kernel") ----
 * orc_dequant: the stored matrix What[i][j] = fmaf(q, scale, zero) (fp32).
 * orc_mp_gemm: y[b][i] = sum_j What[i][j] * x[b][j] in float64 (x: bf16 patterns,
 * [batch][C]; y: [batch][R]).  Arguments as orc_pack's outputs.                 */
void orc_dequant(const uint8_t *codes, const float *scale, const float *zero, const uint8_t *level,
                 const int64_t *byte_off, int64_t block_base, int64_t R, int64_t C, int m, int n,
                 const int32_t *bits, float *What);
void orc_mp_gemm(const uint8_t *codes, const float *scale, const float *zero, const uint8_t *level,
                 const int64_t *byte_off, int64_t block_base, int64_t R, int64_t C, int m, int n,
                 const int32_t *bits, const uint16_t *x, int batch, double *y);

#ifdef __cplusplus
}
#endif
#endif
