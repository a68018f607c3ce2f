/* Drives every function of the oracle once on small, deliberately awkward inputs (strided input,
 * one block, nine candidates with the pruned one, pruned blocks at the ends of the stream, a trace
 * buffer shorter than the run, ties).  Built with -fsanitize=address,undefined by
 * tests/test_oracle_sanitizers.py: every allocation in the oracle is sized exactly, so an index
 * past an array's end, an uninitialised shift or a signed overflow stops the program here.
 * Test infrastructure, like the rest of this folder; it checks no values (the pins do that).   */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sbits_oracle.h"

static uint32_t lcg_state = 12345u;
static float frand(void)                      /* uniform in (-1, 1) */
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)((double)(lcg_state >> 8) / 8388608.0 - 1.0);
}
static uint16_t bf16_of(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

#define NEW(T, n) ((T *)malloc(sizeof(T) * (size_t)(n)))

static void run_matrix(int R, int C, int m, int n, const int32_t *bits, int K, int power)
{
    const int64_t ld = C + 3;                                     /* a pitch wider than the row */
    float *S = NEW(float, R * ld), *Sd = NEW(float, R * C), *Gd = NEW(float, R * C);
    uint16_t *W = NEW(uint16_t, R * ld), *Wp = NEW(uint16_t, R * C);
    float *rs = NEW(float, R), *cs = NEW(float, C);
    int32_t *rp = NEW(int32_t, R), *cp = NEW(int32_t, C);
    for (int64_t i = 0; i < R * ld; ++i) { S[i] = fabsf(frand()) + (i % 7 == 0 ? 0.0f : 0.01f); W[i] = bf16_of(0.05f * frand()); }
    orc_channel_scores(S, R, C, ld, rs, cs);
    (void)orc_canon8(S, C, 1);
    (void)orc_canon8(S, R, ld);
    orc_argsort_desc(rs, R, rp);
    orc_argsort_desc(cs, C, cp);
    {
        const float *members[2] = {cs, cs};
        float *sum = NEW(float, C);
        int32_t *pp = NEW(int32_t, C);
        orc_group_scores(members, 2, C, sum);
        orc_argsort_desc_pieces(sum, C, n, pp);
        orc_argsort_desc_pieces(sum, C, 0, pp);
        free(sum); free(pp);
    }
    orc_gather_bf16(W, R, C, ld, rp, cp, Wp);
    orc_gather_f32(S, R, C, ld, rp, cp, Sd);
    for (int64_t i = 0; i < (int64_t)R * C; ++i) Gd[i] = frand();

    const int64_t N = (int64_t)(R / m) * (C / n);
    float *cost = NEW(float, N * K);
    orc_cost_table_pow(Wp, Sd, R, C, m, n, bits, K, power, cost);
    (void)orc_cost_shift(cost, N, K);
    (void)orc_fx(cost[0], orc_cost_shift(cost, N, K));

    uint8_t *level = NEW(uint8_t, N), *level2 = NEW(uint8_t, N);
    orc_stats st;
    orc_trace tr[3];                                             /* shorter than most runs */
    int64_t ntr = 0;
    const double budgets[3] = {(double)bits[0], 0.5 * (bits[0] + bits[K - 1]), (double)bits[K - 1] + 1.0};
    for (int b = 0; b < 3; ++b)
        for (int init = 0; init < 2; ++init) {
            orc_params prm = {0.3, 0.0, init, 1000};
            (void)orc_allocate(cost, N, bits, K, budgets[b], &prm, level, &st, tr, 3, &ntr);
        }
    orc_params dflt = {0.05, 0.02, 0, 1000};
    (void)orc_allocate(cost, N, bits, K, budgets[1], &dflt, level, &st, NULL, 0, NULL);
    orc_classic_greedy(cost, N, bits, K, budgets[1], level2);
    if (N <= 6) (void)orc_brute_force(cost, (int)N, bits, K, budgets[1], level2);

    float *up = NEW(float, N), *dn = NEW(float, N);
    orc_surrogates(Wp, Gd, R, C, m, n, bits, level, up, dn);
    int64_t nu, nd, bb, ba;
    (void)orc_propose(up, dn, level, N, bits, K, budgets[1], N / 3 + 1, level2, &nu, &nd, &bb, &ba);
    (void)orc_propose(up, dn, level, N, bits, K, (double)bits[K - 1], 1, level2, &nu, &nd, &bb, &ba);

    /* storage: the first and the last block at the lowest candidate (pruned if that is 0 bits) */
    level[0] = 0; level[N - 1] = 0;
    int64_t *off = NEW(int64_t, N + 1);
    orc_offsets(level, N, m, n, bits, off);
    uint8_t *codes = NEW(uint8_t, off[N] > 0 ? off[N] : 1);     /* exactly the stream's size */
    float *scale = NEW(float, N * m), *zero = NEW(float, N * m), *What = NEW(float, (int64_t)R * C);
    orc_pack(Wp, R, C, m, n, bits, K, level, off, 0, codes, scale, zero);
    orc_dequant(codes, scale, zero, level, off, 0, R, C, m, n, bits, What);
    uint16_t *x = NEW(uint16_t, 3 * C);
    double *y = NEW(double, 3 * R);
    for (int i = 0; i < 3 * C; ++i) x[i] = bf16_of(frand());
    orc_mp_gemm(codes, scale, zero, level, off, 0, R, C, m, n, bits, x, 3, y);

    free(S); free(Sd); free(Gd); free(W); free(Wp); free(rs); free(cs); free(rp); free(cp); free(cost);
    free(level); free(level2); free(up); free(dn); free(off); free(codes); free(scale); free(zero);
    free(What); free(x); free(y);
}

int main(void)
{
    const int32_t b19[9] = {0, 1, 2, 3, 4, 5, 6, 7, 8}, b234[3] = {2, 3, 4}, b1[1] = {3}, b048[3] = {0, 4, 8};
    float w[8] = {-1.5f, 2.0f, 0.25f, 7.0f, -3.0f, 0.0f, 1.0f, 4.0f}, sc, ze;
    int32_t q[8];
    for (int b = 0; b <= 8; ++b) orc_quant_group(w, 8, b, q, &sc, &ze);
    orc_quant_group(w, 8, 4, NULL, &sc, &ze);
    run_matrix(8, 8, 8, 8, b19, 9, 2);              /* one block, nine candidates */
    run_matrix(24, 40, 8, 8, b19, 9, 1);            /* ragged against every tree width */
    run_matrix(32, 96, 16, 32, b234, 3, 2);
    run_matrix(16, 64, 8, 64, b1, 1, 2);            /* a single candidate */
    run_matrix(64, 128, 64, 128, b048, 3, 2);       /* one paper-sized block, uneven steps from 0 */
    run_matrix(16, 24, 8, 8, b048, 3, 1);
    puts("oracle sanitize check: ok");
    return 0;
}
