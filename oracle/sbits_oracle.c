/*
 * ScaleBITS bitwidth-allocation search -- CPU ORACLE (test infrastructure).
 * See sbits_oracle.h for the contract.  Plain C99, single-threaded, no
 * blocking, no fusion beyond the fmaf() calls the definition names.
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include "sbits_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ utils */

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* adjacent-pair binary tree, in place; P is a power of two */
static float pair_tree(float *y, int64_t P)
{
    while (P > 1) {
        for (int64_t j = 0; j < P / 2; ++j)
            y[j] = y[2 * j] + y[2 * j + 1];
        P /= 2;
    }
    return y[0];
}

static int64_t next_pow2(int64_t v)
{
    int64_t p = 1;
    while (p < v) p *= 2;
    return p;
}

/* ---------------------------------------------------------------- CANON8 */

float orc_canon8(const float *x, int64_t L, int64_t stride)
{
    int64_t nchunks = (L + 7) / 8;
    int64_t P = next_pow2(nchunks > 0 ? nchunks : 1);
    float *y = (float *)calloc((size_t)P, sizeof(float)); /* +0.0f padding */
    for (int64_t ch = 0; ch < nchunks; ++ch) {
        float a = 0.0f;
        for (int e = 0; e < 8; ++e) {
            int64_t i = ch * 8 + e;
            float v = (i < L) ? x[i * stride] : 0.0f;
            a = a + v;
        }
        y[ch] = a;
    }
    float r = pair_tree(y, P);
    free(y);
    return r;
}

/* ----------------------------------------------------- a1: channel scores */

void orc_channel_scores(const float *S, int64_t R, int64_t C, int64_t ld,
                        float *rs, float *cs)
{
    float *tmp = (float *)malloc(sizeof(float) * (size_t)(R > C ? R : C));
    for (int64_t i = 0; i < R; ++i) {
        for (int64_t j = 0; j < C; ++j) tmp[j] = fabsf(S[i * ld + j]);
        rs[i] = orc_canon8(tmp, C, 1);
    }
    for (int64_t j = 0; j < C; ++j) {
        for (int64_t i = 0; i < R; ++i) tmp[i] = fabsf(S[i * ld + j]);
        cs[j] = orc_canon8(tmp, R, 1);
    }
    free(tmp);
}

/* ------------------------------------------------------------ a2: argsort */

/* a precedes b  <=>  score[a] > score[b], or equal and a < b */
static int precedes_desc(const float *s, int32_t a, int32_t b)
{
    if (s[a] > s[b]) return 1;
    if (s[a] < s[b]) return 0;
    return a < b;
}

void orc_argsort_desc(const float *score, int64_t n, int32_t *perm)
{
    /* insertion into a sorted prefix by binary search: O(n^2) moves at worst,
     * plainly correct; n is at most a few tens of thousands. */
    for (int64_t i = 0; i < n; ++i) {
        int64_t lo = 0, hi = i;
        while (lo < hi) {
            int64_t mid = (lo + hi) / 2;
            if (precedes_desc(score, perm[mid], (int32_t)i)) lo = mid + 1;
            else hi = mid;
        }
        memmove(perm + lo + 1, perm + lo, sizeof(int32_t) * (size_t)(i - lo));
        perm[lo] = (int32_t)i;
    }
}

/* Coupled reordering (App. "Channel Reordering", Sec. 4.1 last paragraph): dimensions that carry
 * the same activation share one permutation, computed from the scores aggregated over the
 * coupled matrices.  Aggregation = plain fp32 sum, member after member in the given order. */
void orc_group_scores(const float *const *member_scores, int n_members, int64_t n, float *out)
{
    for (int64_t j = 0; j < n; ++j) {
        float acc = member_scores[0][j];
        for (int k = 1; k < n_members; ++k) acc = acc + member_scores[k][j];
        out[j] = acc;
    }
}

/* The same order as orc_argsort_desc, applied inside consecutive pieces of `piece` channels
 * (attention heads keep their channels); piece = 0 or n: the whole array. */
void orc_argsort_desc_pieces(const float *score, int64_t n, int64_t piece, int32_t *perm)
{
    if (piece <= 0 || piece > n) piece = n;
    for (int64_t p0 = 0; p0 < n; p0 += piece) {
        const int64_t len = (n - p0 < piece) ? n - p0 : piece;
        orc_argsort_desc(score + p0, len, perm + p0);
        for (int64_t i = 0; i < len; ++i) perm[p0 + i] += (int32_t)p0;
    }
}

/* ------------------------------------------------------------- a3: gather */

void orc_gather_bf16(const uint16_t *W, int64_t R, int64_t C, int64_t ld,
                     const int32_t *rp, const int32_t *cp, uint16_t *out)
{
    for (int64_t i = 0; i < R; ++i)
        for (int64_t j = 0; j < C; ++j)
            out[i * C + j] = W[(int64_t)rp[i] * ld + cp[j]];
}

void orc_gather_f32(const float *S, int64_t R, int64_t C, int64_t ld,
                    const int32_t *rp, const int32_t *cp, float *out)
{
    for (int64_t i = 0; i < R; ++i)
        for (int64_t j = 0; j < C; ++j)
            out[i * C + j] = S[(int64_t)rp[i] * ld + cp[j]];
}

/* -------------------------------------------------------------- quantizer */

typedef struct {
    float mn;      /* group minimum = grid origin ("zero")    */
    float inv;     /* qmax / range                            */
    float scale;   /* range / qmax                            */
    int   qmax;
} grid_t;

static grid_t group_grid(const float *w, int n, int bits)
{
    grid_t g;
    if (bits == 0) {                 /* Sec. 3: a component at 0 bits is pruned, what = 0 for all of it: */
        g.mn = 0.0f;                 /* origin 0, step 0, the only code 0; nothing of the group is kept  */
        g.inv = 0.0f;
        g.scale = 0.0f;
        g.qmax = 0;
        return g;
    }
    float mn = w[0], mx = w[0];
    for (int e = 1; e < n; ++e) {
        if (w[e] < mn) mn = w[e];
        if (w[e] > mx) mx = w[e];
    }
    float range = mx - mn;
    g.qmax = (1 << bits) - 1;
    float qf = (float)g.qmax;
    float inv = qf / range;
    if (!isfinite(inv)) {            /* constant group (range 0) or overflow */
        g.inv = 0.0f;
        g.scale = 0.0f;
    } else {
        g.inv = inv;
        g.scale = range / qf;
    }
    g.mn = mn;
    return g;
}

static int quant_code(float x, const grid_t *g)
{
    float t = x * g->inv;
    int q = (int)rintf(t);           /* round half to even */
    if (q < 0) q = 0;
    if (q > g->qmax) q = g->qmax;
    return q;
}

void orc_quant_group(const float *w, int n, int bits,
                     int32_t *q_out, float *scale, float *zero)
{
    grid_t g = group_grid(w, n, bits);
    if (q_out)
        for (int e = 0; e < n; ++e) q_out[e] = quant_code(w[e] - g.mn, &g);
    *scale = g.scale;
    *zero = g.mn + 0.0f;             /* -0 -> +0 */
}

/* --------------------------------------------------------- a5: cost table */

void orc_cost_table_pow(const uint16_t *Wp, const float *Sp, int64_t R, int64_t C,
                        int m, int n, const int32_t *bits, int K, int power, float *cost)
{
    int64_t nbr = R / m, nbc = C / n;
    int nj = n / 8, no = m / 8;
    float *wrow = (float *)malloc(sizeof(float) * (size_t)n);
    grid_t *grid = (grid_t *)malloc(sizeof(grid_t) * (size_t)m);
    float *O = (float *)malloc(sizeof(float) * (size_t)nj);
    float *osum = (float *)malloc(sizeof(float) * (size_t)no);

    for (int64_t I = 0; I < nbr; ++I)
    for (int64_t J = 0; J < nbc; ++J)
    for (int l = 0; l < K; ++l) {
        /* one grid per block row (= quantization group) */
        for (int r = 0; r < m; ++r) {
            const uint16_t *src = Wp + (I * m + r) * C + J * n;
            for (int e = 0; e < n; ++e) wrow[e] = bf16_to_f32(src[e]);
            grid[r] = group_grid(wrow, n, bits[l]);
        }
        for (int o = 0; o < no; ++o) {
            for (int j = 0; j < nj; ++j) {
                float E[8];
                for (int rr = 0; rr < 8; ++rr) {
                    int r = o * 8 + rr;
                    const grid_t *g = &grid[r];
                    const uint16_t *wsrc = Wp + (I * m + r) * C + J * n + j * 8;
                    const float *ssrc = Sp + (I * m + r) * C + J * n + j * 8;
                    float a = 0.0f;
                    for (int e = 0; e < 8; ++e) {
                        float x = bf16_to_f32(wsrc[e]) - g->mn;
                        int q = quant_code(x, g);
                        float d = fmaf(-(float)q, g->scale, x);   /* w - what */
                        float e2 = power == 1 ? fabsf(d) : d * d;
                        a = fmaf(ssrc[e], e2, a);
                    }
                    E[rr] = a;
                }
                O[j] = pair_tree(E, 8);
            }
            osum[o] = pair_tree(O, nj);
        }
        cost[(I * nbc + J) * K + l] = pair_tree(osum, no);
    }
    free(wrow); free(grid); free(O); free(osum);
}

void orc_cost_table(const uint16_t *Wp, const float *Sp, int64_t R, int64_t C,
                    int m, int n, const int32_t *bits, int K, float *cost)
{
    orc_cost_table_pow(Wp, Sp, R, C, m, n, bits, K, 2, cost);
}

/* Dynamic-sensitivity surrogates of one iteration (App. "choice of sensitivity statistics",
 * the two displayed equations): for every block at its CURRENT bitwidth b (level[] indexes bits[]),
 *   s_up   = sum over the block of  g * (w - what)          (signed, first order gain of one more bit)
 *   s_down = 2^-b * sum over the block of |g * what|        (expected loss of one bit less)
 * with what = fmaf(q, scale, min) the dequantized weight of the block's row grid and g the
 * gradient at the quantized model (an input here).  Sums in the canonical order of the cost
 * table; the chunk steps are a = fmaf(g, w - what, a) and a = a + |g * what|.
 * Wp, Gp: reordered, dense; level: one entry per block of THIS matrix (row-major block grid). */
void orc_surrogates(const uint16_t *Wp, const float *Gp, int64_t R, int64_t C, int m, int n,
                    const int32_t *bits, const uint8_t *level, float *s_up, float *s_down)
{
    int64_t nbr = R / m, nbc = C / n;
    int nj = n / 8, no = m / 8;
    float *wrow = (float *)malloc(sizeof(float) * (size_t)n);
    grid_t *grid = (grid_t *)malloc(sizeof(grid_t) * (size_t)m);
    float *O = (float *)malloc(sizeof(float) * (size_t)nj);
    float *osum = (float *)malloc(sizeof(float) * (size_t)no);

    for (int64_t I = 0; I < nbr; ++I)
    for (int64_t J = 0; J < nbc; ++J) {
        const int b = bits[level[I * nbc + J]];
        for (int r = 0; r < m; ++r) {
            const uint16_t *src = Wp + (I * m + r) * C + J * n;
            for (int e = 0; e < n; ++e) wrow[e] = bf16_to_f32(src[e]);
            grid[r] = group_grid(wrow, n, b);
        }
        for (int which = 0; which < 2; ++which) {
            for (int o = 0; o < no; ++o) {
                for (int j = 0; j < nj; ++j) {
                    float E[8];
                    for (int rr = 0; rr < 8; ++rr) {
                        int r = o * 8 + rr;
                        const grid_t *g = &grid[r];
                        const uint16_t *wsrc = Wp + (I * m + r) * C + J * n + j * 8;
                        const float *gsrc = Gp + (I * m + r) * C + J * n + j * 8;
                        float a = 0.0f;
                        for (int e = 0; e < 8; ++e) {
                            float w = bf16_to_f32(wsrc[e]);
                            int q = quant_code(w - g->mn, g);
                            float what = fmaf((float)q, g->scale, g->mn);
                            if (which == 0) a = fmaf(gsrc[e], w - what, a);
                            else a = a + fabsf(gsrc[e] * what);
                        }
                        E[rr] = a;
                    }
                    O[j] = pair_tree(E, 8);
                }
                osum[o] = pair_tree(O, nj);
            }
            float t = pair_tree(osum, no);
            if (which == 0) s_up[I * nbc + J] = t;
            else s_down[I * nbc + J] = ldexpf(t, -b);
        }
    }
    free(wrow); free(grid); free(O); free(osum);
}

/* ------------------------------------------------- a6-a8: scalable greedy */

static int ceil_log2_i64(int64_t v)
{
    int p = 0;
    while (((int64_t)1 << p) < v) ++p;
    return p;
}

int32_t orc_cost_shift(const float *cost, int64_t N, int K)
{
    float mx = 0.0f;
    for (int64_t i = 0; i < N * K; ++i)
        if (cost[i] > mx) mx = cost[i];
    if (!(mx > 0.0f)) return 0;
    return 61 - ceil_log2_i64(N) - (ilogbf(mx) + 1);
}

int64_t orc_fx(float v, int32_t shift)
{
    return llrint(ldexp((double)v, shift));
}

/* index sort by (value, index) with a direction flag; merge sort */
typedef struct { const float *v; int desc; } order_t;

static int before(const order_t *o, int64_t a, int64_t b)
{
    float va = o->v[a], vb = o->v[b];
    if (va != vb) return o->desc ? (va > vb) : (va < vb);
    return a < b;
}

static void msort(int64_t *idx, int64_t *tmp, int64_t n, const order_t *o)
{
    if (n < 2) return;
    int64_t h = n / 2;
    msort(idx, tmp, h, o);
    msort(idx + h, tmp, n - h, o);
    int64_t i = 0, j = h, k = 0;
    while (i < h && j < n)
        tmp[k++] = before(o, idx[j], idx[i]) ? idx[j++] : idx[i++];
    while (i < h) tmp[k++] = idx[i++];
    while (j < n) tmp[k++] = idx[j++];
    memcpy(idx, tmp, sizeof(int64_t) * (size_t)n);
}

/* One step of Algorithm 2 (lines 6-10) with the caller's own estimates: s_up[i] is the estimated
 * gain of raising block i by one candidate, s_down[i] the estimated loss of lowering it by one
 * (App. "choice of sensitivity statistics"); the values are ranked as given.  level_out receives
 * the proposal.  Returns 1 = expansion (lines 6-7: the first min(k, eligible) blocks by
 * (s_up descending, lower index first), cut at the first s_up <= 0 and at the budget),
 * 2 = balanced swap to be accepted or rejected by the caller's own loss test (lines 9-12:
 * U = first h = max(1, k/2) by s_up, D = first h by (s_down ascending, lower index first)
 * outside U, U' = longest prefix of U that fits the slack plus the bits D frees),
 * 0 = nothing to propose (level_out = level_in).  Negative: bad arguments.               */
int orc_propose(const float *s_up, const float *s_down, const uint8_t *level_in, int64_t N,
                const int32_t *bits, int K, double avg_bits, int64_t k, uint8_t *level_out,
                int64_t *n_up, int64_t *n_dn, int64_t *bits_before, int64_t *bits_after)
{
    if (!s_up || !s_down || !level_in || !level_out || N <= 0 || !bits || K <= 0 || k < 1) return -3;
    const int64_t T = (int64_t)floor(avg_bits * (double)N);
    int64_t used = 0;
    for (int64_t i = 0; i < N; ++i) { level_out[i] = level_in[i]; used += bits[level_in[i]]; }
    const int64_t slack = T - used;
    *n_up = *n_dn = 0;
    *bits_before = *bits_after = used;

    float *up = (float *)malloc(sizeof(float) * (size_t)N);
    float *dn = (float *)malloc(sizeof(float) * (size_t)N);
    int64_t *ordU = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    int64_t *ordD = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    int64_t *tmp = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
    uint8_t *inU = (uint8_t *)calloc((size_t)N, 1);
    int64_t n_eu = 0, n_ed = 0;
    for (int64_t i = 0; i < N; ++i) {
        up[i] = s_up[i] + 0.0f;                       /* -0 ranks as +0 */
        dn[i] = s_down[i] + 0.0f;
        if (level_in[i] < K - 1) ordU[n_eu++] = i;
        if (level_in[i] > 0) ordD[n_ed++] = i;
    }
    order_t oup = { up, 1 }, odn = { dn, 0 };
    msort(ordU, tmp, n_eu, &oup);
    msort(ordD, tmp, n_ed, &odn);

    int kind = 0;
    if (slack > 0) {                                  /* expansion */
        int64_t lim = k < n_eu ? k : n_eu, cum = 0, p = 0;
        while (p < lim) {
            int64_t i = ordU[p];
            int step = bits[level_in[i] + 1] - bits[level_in[i]];
            if (!(up[i] > 0.0f) || cum + step > slack) break;
            cum += step;
            ++p;
        }
        if (p > 0) {
            for (int64_t q = 0; q < p; ++q) level_out[ordU[q]]++;
            *n_up = p;
            *bits_after = used + cum;
            kind = 1;
        }
    }
    if (kind == 0) {                                  /* balanced swap */
        int64_t h = k / 2;
        if (h < 1) h = 1;
        int64_t nU = h < n_eu ? h : n_eu;
        for (int64_t q = 0; q < nU; ++q) inU[ordU[q]] = 1;
        int64_t nD = 0, freed = 0;
        for (int64_t q = 0; q < n_ed && nD < h; ++q) {
            int64_t i = ordD[q];
            if (inU[i]) continue;
            ordD[nD++] = i;
            freed += bits[level_in[i]] - bits[level_in[i] - 1];
        }
        int64_t nUp = 0, cum = 0;
        while (nUp < nU) {
            int64_t i = ordU[nUp];
            int step = bits[level_in[i] + 1] - bits[level_in[i]];
            if (cum + step > slack + freed) break;
            cum += step;
            ++nUp;
        }
        if (nUp > 0 && nD > 0) {
            for (int64_t q = 0; q < nUp; ++q) level_out[ordU[q]]++;
            for (int64_t q = 0; q < nD; ++q) level_out[ordD[q]]--;
            *n_up = nUp;
            *n_dn = nD;
            *bits_after = used + cum - freed;
            kind = 2;
        }
    }
    free(up); free(dn); free(ordU); free(ordD); free(tmp); free(inU);
    return kind;
}

int orc_allocate(const float *cost, int64_t N, const int32_t *bits, int K,
                 double avg_bits, const orc_params *prm, uint8_t *level,
                 orc_stats *stats, orc_trace *trace, int64_t trace_cap,
                 int64_t *n_trace)
{
    if (!cost || N <= 0 || !bits || K <= 0 || !prm || !level) return -3;
    if (n_trace) *n_trace = 0;
    if (avg_bits < (double)bits[0]) return -1;

    int64_t T = (int64_t)floor(avg_bits * (double)N);   /* Eq. 1 budget */
    int32_t shift = orc_cost_shift(cost, N, K);
    int rc = 0;

    orc_stats st;
    memset(&st, 0, sizeof st);
    st.bits_budget = T;
    st.cost_shift = shift;

    int64_t k = (int64_t)floor(prm->gamma0 * (double)N);
    int64_t kmin = (int64_t)floor(prm->gammaT * (double)N);
    if (k < 1) k = 1;
    if (kmin < 1) kmin = 1;

    if (avg_bits >= (double)bits[K - 1]) {
        for (int64_t i = 0; i < N; ++i) level[i] = (uint8_t)(K - 1);
    } else {
        int l0 = 0;
        if (prm->init_mode == 0) {
            double fb = floor(avg_bits);
            for (int l = 0; l < K; ++l)
                if ((double)bits[l] <= fb) l0 = l;
        }
        for (int64_t i = 0; i < N; ++i) level[i] = (uint8_t)l0;

        float *up = (float *)malloc(sizeof(float) * (size_t)N);
        float *dn = (float *)malloc(sizeof(float) * (size_t)N);
        int64_t *ord = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
        int64_t *ord2 = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
        int64_t *tmp = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
        uint8_t *inU = (uint8_t *)malloc((size_t)N);

        while (k >= kmin) {
            if (st.iters >= prm->max_iters) { rc = -2; break; }
            st.iters++;
            orc_trace tr;
            memset(&tr, 0, sizeof tr);
            tr.k = k;

            int64_t used = 0;
            for (int64_t i = 0; i < N; ++i) used += bits[level[i]];
            int64_t slack = T - used;
            tr.bits_before = used;

            /* marginal change per bit, from the table (Alg. 2 line 5) */
            int64_t n_eu = 0, n_ed = 0;
            for (int64_t i = 0; i < N; ++i) {
                int l = level[i];
                const float *c = cost + i * K;
                if (l < K - 1) {
                    float g = (c[l] - c[l + 1]) / (float)(bits[l + 1] - bits[l]);
                    up[i] = g + 0.0f;
                    ord[n_eu++] = i;
                }
                if (l > 0) {
                    float g = (c[l - 1] - c[l]) / (float)(bits[l] - bits[l - 1]);
                    dn[i] = g + 0.0f;
                    ord2[n_ed++] = i;
                }
            }
            order_t oup = { up, 1 }, odn = { dn, 0 };
            msort(ord, tmp, n_eu, &oup);     /* largest gain first   */
            msort(ord2, tmp, n_ed, &odn);    /* smallest loss first  */

            /* ---- expansion (Alg. 2 lines 6-7), capped by the budget */
            if (slack > 0) {
                int64_t lim = k < n_eu ? k : n_eu, cum = 0, p = 0;
                while (p < lim) {
                    int64_t i = ord[p];
                    int step = bits[level[i] + 1] - bits[level[i]];
                    if (!(up[i] > 0.0f) || cum + step > slack) break;
                    cum += step;
                    ++p;
                }
                if (p > 0) {
                    for (int64_t q = 0; q < p; ++q) level[ord[q]]++;
                    st.expansions++;
                    tr.kind = 0; tr.n_up = tr.p_up = p;
                    tr.bits_after = used + cum;
                    if (trace && st.iters - 1 < trace_cap) trace[st.iters - 1] = tr;
                    continue;
                }
            }

            /* ---- balanced swap (Alg. 2 lines 9-12) */
            int64_t h = k / 2;
            if (h < 1) h = 1;
            int64_t nU = h < n_eu ? h : n_eu;
            memset(inU, 0, (size_t)N);
            for (int64_t q = 0; q < nU; ++q) inU[ord[q]] = 1;

            int64_t nD = 0, freed = 0, lossD = 0;
            for (int64_t q = 0; q < n_ed && nD < h; ++q) {
                int64_t i = ord2[q];
                if (inU[i]) continue;
                int l = level[i];
                ord2[nD++] = i;              /* compact D to the front */
                freed += bits[l] - bits[l - 1];
                lossD += orc_fx(cost[i * K + l - 1] - cost[i * K + l], shift);
            }
            int64_t nUp = 0, cum = 0, gainU = 0;
            while (nUp < nU) {
                int64_t i = ord[nUp];
                int l = level[i];
                int step = bits[l + 1] - bits[l];
                if (cum + step > slack + freed) break;
                cum += step;
                gainU += orc_fx(cost[i * K + l] - cost[i * K + l + 1], shift);
                ++nUp;
            }
            int64_t delta = lossD - gainU;
            tr.p_up = nUp; tr.p_dn = nD; tr.delta_fixed = delta;
            if (nUp > 0 && nD > 0 && delta < 0) {
                for (int64_t q = 0; q < nUp; ++q) level[ord[q]]++;
                for (int64_t q = 0; q < nD; ++q) level[ord2[q]]--;
                st.swaps_ok++;
                tr.kind = 1; tr.n_up = nUp; tr.n_dn = nD;
                tr.bits_after = used + cum - freed;
            } else {
                k = k / 2;
                st.swaps_rej++;
                tr.kind = 2;
                tr.bits_after = used;
            }
            if (trace && st.iters - 1 < trace_cap) trace[st.iters - 1] = tr;
        }
        free(up); free(dn); free(ord); free(ord2); free(tmp); free(inU);
    }

    st.k_final = k;
    for (int64_t i = 0; i < N; ++i) {
        st.bits_used += bits[level[i]];
        st.cost_fixed += orc_fx(cost[i * K + level[i]], shift);
    }
    if (stats) *stats = st;
    if (n_trace) *n_trace = st.iters;
    return rc;
}

/* ------------------------------------------------ Algorithm 1 on a table */

void orc_classic_greedy(const float *cost, int64_t N, const int32_t *bits,
                        int K, double avg_bits, uint8_t *level)
{
    int64_t T = (int64_t)floor(avg_bits * (double)N);
    int64_t used = 0;
    for (int64_t i = 0; i < N; ++i) { level[i] = 0; used += bits[0]; }
    for (;;) {
        int64_t best = -1;
        float bestg = 0.0f;
        for (int64_t i = 0; i < N; ++i) {
            int l = level[i];
            if (l >= K - 1) continue;
            int step = bits[l + 1] - bits[l];
            if (used + step > T) continue;
            float g = (cost[i * K + l] - cost[i * K + l + 1]) / (float)step;
            if (best < 0 || g > bestg) { best = i; bestg = g; }
        }
        if (best < 0) break;
        used += bits[level[best] + 1] - bits[level[best]];
        level[best]++;
    }
}

/* ------------------------------------------------------------ brute force */

double orc_brute_force(const float *cost, int N, const int32_t *bits, int K,
                       double avg_bits, uint8_t *best_level)
{
    int64_t T = (int64_t)floor(avg_bits * (double)N);
    uint8_t cur[32];
    double best = INFINITY;
    if (N > 32) return NAN;
    memset(cur, 0, sizeof cur);
    for (;;) {
        int64_t used = 0;
        double c = 0.0;
        for (int i = 0; i < N; ++i) {
            used += bits[cur[i]];
            c += (double)cost[i * K + cur[i]];
        }
        if (used <= T && c < best) {
            best = c;
            if (best_level) memcpy(best_level, cur, (size_t)N);
        }
        int d = 0;                          /* odometer */
        while (d < N && ++cur[d] == K) cur[d++] = 0;
        if (d == N) break;
    }
    return best;
}

/* --------------------------------------------------- a9: offsets and pack */

void orc_offsets(const uint8_t *level, int64_t N, int m, int n,
                 const int32_t *bits, int64_t *byte_off)
{
    int64_t acc = 0;
    for (int64_t i = 0; i < N; ++i) {
        byte_off[i] = acc;
        acc += (int64_t)m * n * bits[level[i]] / 8;
    }
    byte_off[N] = acc;
}

void orc_pack(const uint16_t *Wp, int64_t R, int64_t C, int m, int n,
              const int32_t *bits, int K, const uint8_t *level,
              const int64_t *byte_off, int64_t block_base,
              uint8_t *codes, float *scale, float *zero)
{
    (void)K;
    int64_t nbr = R / m, nbc = C / n;
    float *wrow = (float *)malloc(sizeof(float) * (size_t)n);
    for (int64_t I = 0; I < nbr; ++I)
    for (int64_t J = 0; J < nbc; ++J) {
        int64_t b = block_base + I * nbc + J;
        int c = bits[level[b]];
        uint8_t *dst = codes + byte_off[b];
        memset(dst, 0, (size_t)((int64_t)m * n * c / 8));
        for (int r = 0; r < m; ++r) {
            const uint16_t *src = Wp + (I * m + r) * C + J * n;
            for (int e = 0; e < n; ++e) wrow[e] = bf16_to_f32(src[e]);
            grid_t g = group_grid(wrow, n, c);
            scale[b * m + r] = g.scale;
            zero[b * m + r] = g.mn + 0.0f;
            for (int e = 0; e < n; ++e) {
                int q = quant_code(wrow[e] - g.mn, &g);
                int64_t bit0 = ((int64_t)r * n + e) * c;
                for (int t = 0; t < c; ++t)
                    if ((q >> t) & 1) {
                        int64_t bit = bit0 + t;
                        dst[bit >> 3] |= (uint8_t)(1u << (bit & 7));
                    }
            }
        }
    }
    free(wrow);
}


/* ------------------------------------------ inference: mixed-precision product (Sec. 5.3) */

/* code of element e of a block stored at `blk` with c bits per code (LSB-first bit stream) */
static unsigned stream_code(const uint8_t *blk, int64_t e, int c)
{
    unsigned q = 0;
    for (int t = 0; t < c; ++t) {
        int64_t bit = e * c + t;
        q |= (unsigned)((blk[bit >> 3] >> (bit & 7)) & 1u) << t;
    }
    return q;
}

/* The stored matrix, dequantized: What[i][j] = fmaf(q, scale, zero) in fp32 (the format's
 * definition of the stored value), from the packed arrays of one matrix of R x C in m x n blocks. */
void orc_dequant(const uint8_t *codes, const float *scale, const float *zero, const uint8_t *level,
                 const int64_t *byte_off, int64_t block_base, int64_t R, int64_t C, int m, int n,
                 const int32_t *bits, float *What)
{
    const int64_t nbc = C / n;
    for (int64_t i = 0; i < R; ++i)
        for (int64_t j = 0; j < C; ++j) {
            const int64_t blk = block_base + (i / m) * nbc + j / n;
            const int r = (int)(i % m), cc = (int)(j % n);
            const int c = bits[level[blk]];
            const unsigned q = stream_code(codes + byte_off[blk], (int64_t)r * n + cc, c);
            What[i * C + j] = fmaf((float)q, scale[blk * m + r], zero[blk * m + r]);
        }
}

/* y[b][i] = sum_j What[i][j] * x[b][j]: the layer's product with the stored weights, x given as
 * bf16 bit patterns [batch][C], the sum in float64 over j ascending. */
void orc_mp_gemm(const uint8_t *codes, const float *scale, const float *zero, const uint8_t *level,
                 const int64_t *byte_off, int64_t block_base, int64_t R, int64_t C, int m, int n,
                 const int32_t *bits, const uint16_t *x, int batch, double *y)
{
    float *What = (float *)malloc(sizeof(float) * (size_t)(R * C));
    orc_dequant(codes, scale, zero, level, byte_off, block_base, R, C, m, n, bits, What);
    for (int b = 0; b < batch; ++b)
        for (int64_t i = 0; i < R; ++i) {
            double a = 0.0;
            for (int64_t j = 0; j < C; ++j)
                a += (double)What[i * C + j] * (double)bf16_to_f32(x[(int64_t)b * C + j]);
            y[(int64_t)b * R + i] = a;
        }
    free(What);
}
