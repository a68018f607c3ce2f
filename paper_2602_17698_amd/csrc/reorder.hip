// Bi-directional channel reordering (paper Sec. 4.1): channel scores, argsort,
// and the reorder-gather of weights and sensitivities.
//
// Scores.  Row score = l1 norm of the row of S, column score = l1 norm of the
// column, each summed in the canonical order: runs of 8 consecutive elements
// left to right from +0, then an adjacent-pair tree over the runs (zero padded
// to a power of two).  One pass over S serves both directions: a lane owns an
// 8 x 8 tile (8 rows, 8 consecutive columns), so it holds 8 row runs and 8
// column runs at once.  A wave covers 8 rows x 512 columns, a workgroup of four
// waves 32 rows x 512 columns.  Partial trees are written to the workspace and
// finished by two small kernels.
//
// Argsort.  Descending by score, ties to the lower index: rank by counting over
// a strict total order, which is exact and needs no multi-pass machinery for
// the at most few ten thousand channels of a matrix.
//
// Gather.  out[i][j] = in[rp[i]][cp[j]]: the source row is staged in LDS with
// coalesced 128-bit loads and read out permuted, so global traffic stays
// coalesced in both directions.
#include "sbits_device.hpp"
#include "sbits_internal.hpp"

namespace sbits {

constexpr int SC_THREADS = 256;
constexpr int SC_ROWS = 32;     // rows per workgroup (4 waves x 8)
constexpr int SC_COLS = 512;    // columns per workgroup (64 lanes x 8)

static inline int64_t pow2_ceil(int64_t v) { int64_t p = 1; while (p < v) p <<= 1; return p; }

// rowpart[r][seg]  : tree over the 64 column runs of segment seg (zero beyond C)
// colpart[band][c] : tree over the 4 row runs of band (zero beyond R)
__global__ __launch_bounds__(SC_THREADS)
void score_partial_kernel(const float *__restrict__ S, int64_t R, int64_t C, int64_t ld,
                          int nseg, float *__restrict__ rowpart, float *__restrict__ colpart)
{
    __shared__ float cbuf[4][SC_COLS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t seg = blockIdx.x, band = blockIdx.y;
    const int64_t r0 = band * SC_ROWS + wave * 8;
    const int64_t c0 = seg * SC_COLS + lane * 8;

    float rowrun[8], colrun[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) colrun[e] = 0.0f;
    const bool col_ok = c0 < C;                      // C is a multiple of 8
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        float v[8];
        if (col_ok && r0 + rr < R) {
            const float *p = S + (r0 + rr) * ld + c0;
            const float4 a = *reinterpret_cast<const float4 *>(p);
            const float4 b = *reinterpret_cast<const float4 *>(p + 4);
            v[0] = fabsf(a.x); v[1] = fabsf(a.y); v[2] = fabsf(a.z); v[3] = fabsf(a.w);
            v[4] = fabsf(b.x); v[5] = fabsf(b.y); v[6] = fabsf(b.z); v[7] = fabsf(b.w);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.0f;
        }
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a = a + v[e];                            // row run: left to right
            colrun[e] = colrun[e] + v[e];            // column run: top to bottom
        }
        rowrun[rr] = a;
    }
    // rows: adjacent-pair tree over the 64 lanes (64 runs = 512 columns)
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const float t = group_allreduce<64>(rowrun[rr], OpAdd{});
        if (lane == 0 && r0 + rr < R) rowpart[(r0 + rr) * nseg + seg] = t;
    }
    // columns: tree over the 4 waves (row runs 4*band .. 4*band+3)
#pragma unroll
    for (int e = 0; e < 8; ++e) cbuf[wave][lane * 8 + e] = colrun[e];
    __syncthreads();
    for (int c = threadIdx.x; c < SC_COLS; c += SC_THREADS) {
        const int64_t col = seg * SC_COLS + c;
        if (col < C)
            colpart[band * C + col] = (cbuf[0][c] + cbuf[1][c]) + (cbuf[2][c] + cbuf[3][c]);
    }
}

// Finishes an adjacent-pair tree over n leaves x[i*stride] (zero padded to a
// power of two; adding the zero padding is the identity, so the stack of
// completed subtrees is folded from the lowest level up).
__device__ __forceinline__ float finish_tree(const float *x, int64_t n, int64_t stride)
{
    float stack[24];
    for (int64_t i = 0; i < n; ++i) {
        float v = x[i * stride];
        int lvl = 0;
        for (int64_t b = i; b & 1; b >>= 1) { v = stack[lvl] + v; ++lvl; }
        stack[lvl] = v;
    }
    float v = 0.0f;
    bool have = false;
    int lvl = 0;
    for (int64_t b = n; b; b >>= 1, ++lvl) {
        if (b & 1) { v = have ? stack[lvl] + v : stack[lvl]; have = true; }
    }
    return v;
}

__global__ void score_finish_kernel(const float *__restrict__ rowpart, const float *__restrict__ colpart,
                                    int64_t R, int64_t C, int nseg, int64_t nband,
                                    float *__restrict__ rs, float *__restrict__ cs)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < R) rs[t] = finish_tree(rowpart + t * nseg, nseg, 1);
    else if (t - R < C) cs[t - R] = finish_tree(colpart + (t - R), nband, C);
}

// ---- argsort: rank by counting ------------------------------------------------
constexpr int AS_THREADS = 256;
constexpr int AS_TILE = 2048;    // keys per j-tile

__global__ __launch_bounds__(AS_THREADS)
void rank_kernel(const float *__restrict__ score, int n, int *__restrict__ rank)
{
    __shared__ float tile[AS_TILE];
    const int i = blockIdx.x * AS_THREADS + threadIdx.x;
    const int j0 = blockIdx.y * AS_TILE;
    const int jn = min(AS_TILE, n - j0);
    for (int j = threadIdx.x; j < jn; j += AS_THREADS) tile[j] = score[j0 + j];
    __syncthreads();
    if (i >= n) return;
    const float si = score[i];
    int cnt = 0;
    for (int j = 0; j < jn; ++j) {
        const float sj = tile[j];
        cnt += (sj > si) || (sj == si && (j0 + j) < i);   // j precedes i
    }
    if (cnt) atomicAdd(&rank[i], cnt);
}

__global__ void scatter_perm_kernel(const int *__restrict__ rank, int n, int32_t *__restrict__ perm)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) perm[rank[i]] = i;
}

__global__ void zero_i32_kernel(int *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// ---- gather -------------------------------------------------------------------
constexpr int GA_THREADS = 256;

// T = uint16_t (bf16) or float.  One workgroup per output row.
template <class T>
__global__ __launch_bounds__(GA_THREADS)
void gather_kernel(const T *__restrict__ in, int64_t R, int64_t C, int64_t ld, const int32_t *__restrict__ rp,
                   const int32_t *__restrict__ cp, T *__restrict__ out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    T *row = reinterpret_cast<T *>(smem);
    constexpr int V = 16 / sizeof(T);               // elements per 128-bit access
    const int64_t i = blockIdx.x;
    int64_t sr = rp[i];
    sr = sr < 0 ? 0 : (sr >= R ? R - 1 : sr);       // a permutation never trips this; keeps a bad one in bounds
    const T *src = in + sr * ld;
    const bool aligned = ((reinterpret_cast<uintptr_t>(src) & 15) == 0);
    if (aligned) {
        for (int64_t j = (int64_t)threadIdx.x * V; j < C; j += (int64_t)GA_THREADS * V)
            *reinterpret_cast<uint4 *>(row + j) = *reinterpret_cast<const uint4 *>(src + j);
    } else {
        for (int64_t j = threadIdx.x; j < C; j += GA_THREADS) row[j] = src[j];
    }
    __syncthreads();
    T *dst = out + i * C;                            // dense output, C % 8 == 0: 16-byte aligned rows
    for (int64_t j = (int64_t)threadIdx.x * V; j < C; j += (int64_t)GA_THREADS * V) {
        T tmp[V];
        const int4 c0 = *reinterpret_cast<const int4 *>(cp + j);
        tmp[0] = row[c0.x]; tmp[1] = row[c0.y]; tmp[2] = row[c0.z]; tmp[3] = row[c0.w];
        if constexpr (V == 8) {
            const int4 c1 = *reinterpret_cast<const int4 *>(cp + j + 4);
            tmp[4] = row[c1.x]; tmp[5] = row[c1.y]; tmp[6] = row[c1.z]; tmp[7] = row[c1.w];
        }
        *reinterpret_cast<uint4 *>(dst + j) = *reinterpret_cast<const uint4 *>(tmp);
    }
}

}  // namespace sbits

using namespace sbits;

// workspace: rowpart [R][nseg] | colpart [nband][C] | rank [max(R,C)] | rs [R] | cs [C]
size_t sbits_score_ws_bytes(int64_t R, int64_t C)
{
    const int64_t nseg = (C + SC_COLS - 1) / SC_COLS, nband = (R + SC_ROWS - 1) / SC_ROWS;
    size_t b = 0;
    b += sbits_align_up((size_t)(R * nseg) * 4, 256);
    b += sbits_align_up((size_t)(nband * C) * 4, 256);
    b += sbits_align_up((size_t)(R > C ? R : C) * 4, 256);
    b += sbits_align_up((size_t)R * 4, 256);
    b += sbits_align_up((size_t)C * 4, 256);
    return b;
}

int sbits_launch_scores(sbits_ctx *ctx, const float *S, int64_t R, int64_t C, int64_t ld,
                        float *row_score, float *col_score, void *ws)
{
    const int64_t nseg = (C + SC_COLS - 1) / SC_COLS, nband = (R + SC_ROWS - 1) / SC_ROWS;
    if (nband > 65535) return SBITS_ERR_BAD_SHAPE;
    char *p = static_cast<char *>(ws);
    float *rowpart = reinterpret_cast<float *>(p);
    p += sbits_align_up((size_t)(R * nseg) * 4, 256);
    float *colpart = reinterpret_cast<float *>(p);
    hipLaunchKernelGGL(score_partial_kernel, dim3((unsigned)nseg, (unsigned)nband), dim3(SC_THREADS), 0,
                       ctx->stream, S, R, C, ld, (int)nseg, rowpart, colpart);
    SBITS_HIP(ctx, hipGetLastError());
    const int64_t tot = R + C;
    hipLaunchKernelGGL(score_finish_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, ctx->stream,
                       rowpart, colpart, R, C, (int)nseg, nband, row_score, col_score);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

int sbits_launch_argsort(sbits_ctx *ctx, const float *score, int64_t n, int32_t *perm, void *ws_rank)
{
    int *rank = static_cast<int *>(ws_rank);
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, rank, n);
    SBITS_HIP(ctx, hipGetLastError());
    dim3 grid((unsigned)((n + AS_THREADS - 1) / AS_THREADS), (unsigned)((n + AS_TILE - 1) / AS_TILE));
    hipLaunchKernelGGL(rank_kernel, grid, dim3(AS_THREADS), 0, ctx->stream, score, (int)n, rank);
    SBITS_HIP(ctx, hipGetLastError());
    hipLaunchKernelGGL(scatter_perm_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream,
                       rank, (int)n, perm);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

int sbits_launch_gather(sbits_ctx *ctx, const void *W, const float *S, int64_t R, int64_t C,
                        int64_t ld_w, int64_t ld_s, const int32_t *rp, const int32_t *cp,
                        void *w_out, float *s_out)
{
    const size_t lds_w = (size_t)C * 2, lds_s = (size_t)C * 4;
    if (lds_s > 160 * 1024) return SBITS_ERR_BAD_SHAPE;
    static bool attr_done = false;
    if (!attr_done) {
        SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gather_kernel<float>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gather_kernel<uint16_t>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_done = true;
    }
    if (w_out) {
        hipLaunchKernelGGL(gather_kernel<uint16_t>, dim3((unsigned)R), dim3(GA_THREADS), lds_w, ctx->stream,
                           static_cast<const uint16_t *>(W), R, C, ld_w, rp, cp, static_cast<uint16_t *>(w_out));
        SBITS_HIP(ctx, hipGetLastError());
    }
    if (s_out) {
        hipLaunchKernelGGL(gather_kernel<float>, dim3((unsigned)R), dim3(GA_THREADS), lds_s, ctx->stream,
                           S, R, C, ld_s, rp, cp, s_out);
        SBITS_HIP(ctx, hipGetLastError());
    }
    return SBITS_OK;
}
