// Block x bitwidth cost table: one HBM pass over the reordered weights (bf16)
// and sensitivities (fp32); every candidate bitwidth is evaluated in registers.
//
// Operation (paper Sec. 5 "Implementation": round-to-nearest uniform quantizer,
// group = one block row; App. E "choice of sensitivity statistics": the exact
// re-quantized change is what the search needs):
//   cost[b][l] = sum over block b of s * (w - what_l)^2
//   what_l : asymmetric min-max grid of 2^c_l levels on each block row,
//            inv = qmax/R, scale = R/qmax (both 0 when qmax/R is not finite),
//            x = w - min, q = rint(x*inv) (half to even), d = fma(-q, scale, x)
//
// Data layout and mapping.  A lane owns 8 consecutive weights of a row (one
// 128-bit bf16 load, two 128-bit fp32 loads); LPG = n/8 adjacent lanes own one
// quantization group.  A lane group walks an "octet" of 8 consecutive rows.
// Summation order (fixed, so results do not depend on the launch shape):
//   chunk  : the lane's 8 elements left to right, a = fma(s, d*d, a)
//   octet  : adjacent-pair tree over the 8 rows, per lane (per 8-column chunk)
//   lanes  : adjacent-pair butterfly over the LPG lanes of the group
//   block  : adjacent-pair tree over the m/8 octets (through LDS)
#include <string.h>

#include <type_traits>

#include "sbits_device.hpp"
#include "sbits_internal.hpp"

namespace sbits {

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int COST_THREADS = 256;

template <int LPG, int K>
__global__ __launch_bounds__(COST_THREADS)
void cost_kernel(const uint16_t *__restrict__ W, const float *__restrict__ S, int64_t C,
                 int m, int nbc, int64_t nblocks, float *__restrict__ cost, GridConsts gc)
{
    constexpr int GPW = COST_THREADS / LPG;          // lane groups per workgroup
    constexpr int NS = (2 * K + LPG - 1) / LPG;      // grid divisions per lane per row
    __shared__ float osum[256 * K];

    const int tid = threadIdx.x;
    const int g = tid / LPG;
    const int lig = tid % LPG;
    const int opb = m >> 3;                          // octets per block
    const int bpw = opb >= GPW ? 1 : GPW / opb;      // blocks per workgroup
    const int passes = opb >= GPW ? opb / GPW : 1;

    // Each lane computes NS of the 2K quotients of a row (slot 2c: qmax_c / R,
    // slot 2c+1: R / qmax_c); they are then broadcast inside the group.
    float my_qf[NS], my_thr[NS];
    bool my_is_scale[NS];
#pragma unroll
    for (int t = 0; t < NS; ++t) {
        const int slot = lig + t * LPG;
        int c = slot >> 1;
        c = c < K ? c : K - 1;
        float qf = gc.qmaxf[0], th = gc.thr[0];
#pragma unroll
        for (int cc = 1; cc < K; ++cc)
            if (c == cc) { qf = gc.qmaxf[cc]; th = gc.thr[cc]; }
        my_qf[t] = qf;
        my_thr[t] = th;
        my_is_scale[t] = (slot & 1) != 0;
    }

    for (int pass = 0; pass < passes; ++pass) {
        const int oct_in_wg = g + pass * GPW;
        const int blk_local = oct_in_wg / opb;
        const int o = oct_in_wg - blk_local * opb;
        int64_t blk = (int64_t)blockIdx.x * bpw + blk_local;
        if (blk >= nblocks) blk = nblocks - 1;       // keep every lane in bounds; result discarded
        const int64_t I = blk / nbc, J = blk - I * nbc;
        const int64_t off0 = (I * m + (int64_t)o * 8) * C + J * (LPG * 8) + lig * 8;

        float t1[K], t2[K], t3[K], cur[K];
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const int64_t off = off0 + (int64_t)rr * C;
            const uint4 wp = *reinterpret_cast<const uint4 *>(W + off);
            const float4 s0 = *reinterpret_cast<const float4 *>(S + off);
            const float4 s1 = *reinterpret_cast<const float4 *>(S + off + 4);
            float w[8];
            unpack8(wp, w);
            const float s[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};

            float mn = fminf(fminf(fminf(w[0], w[1]), fminf(w[2], w[3])),
                             fminf(fminf(w[4], w[5]), fminf(w[6], w[7])));
            float mx = fmaxf(fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])),
                             fmaxf(fmaxf(w[4], w[5]), fmaxf(w[6], w[7])));
            mn = group_allreduce<LPG>(mn, OpMin{});
            mx = group_allreduce<LPG>(mx, OpMax{});
            const float R = mx - mn;

            float val[NS];
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                const float num = my_is_scale[t] ? R : my_qf[t];
                const float den = my_is_scale[t] ? my_qf[t] : R;
                const float v = num / den;           // IEEE correctly rounded
                val[t] = (R < my_thr[t]) ? 0.0f : v;
            }

            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = w[e] - mn;

            static_for<0, K>([&](auto ic) {
                constexpr int c = decltype(ic)::value;
                const float inv = group_bcast<LPG, (2 * c) % LPG>(val[(2 * c) / LPG]);
                const float scl = group_bcast<LPG, (2 * c + 1) % LPG>(val[(2 * c + 1) / LPG]);
                float a = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float q = rintf(x[e] * inv);
                    const float d = fmaf(-q, scl, x[e]);
                    a = fmaf(s[e], d * d, a);
                }
                cur[c] = a;
            });

            // adjacent-pair tree over the 8 rows of the octet
#pragma unroll
            for (int c = 0; c < K; ++c) {
                float v = cur[c];
                if (rr & 1) {
                    v = t1[c] + v;
                    if (rr & 2) {
                        v = t2[c] + v;
                        if (rr & 4) v = t3[c] + v;
                        else t3[c] = v;
                    } else {
                        t2[c] = v;
                    }
                } else {
                    t1[c] = v;
                }
                cur[c] = v;
            }
        }
        // cur[c] now holds the octet sum of this lane's 8-column chunk
#pragma unroll
        for (int c = 0; c < K; ++c) {
            const float v = group_allreduce<LPG>(cur[c], OpAdd{});
            if (lig == 0) osum[oct_in_wg * K + c] = v;
        }
    }
    __syncthreads();

    const int noct_wg = bpw * opb;
    for (int s = 1; s < opb; s <<= 1) {
        const int npairs = noct_wg / (2 * s);
        for (int p = tid; p < npairs * K; p += COST_THREADS) {
            const int pi = p / K, c = p - pi * K;
            const int oo = pi * 2 * s;
            osum[oo * K + c] = osum[oo * K + c] + osum[(oo + s) * K + c];
        }
        __syncthreads();
    }
    for (int p = tid; p < bpw * K; p += COST_THREADS) {
        const int bl = p / K, c = p - bl * K;
        const int64_t blk = (int64_t)blockIdx.x * bpw + bl;
        if (blk < nblocks) cost[blk * K + c] = osum[(bl * opb) * K + c];
    }
}

// smallest positive float R with qmax / R finite (qmax / R is non-increasing in R)
static float finite_threshold(float qf)
{
    uint32_t lo = 1, hi = 0x7f7fffffu;               // bit patterns of positive floats
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        float r;
        memcpy(&r, &mid, 4);
        volatile float q = qf / r;
        if (q <= 3.402823466e+38f) hi = mid; else lo = mid + 1;
    }
    float r;
    memcpy(&r, &lo, 4);
    return r;
}

template <int LPG, int K>
static int launch_lk(sbits_ctx *ctx, const uint16_t *W, const float *S, int64_t C, int m, int nbc,
                     int64_t nblocks, float *cost, const GridConsts &gc)
{
    constexpr int GPW = COST_THREADS / LPG;
    const int opb = m / 8;
    const int bpw = opb >= GPW ? 1 : GPW / opb;
    const int64_t nwg = (nblocks + bpw - 1) / bpw;
    if (nwg > 0x7fffffff) return SBITS_ERR_BAD_SHAPE;
    hipLaunchKernelGGL((cost_kernel<LPG, K>), dim3((unsigned)nwg), dim3(COST_THREADS), 0, ctx->stream,
                       W, S, C, m, nbc, nblocks, cost, gc);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

template <int LPG>
static int launch_l(int K, sbits_ctx *ctx, const uint16_t *W, const float *S, int64_t C, int m,
                    int nbc, int64_t nblocks, float *cost, const GridConsts &gc)
{
    switch (K) {
    case 1: return launch_lk<LPG, 1>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 2: return launch_lk<LPG, 2>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 3: return launch_lk<LPG, 3>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 4: return launch_lk<LPG, 4>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 5: return launch_lk<LPG, 5>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 6: return launch_lk<LPG, 6>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 7: return launch_lk<LPG, 7>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    case 8: return launch_lk<LPG, 8>(ctx, W, S, C, m, nbc, nblocks, cost, gc);
    }
    return SBITS_ERR_BAD_BITWIDTHS;
}

}  // namespace sbits

void sbits_fill_grid_consts(const int32_t *bits, int K, sbits::GridConsts *gc)
{
    for (int c = 0; c < 8; ++c) {
        const int b = c < K ? bits[c] : bits[K - 1];
        gc->bits[c] = b;
        gc->qmaxf[c] = (float)((1 << b) - 1);
        gc->thr[c] = sbits::finite_threshold(gc->qmaxf[c]);
    }
}

int sbits_launch_cost(sbits_ctx *ctx, const void *Wp, const float *Sp, int64_t R, int64_t C,
                      int m, int n, const int32_t *bits, int K, float *cost_rows)
{
    using namespace sbits;
    GridConsts gc;
    sbits_fill_grid_consts(bits, K, &gc);
    const int nbc = (int)(C / n);
    const int64_t nblocks = (R / m) * (C / n);
    const uint16_t *W = static_cast<const uint16_t *>(Wp);
    switch (n / 8) {
    case 1:  return launch_l<1>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    case 2:  return launch_l<2>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    case 4:  return launch_l<4>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    case 8:  return launch_l<8>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    case 16: return launch_l<16>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    case 32: return launch_l<32>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    case 64: return launch_l<64>(K, ctx, W, Sp, C, m, nbc, nblocks, cost_rows, gc);
    }
    return SBITS_ERR_BAD_SHAPE;
}
