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
//
// Launch shape.  The kernel is persistent: a fixed grid of workgroups strides
// over "units" (whole blocks), and every lane keeps the next half octet's loads
// in flight while it computes on the current one, so HBM latency is hidden by
// the kernel's own arithmetic rather than by occupancy (the kernel needs ~190
// VGPRs, i.e. two waves per SIMD).
#include <math.h>
#include <string.h>

#include <type_traits>
#include <vector>

#include "cost_core.hpp"
#include "sbits_device.hpp"
#include "sbits_internal.hpp"

void sbits_fill_grid_consts(const int32_t *bits, int K, sbits::GridConsts *gc);

namespace sbits {

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uni64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

constexpr int COST_THREADS = 256;
constexpr int HALF = 4;                               // rows per pipeline stage
#ifndef SBITS_COST_STRIDED
#define SBITS_COST_STRIDED true
#endif

// the raw loads of HALF consecutive rows of one lane
struct HalfBuf {
    uint4 w[HALF];
    float4 s0[HALF], s1[HALF];
};

// Uniform 64-bit bases plus per-lane 32-bit byte offsets (a matrix is below 4 GiB), so the
// loads use the scalar-base + vector-offset addressing form and need one add per row.
// The weights of a lane are 16 contiguous bytes, so a wave's load covers whole cache lines.
// The 8 sensitivities of a lane are 32 bytes: loaded directly, each instruction would touch
// every other 16 bytes of 2 KiB.  With SWIZZLE the wave instead loads its 2 KiB run as two
// fully contiguous 1 KiB instructions (lane l takes bytes 16 l and 1024 + 16 l of the run, byte
// offsets soA / soB) and the lanes exchange the values through LDS before use (swizzle_s).
template <bool SWIZZLE>
__device__ __forceinline__ void load_half(HalfBuf &h, const char *__restrict__ Wb, const char *__restrict__ Sb,
                                          uint32_t woff, uint32_t wstride, uint32_t soA, uint32_t soB)
{
    // S is fp32, W bf16, same element index: byte offsets differ by a factor of two
#pragma unroll
    for (int j = 0; j < HALF; ++j) {
        const uint32_t wo = woff + (uint32_t)j * wstride;
        const uint32_t oa = SWIZZLE ? soA + 2u * (uint32_t)j * wstride : 2u * wo;
        const uint32_t ob = SWIZZLE ? soB + 2u * (uint32_t)j * wstride : 2u * wo + 16u;
        const u32x4_t tw = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(Wb + wo));
        const f32x4_t ta = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(Sb + oa));
        const f32x4_t tb = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(Sb + ob));
        h.w[j] = make_uint4(tw.x, tw.y, tw.z, tw.w);
        h.s0[j] = make_float4(ta.x, ta.y, ta.z, ta.w);
        h.s1[j] = make_float4(tb.x, tb.y, tb.z, tb.w);
    }
}

// Lane exchange of one row of sensitivities loaded with SWIZZLE: xrow is 2 KiB of LDS private
// to the wave.  Lane l stores its two 16-byte pieces where they sit in the run and reads back
// the 32 bytes at 32 l.  Only lanes of one wave touch xrow and a wave's LDS operations complete
// in order, so no workgroup barrier is needed.
__device__ __forceinline__ void swizzle_s(float4 *xrow, int lane, float4 &a, float4 &b)
{
    xrow[lane] = a;
    xrow[64 + lane] = b;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    a = xrow[2 * lane];
    b = xrow[2 * lane + 1];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// HALF rows of one octet: rows R_BASE .. R_BASE + HALF - 1 (R_BASE is 0 or 4).  Updates the
// pending levels of the row tree (t1, t2, t3) and leaves the running result in cur.
template <int LPG, int K, int R_BASE, bool SWIZZLE, bool Z0>
__device__ __forceinline__ void compute_half(const HalfBuf &h, const DivPlan<LPG, K - Z0> &dp,
                                             float (&t1)[K], float (&t2)[K], float (&t3)[K], float (&cur)[K],
                                             float4 *xw, int lane)
{
    using DP = DivPlan<LPG, K - Z0>;
    constexpr int RP = DP::RP < HALF ? DP::RP : HALF;
#pragma unroll
    for (int r0 = 0; r0 < HALF; r0 += RP) {
        uint4 wr[RP];
        float s[RP][8], out[RP][K];
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            wr[j] = h.w[r0 + j];
            float4 a = h.s0[r0 + j], b = h.s1[r0 + j];
            if constexpr (SWIZZLE) swizzle_s(xw + (r0 + j) * 128, lane, a, b);
            s[j][0] = a.x; s[j][1] = a.y; s[j][2] = a.z; s[j][3] = a.w;
            s[j][4] = b.x; s[j][5] = b.y; s[j][6] = b.z; s[j][7] = b.w;
        }
        quant_cost_round<LPG, K, RP, Z0>(wr, s, dp, out);
#pragma unroll
        for (int j = 0; j < RP; ++j) {
            const int rr = R_BASE + r0 + j;
#pragma unroll
            for (int c = 0; c < K; ++c) cur[c] = octet_tree_push(out[j][c], rr, t1[c], t2[c], t3[c]);
        }
        // keep the rounds apart: interleaving them only lengthens live ranges
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Work decomposition.  A wave holds GW = 64/LPG lane groups.  BX = min(GW, 8) of them sit side
// by side on BX adjacent blocks of one block row and walk the same octet, so every load
// instruction of a wave reads one contiguous run per row (1 KiB of weights, 2 KiB of
// sensitivities for LPG >= 8).  The remaining OW = GW/BX groups of the wave and the four waves
// of the workgroup take different octets: OS = 4*OW octets per step.
//   opb >= OS : a unit is BX blocks, walked in opb/OS steps
//   opb <  OS : a unit is BX*(OS/opb) blocks, one step
// (the last unit of a block row may be ragged: surplus groups recompute the row's last block
// and their result is dropped).  unit_start[] (n_mats + 1 entries) is the prefix of units per
// matrix.  Unit bookkeeping is scalar; a lane's offset inside a unit is a constant of the lane
// (times the row pitch).  STRIDED: workgroup w takes units w, w + G, ...; otherwise a
// contiguous range.
template <int LPG>
struct CostGeom {
    static constexpr int GW = 64 / LPG;
    static constexpr int BX = GW < 8 ? GW : 8;
    static constexpr int OW = GW / BX;
    static constexpr int OS = 4 * OW;
    static int blocks_per_unit(int m) { const int opb = m / 8; return opb >= OS ? BX : BX * (OS / opb); }
};

// K candidates; with Z0 the first one is "0 bits" (pruned block) and gc holds the other K - 1 grids.
// Up to four candidates fit the 256 registers that two waves per SIMD leave a lane; five and more need up
// to 345, and run with one wave per SIMD rather than spill (K = 8: 12 ms for the 8B-shaped model against 21).
template <int LPG, int K, bool STRIDED, bool Z0>
__global__ __launch_bounds__(COST_THREADS, (K > 4 ? 1 : 2))
void cost_kernel(const MatDesc *__restrict__ descs, MatDesc one, const int *__restrict__ unit_start,
                 int n_mats, int total_units, const uint16_t *__restrict__ W, const float *__restrict__ S,
                 int m, float *__restrict__ cost, GridConsts gc, int kstride, int koff)
{
    // kstride, koff: the K sums of a block go to cost[block][koff .. koff + K) of kstride values (a launch
    // may cover a subset of the candidates)
    using G = CostGeom<LPG>;
    constexpr int BX = G::BX, OS = G::OS;
    constexpr bool SWZ = G::OW == 1;                 // a wave walks ONE octet: 512 contiguous columns per row
    __shared__ float osum[BX * 128 * K];             // [block in unit][octet][candidate]
    __shared__ float4 xbuf[SWZ ? 4 * HALF * 128 : 1];    // per wave: HALF rows of 2 KiB for the lane exchange

    const int tid = threadIdx.x;
    const int lig = tid % LPG;
    const int gw = (tid & 63) / LPG;                 // lane group inside the wave
    const int slot = (tid >> 6) * G::OW + gw / BX;   // octet slot of this group, 0 .. OS-1
    const int opb = m >> 3;
    const int bpu = opb >= OS ? BX : BX * (OS / opb);           // blocks per unit
    const int steps = opb >= OS ? opb / OS : 1;                 // steps per unit
    const int bl = (gw % BX) + (opb >= OS ? 0 : BX * (slot / opb));   // this group's block inside the unit
    const int o0 = opb >= OS ? slot : slot % opb;               // this group's octet (plus p*OS in step p)
    const int lane = tid & 63;
    float4 *const xw = xbuf + (SWZ ? (tid >> 6) * (HALF * 128) : 0);

    DivPlan<LPG, K - Z0> dp;
    dp.init(gc, lig);

    int u_begin, u_end, u_step;
    if (STRIDED) {
        u_begin = (int)blockIdx.x; u_end = total_units; u_step = (int)gridDim.x;
    } else {
        const int per = (total_units + (int)gridDim.x - 1) / (int)gridDim.x;
        u_begin = (int)blockIdx.x * per; u_end = min(u_begin + per, total_units); u_step = 1;
    }
    if (u_begin >= u_end) return;
    const int nsteps = ((u_end - u_begin + u_step - 1) / u_step) * steps;

    // ---- scalar state of the unit being LOADED (runs ahead of the one being computed) ----
    // Everything here is the same in all lanes; readfirstlane tells the compiler so, which keeps
    // the bookkeeping in scalar registers and the loads in scalar-base + vector-offset form.
    int mat = 0, mat_begin = 0, mat_end = total_units;
    int d_cols, d_nbc, upr;
    int64_t d_elem, d_cbase;
    int unit = u_begin, I = 0, U = 0, p = 0;
    auto enter_unit = [&](bool first) {              // (mat, I, U) of `unit`
        if (descs && (first || unit >= mat_end)) {
            if (first) mat = uni(find_matrix(unit_start, n_mats, unit));
            else while (unit >= uni(unit_start[mat + 1])) ++mat;
            mat_begin = uni(unit_start[mat]);
            mat_end = uni(unit_start[mat + 1]);
        }
        if (first || descs) {
            const MatDesc &d = descs ? descs[mat] : one;
            d_cols = uni((int)d.cols);
            d_nbc = uni(d.nbc);
            d_elem = uni64(d.elem_off);
            d_cbase = uni64(d.block_base * kstride + koff);
            upr = (d_nbc + bpu - 1) / bpu;
        }
        const int ul = unit - mat_begin;
        I = uni(ul / upr);
        U = ul - I * upr;
    };
    enter_unit(true);

    struct StepAddr {
        const char *Wb, *Sb;      // uniform
        uint32_t voff;            // per-lane byte offset (bf16 units) inside the step
        uint32_t wstride;
        uint32_t soA, soB;        // per-lane byte offsets of the two contiguous sensitivity loads (SWZ)
        int J0, nbc, I;           // uniform: first block column of the unit, block columns, block row
        float *cbase;             // uniform: cost rows of the matrix
    };
    auto address = [&]() {
        StepAddr a;
        const int J0 = U * bpu;
        const int64_t ubase = ((int64_t)I * m + (int64_t)p * OS * 8) * d_cols + (int64_t)J0 * (LPG * 8);
        a.Wb = reinterpret_cast<const char *>(W + d_elem + ubase);
        a.Sb = reinterpret_cast<const char *>(S + d_elem + ubase);
        const int lim = d_nbc - 1 - J0;              // ragged unit: clamp the block column
        const int ble = bl < lim ? bl : lim;
        a.voff = ((uint32_t)o0 * 8u * (uint32_t)d_cols + (uint32_t)ble * (LPG * 8) + (uint32_t)lig * 8u) * 2u;
        a.wstride = (uint32_t)d_cols * 2u;
        a.soA = a.soB = 0;
        if constexpr (SWZ) {
            // column (relative to the unit) of the 4 values a lane loads from the wave's 512-column
            // run; a block column past the row's end is clamped like ble above
            const int c0 = (bl - gw % BX) * (LPG * 8) + 4 * lane, c1 = c0 + 256;
            const int b0 = c0 / (LPG * 8), b1 = c1 / (LPG * 8);
            const int e0 = (b0 < lim ? b0 : lim) * (LPG * 8) + c0 % (LPG * 8);
            const int e1 = (b1 < lim ? b1 : lim) * (LPG * 8) + c1 % (LPG * 8);
            a.soA = ((uint32_t)o0 * 8u * (uint32_t)d_cols + (uint32_t)e0) * 4u;
            a.soB = ((uint32_t)o0 * 8u * (uint32_t)d_cols + (uint32_t)e1) * 4u;
        }
        a.J0 = J0; a.nbc = d_nbc; a.I = I;
        a.cbase = cost + d_cbase;
        return a;
    };
    auto advance = [&]() {                           // to the next step, possibly the next unit / matrix
        if (++p < steps) return;
        if (unit + u_step >= u_end) { p = steps - 1; return; }  // stay on the last step
        p = 0;
        unit += u_step;
        if (STRIDED || unit >= mat_end) {
            enter_unit(false);
        } else if (++U >= upr) {
            U = 0; ++I;
        }
    };

    HalfBuf A, B;
    StepAddr nxt = address();
    load_half<SWZ>(A, nxt.Wb, nxt.Sb, nxt.voff, nxt.wstride, nxt.soA, nxt.soB);

    int pc = 0;                                      // step inside the unit being computed
    for (int sidx = 0; sidx < nsteps; ++sidx) {
        const StepAddr now = nxt;
        load_half<SWZ>(B, now.Wb, now.Sb, now.voff + HALF * now.wstride, now.wstride,
                       now.soA + 2u * HALF * now.wstride, now.soB + 2u * HALF * now.wstride);
        float t1[K], t2[K], t3[K], cur[K];
        compute_half<LPG, K, 0, SWZ, Z0>(A, dp, t1, t2, t3, cur, xw, lane);

        // the next step's first half goes in flight before this step's second half is computed
        // (after the last step this re-reads the last step: harmless, keeps the loop branch-free)
        advance();
        nxt = address();
        load_half<SWZ>(A, nxt.Wb, nxt.Sb, nxt.voff, nxt.wstride, nxt.soA, nxt.soB);
        compute_half<LPG, K, HALF, SWZ, Z0>(B, dp, t1, t2, t3, cur, xw, lane);

        const int oct = bl * opb + o0 + pc * OS;
#pragma unroll
        for (int c = 0; c < K; ++c) {
            const float v = group_allreduce<LPG>(cur[c], OpAdd{});
            if (lig == 0) osum[oct * K + c] = v;
        }
        if (++pc == steps) {
            pc = 0;
            __syncthreads();
            const int noct = bpu * opb;
            for (int s = 1; s < opb; s <<= 1) {
                const int npairs = noct / (2 * s);
                for (int q = tid; q < npairs * K; q += COST_THREADS) {
                    const int pi = q / K, c = q - pi * K;
                    const int oo = pi * 2 * s;
                    osum[oo * K + c] = osum[oo * K + c] + osum[(oo + s) * K + c];
                }
                __syncthreads();
            }
            for (int q = tid; q < bpu * K; q += COST_THREADS) {
                const int b2 = q / K, c = q - b2 * K;
                const int J = now.J0 + b2;
                if (J < now.nbc) now.cbase[((int64_t)now.I * now.nbc + J) * kstride + c] = osum[(b2 * opb) * K + c];
            }
            __syncthreads();
        }
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

static int persistent_grid(sbits_ctx *ctx, int64_t total_units)
{
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device) != hipSuccess || n_cu <= 0)
        n_cu = 256;
    const int64_t g = (int64_t)n_cu * 2;             // two workgroups (8 waves) per CU
    return (int)(total_units < g ? total_units : g);
}

struct CostLaunch {
    const MatDesc *descs;   // device table or null
    MatDesc one;            // used when descs == null
    const int *unit_start;  // device prefix or null
    int n_mats;
    int64_t total_units;
    const uint16_t *W;
    const float *S;
    int m;
    float *cost;
    GridConsts gc;
    int kstride, koff;      // row length of the table and first column this launch writes
};

template <int LPG, int K, bool Z0>
static int launch_lk(sbits_ctx *ctx, const CostLaunch &a)
{
    if (a.total_units > 0x7fffffff) return SBITS_ERR_BAD_SHAPE;
    const int grid = persistent_grid(ctx, a.total_units);
    if (grid == 0) return SBITS_OK;
    hipLaunchKernelGGL((cost_kernel<LPG, K, SBITS_COST_STRIDED, Z0>), dim3((unsigned)grid), dim3(COST_THREADS), 0, ctx->stream,
                       a.descs, a.one, a.unit_start, a.n_mats, (int)a.total_units, a.W, a.S, a.m, a.cost, a.gc,
                       a.kstride, a.koff);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

// K: all candidates; z0: the first of them is 0 bits (then 2 <= K <= 9, else 1 <= K <= 8)
template <int LPG>
static int launch_l(int K, bool z0, sbits_ctx *ctx, const CostLaunch &a)
{
    if (z0) switch (K) {
    case 2: return launch_lk<LPG, 2, true>(ctx, a);
    case 3: return launch_lk<LPG, 3, true>(ctx, a);
    case 4: return launch_lk<LPG, 4, true>(ctx, a);
    case 5: return launch_lk<LPG, 5, true>(ctx, a);
    case 6: return launch_lk<LPG, 6, true>(ctx, a);
    case 7: return launch_lk<LPG, 7, true>(ctx, a);
    case 8: return launch_lk<LPG, 8, true>(ctx, a);
    case 9:
        if constexpr (LPG != 8) return launch_lk<LPG, 9, true>(ctx, a);   // (64-column blocks: split by the caller)
        break;
    }
    else switch (K) {
    case 1: return launch_lk<LPG, 1, false>(ctx, a);
    case 2: return launch_lk<LPG, 2, false>(ctx, a);
    case 3: return launch_lk<LPG, 3, false>(ctx, a);
    case 4: return launch_lk<LPG, 4, false>(ctx, a);
    case 5: return launch_lk<LPG, 5, false>(ctx, a);
    case 6: return launch_lk<LPG, 6, false>(ctx, a);
    case 7: return launch_lk<LPG, 7, false>(ctx, a);
    case 8: return launch_lk<LPG, 8, false>(ctx, a);
    }
    return SBITS_ERR_BAD_BITWIDTHS;
}

static int launch_n(int n, int K, bool z0, sbits_ctx *ctx, const CostLaunch &a)
{
    switch (n / 8) {
    case 1:  return launch_l<1>(K, z0, ctx, a);
    case 2:  return launch_l<2>(K, z0, ctx, a);
    case 4:  return launch_l<4>(K, z0, ctx, a);
    case 8:  return launch_l<8>(K, z0, ctx, a);
    case 16: return launch_l<16>(K, z0, ctx, a);
    case 32: return launch_l<32>(K, z0, ctx, a);
    case 64: return launch_l<64>(K, z0, ctx, a);
    }
    return SBITS_ERR_BAD_SHAPE;
}

// All K candidates bits[0 .. K) of the table.  Nine candidates (0 .. 8 bits) on 64-column blocks would
// need more LDS for the octet sums than a workgroup may declare: they take two launches over the
// candidates, 0 .. 4 and 5 .. 8 (the grids are independent per candidate: the same table, bit for bit).
static int launch(int n, const int32_t *bits, int K, sbits_ctx *ctx, CostLaunch a)
{
    const bool z0 = bits[0] == 0;
    a.kstride = K;
    if (K == 9 && n == 64) {
        sbits_fill_grid_consts(bits + 1, 4, &a.gc);
        a.koff = 0;
        const int rc = launch_n(n, 5, true, ctx, a);
        if (rc) return rc;
        sbits_fill_grid_consts(bits + 5, 4, &a.gc);
        a.koff = 5;
        return launch_n(n, 4, false, ctx, a);
    }
    sbits_fill_grid_consts(bits + z0, K - z0, &a.gc);     // the kernels take the real grids only
    a.koff = 0;
    return launch_n(n, K, z0, ctx, a);
}

static int blocks_per_unit(int m, int n)
{
    switch (n / 8) {
    case 1:  return CostGeom<1>::blocks_per_unit(m);
    case 2:  return CostGeom<2>::blocks_per_unit(m);
    case 4:  return CostGeom<4>::blocks_per_unit(m);
    case 8:  return CostGeom<8>::blocks_per_unit(m);
    case 16: return CostGeom<16>::blocks_per_unit(m);
    case 32: return CostGeom<32>::blocks_per_unit(m);
    case 64: return CostGeom<64>::blocks_per_unit(m);
    }
    return 1;
}

}  // namespace sbits

// Grid constants of the K candidates bits[0 .. K) (entries beyond K repeat the last one).  A 0-bit
// candidate gets qmax 0 and an infinite threshold (see GridConsts).
void sbits_fill_grid_consts(const int32_t *bits, int K, sbits::GridConsts *gc)
{
    for (int c = 0; c < sbits::MAX_CAND; ++c) {
        const int b = c < K ? bits[c] : bits[K - 1];
        gc->bits[c] = b;
        gc->qmaxf[c] = (float)((1 << b) - 1);
        gc->thr[c] = b == 0 ? HUGE_VALF : sbits::finite_threshold(gc->qmaxf[c]);
    }
}

// one matrix: the descriptor travels as a kernel argument, nothing is read from a table
int sbits_launch_cost(sbits_ctx *ctx, const void *Wp, const float *Sp, int64_t R, int64_t C,
                      int m, int n, const int32_t *bits, int K, float *cost_rows)
{
    using namespace sbits;
    CostLaunch a;
    memset(&a, 0, sizeof a);
    a.one.rows = R; a.one.cols = C; a.one.nbr = (int)(R / m); a.one.nbc = (int)(C / n);
    const int bpu = blocks_per_unit(m, n);
    a.n_mats = 1;
    a.total_units = (R / m) * ((C / n + bpu - 1) / bpu);
    a.W = static_cast<const uint16_t *>(Wp);
    a.S = Sp;
    a.m = m;
    a.cost = cost_rows;
    return launch(n, bits, K, ctx, a);
}

// all matrices of the plan in one launch; the descriptor table is already in the workspace head
int sbits_launch_cost_all(sbits_plan *plan, const void *w_re, const float *s_re, float *cost, void *ws)
{
    using namespace sbits;
    sbits_ctx *ctx = plan->ctx;
    CostLaunch a;
    memset(&a, 0, sizeof a);
    if (plan->cost_unit_start.empty()) {             // depends on shapes only: computed once, kept for the copies
        const int bpu = blocks_per_unit(plan->m, plan->n);
        int64_t t = 0;
        for (int i = 0; i < plan->n_mats; ++i) {
            plan->cost_unit_start.push_back((int)t);
            t += (int64_t)plan->descs[i].nbr * ((plan->descs[i].nbc + bpu - 1) / bpu);
            if (t > 0x7fffffff) { plan->cost_unit_start.clear(); return SBITS_ERR_BAD_SHAPE; }
        }
        plan->cost_unit_start.push_back((int)t);
    }
    const int64_t tot = plan->cost_unit_start.back();
    int *d_pre = sbits_prefix_ptr(plan, ws, 0);
    SBITS_HIP(ctx, hipMemcpyAsync(d_pre, plan->cost_unit_start.data(), plan->cost_unit_start.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    a.descs = sbits_desc_ptr(ws);
    a.unit_start = d_pre;
    a.n_mats = plan->n_mats;
    a.total_units = tot;
    a.W = static_cast<const uint16_t *>(w_re);
    a.S = s_re;
    a.m = plan->m;
    a.cost = cost;
    return launch(plan->n, plan->bits, plan->K, ctx, a);
}

// which cost this build computes (the arithmetic core fixes it at compile time)
extern "C" int sbits_cost_power(void) { return SBITS_COST_POWER; }
