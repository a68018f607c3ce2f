// Arithmetic core of the block x bitwidth cost: the per-row round-to-nearest grid of
// every candidate bitwidth and the sensitivity-weighted squared change of a lane's 8 elements
// (paper Sec. 5 "Implementation", group = one block row).  Shared by the kernel that reads
// reordered matrices and by the one that reorders on the fly, so both produce the same bits.
#pragma once

#include "sbits_device.hpp"

namespace sbits {

constexpr int COST_MAX_ROUND = 4;                     // rows that may share one round of divisions

// Power of the quantization change in the block cost, fixed when the library is built:
//   2 (default): cost = sum s * d^2   (the sensitivity weighs the squared change)
//   1          : cost = sum s * |d|   (element-wise first-order form of paper Eq. 3 with s = |gradient|)
#ifndef SBITS_COST_POWER
#define SBITS_COST_POWER 2
#endif
static_assert(SBITS_COST_POWER == 1 || SBITS_COST_POWER == 2, "cost power is 1 or 2");

// value held by lane j*SP + SLOT of the caller's lane group, j in [0, LPG/SP)
template <int LPG, int SP, int SLOT>
__device__ __forceinline__ float bcast_row(float v, int j)
{
    constexpr int RPG = LPG / SP;
    if (RPG <= 1 || j == 0) return group_bcast<LPG, SLOT>(v);
    if (RPG >= 2 && j == 1) return group_bcast<LPG, (1 * SP + SLOT) % LPG>(v);
    if (RPG >= 4 && j == 2) return group_bcast<LPG, (2 * SP + SLOT) % LPG>(v);
    return group_bcast<LPG, (3 * SP + SLOT) % LPG>(v);
}

// Per-lane constants of the distributed grid divisions.  The 2K quotients of a
// row (slot 2c: qmax_c / R, slot 2c+1: R / qmax_c) are spread over the lanes of
// the group, one division per lane, and broadcast afterwards.  When the group
// has more lanes than slots, RP rows share one round of divisions.
template <int LPG, int K>
struct DivPlan {
    static constexpr int SP = (2 * K <= 2) ? 2 : (2 * K <= 4) ? 4 : (2 * K <= 8) ? 8 : 16;   // slots per row
    static constexpr int RP0 = (LPG >= SP) ? (LPG / SP) : 1;
    static constexpr int RP = RP0 < COST_MAX_ROUND ? RP0 : COST_MAX_ROUND;                                         // rows per round
    static constexpr int NS = (LPG >= SP) ? 1 : (2 * K + LPG - 1) / LPG;                       // divisions per lane
    float qf[NS], thr[NS];
    bool is_scale[NS];
    int my_row;

    __device__ __forceinline__ void init(const GridConsts &gc, int lig)
    {
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const int slot = (LPG >= SP) ? (lig % SP) : (lig + t * LPG);
            int c = slot >> 1;
            c = c < K ? c : K - 1;
            float q = gc.qmaxf[0], th = gc.thr[0];
#pragma unroll
            for (int cc = 1; cc < K; ++cc)
                if (c == cc) { q = gc.qmaxf[cc]; th = gc.thr[cc]; }
            qf[t] = q;
            thr[t] = th;
            is_scale[t] = (slot & 1) != 0;
        }
        my_row = (LPG >= SP) ? (lig / SP) : 0;
    }
};

// minimum / maximum of a lane's 8 elements as a chain (three 3-operand instructions and one 2-operand)
__device__ __forceinline__ float min8(const float (&w)[8])
{
    float m = fminf(fminf(w[0], w[1]), w[2]);
    m = fminf(fminf(m, w[3]), w[4]);
    m = fminf(fminf(m, w[5]), w[6]);
    return fminf(m, w[7]);
}
__device__ __forceinline__ float max8(const float (&w)[8])
{
    float m = fmaxf(fmaxf(w[0], w[1]), w[2]);
    m = fmaxf(fmaxf(m, w[3]), w[4]);
    m = fmaxf(fmaxf(m, w[5]), w[6]);
    return fmaxf(m, w[7]);
}

// One round: NI rows (NI <= DivPlan::RP), each owned by the caller's lane group, the lane holding
// 8 consecutive elements of every row: weights w[j][0..7] (bf16 values as floats) and sensitivities
// s[j][0..7].
// out[j][c] = the lane's partial cost of row j at candidate c (elements left to right,
// a = fma(s, d*d, a); with SBITS_COST_POWER == 1: a = fma(s, |d|, a)).
// K counts all candidates.  Z0: candidate 0 is "0 bits" (the block is pruned, paper Sec. 3: its
// change is the weight itself, d = w); the division plan then holds the other K - 1 grids.
// The round has two halves so that a caller may fetch the sensitivities while the first runs:
// quant_cost_prep needs the weights only (row minimum and range, the shared divisions, x = w - min),
// quant_cost_finish scores the candidates.
template <int LPG, int K, int NI, bool Z0>
__device__ __forceinline__ void quant_cost_prep(const float (&w)[NI][8], const DivPlan<LPG, K - Z0> &dp,
                                                float (&x)[NI][8], float (&val)[DivPlan<LPG, K - Z0>::NS])
{
    using DP = DivPlan<LPG, K - Z0>;
    constexpr int NS = DP::NS;
    static_assert(NI >= 1 && NI <= DP::RP, "too many rows for one round of divisions");
    float Rg[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const float mn = group_allreduce<LPG>(min8(w[j]), OpMin{});
        const float mx = group_allreduce<LPG>(max8(w[j]), OpMax{});
        Rg[j] = mx - mn;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[j][e] = w[j][e] - mn;
    }
    float Rsel = Rg[0];
#pragma unroll
    for (int j = 1; j < NI; ++j)
        if (dp.my_row == j) Rsel = Rg[j];
#pragma unroll
    for (int t = 0; t < NS; ++t) {
        const float num = dp.is_scale[t] ? Rsel : dp.qf[t];
        const float den = dp.is_scale[t] ? dp.qf[t] : Rsel;
        const float v = num / den;           // IEEE correctly rounded
        val[t] = (Rsel < dp.thr[t]) ? 0.0f : v;
    }
}

// x * (the value lane LANE of the caller's 16-lane row holds in val): the broadcast rides on the multiply
// (v_mul_f32 with a DPP source) instead of taking a move of its own.  val must have been written at least
// two instructions earlier (the hardware does not interlock a DPP read after a vector write): callers
// pass it through dpp_settle() first.
template <int LANE>
__device__ __forceinline__ float mul_bcast16(float val, float x)
{
    float t;
    asm("v_mul_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1"
        : "=v"(t) : "v"(val), "v"(x), "n"(LANE));
    return t;
}
__device__ __forceinline__ void dpp_settle(float &val) { asm volatile("s_nop 1" : "+v"(val)); }

// RIDE_OK: let the reciprocal's broadcast ride on the multiply where the group is a DPP row (see
// mul_bcast16; a kernel that is short of registers does better without: the compiler cannot
// reschedule around those multiplies as freely).
template <int LPG, int K, int NI, bool Z0, bool RIDE_OK = false>
__device__ __forceinline__ void quant_cost_finish(const float (&w)[NI][8], const float (&x)[NI][8],
                                                  const float (&val)[DivPlan<LPG, K - Z0>::NS],
                                                  const float (&s)[NI][8], float (&out)[NI][K])
{
    using DP = DivPlan<LPG, K - Z0>;
    constexpr int SP = DP::SP;
    constexpr bool RIDE = RIDE_OK && LPG == 16 && LPG >= SP;   // the reciprocal's broadcast rides on the multiply
    float v0 = val[0];
    if constexpr (RIDE) dpp_settle(v0);
    static_for<0, NI>([&](auto ij) {
        constexpr int j = decltype(ij)::value;
        if constexpr (Z0) {
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                acc = fmaf(s[j][e], SBITS_COST_POWER == 1 ? fabsf(w[j][e]) : w[j][e] * w[j][e], acc);
            out[j][0] = acc;
        }
        static_for<0, K - Z0>([&](auto ic) {
            constexpr int c = decltype(ic)::value;
            float inv = 0.0f, scl;
            if constexpr (RIDE) {
                scl = bcast_row<LPG, SP, 2 * c + 1>(v0, j);
            } else if constexpr (LPG >= SP) {
                inv = bcast_row<LPG, SP, 2 * c>(val[0], j);
                scl = bcast_row<LPG, SP, 2 * c + 1>(val[0], j);
            } else {
                inv = group_bcast<LPG, (2 * c) % LPG>(val[(2 * c) / LPG]);
                scl = group_bcast<LPG, (2 * c + 1) % LPG>(val[(2 * c + 1) / LPG]);
            }
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float t;
                if constexpr (RIDE) t = mul_bcast16<((LPG / SP > 1 ? j : 0) * SP + 2 * c) % 16>(v0, x[j][e]);
                else t = x[j][e] * inv;
                const float q = rintf(t);
                const float d = fmaf(-q, scl, x[j][e]);
                acc = fmaf(s[j][e], SBITS_COST_POWER == 1 ? fabsf(d) : d * d, acc);
            }
            out[j][Z0 + c] = acc;
        });
    });
}

template <int LPG, int K, int NI, bool Z0, bool RIDE_OK = false>
__device__ __forceinline__ void quant_cost_round_f(const float (&w)[NI][8], const float (&s)[NI][8],
                                                   const DivPlan<LPG, K - Z0> &dp, float (&out)[NI][K])
{
    float x[NI][8], val[DivPlan<LPG, K - Z0>::NS];
    quant_cost_prep<LPG, K, NI, Z0>(w, dp, x, val);
    quant_cost_finish<LPG, K, NI, Z0, RIDE_OK>(w, x, val, s, out);
}

// the same from raw bf16 weights (8 consecutive elements per 128-bit word)
template <int LPG, int K, int NI, bool Z0>
__device__ __forceinline__ void quant_cost_round(const uint4 (&wraw)[NI], const float (&s)[NI][8],
                                                 const DivPlan<LPG, K - Z0> &dp, float (&out)[NI][K])
{
    float w[NI][8];
#pragma unroll
    for (int j = 0; j < NI; ++j) unpack8(wraw[j], w[j]);
    quant_cost_round_f<LPG, K, NI, Z0>(w, s, dp, out);
}

// Adjacent-pair tree over the 8 rows of an octet, fed one row at a time: rr is the row's index
// in the octet, t1..t3 hold the pending left operands of the three levels.  Returns the value of
// the deepest level completed by this row (the octet's sum when rr == 7).
__device__ __forceinline__ float octet_tree_push(float v, int rr, float &t1, float &t2, float &t3)
{
    if (rr & 1) {
        v = t1 + v;
        if (rr & 2) {
            v = t2 + v;
            if (rr & 4) v = t3 + v;
            else t3 = v;
        } else {
            t2 = v;
        }
    } else {
        t1 = v;
    }
    return v;
}

// The same for a row index that is only known at run time (but uniform over the wave): selects
// instead of branches.  (Sums formed with a not yet written t are discarded by the selects.)
__device__ __forceinline__ float octet_tree_push_rt(float v, int rr, float &t1, float &t2, float &t3)
{
    const bool b1 = (rr & 1) != 0, s2 = (rr & 3) == 1, b2 = (rr & 3) == 3, s3 = (rr & 7) == 3, b3 = (rr & 7) == 7;
    const float v1 = b1 ? t1 + v : v;
    t1 = b1 ? t1 : v;
    const float v2 = b2 ? t2 + v1 : v1;
    t2 = s2 ? v1 : t2;
    const float v3 = b3 ? t3 + v2 : v2;
    t3 = s3 ? v2 : t3;
    return v3;
}

// Two consecutive rows at once: v = (row 2p) + (row 2p + 1), the first level of the tree already
// done; p = pair index in the octet (0..3), run-time uniform.
__device__ __forceinline__ float octet_tree_push_pair_rt(float v, int p, float &t2, float &t3)
{
    const bool b2 = (p & 1) != 0, s3 = (p & 3) == 1, b3 = (p & 3) == 3;
    const float v2 = b2 ? t2 + v : v;
    t2 = b2 ? t2 : v;
    const float v3 = b3 ? t3 + v2 : v2;
    t3 = s3 ? v2 : t3;
    return v3;
}

}  // namespace sbits
