// Arithmetic core of the packing stage: re-quantization of one block row at the block's chosen
// bitwidth (paper Sec. 5 "Implementation": asymmetric min-max round-to-nearest grid, group =
// one block row) and the little-endian bit string of a lane's 8 codes.  Shared by the kernel
// that reads reordered weights and by the one that reorders on the fly.
#pragma once

#include "sbits_device.hpp"

namespace sbits {

// bitwidth, qmax and the finite-quotient threshold of candidate `lv` (c == 0: a pruned block)
struct LevelConsts {
    int c;
    float qf, th;
    unsigned int qmax;
    unsigned int keep;       // all ones, or 0 for a pruned block: ANDed onto the bits of the group minimum
};
// (one AND per row; a compare-and-select on c here costs the packing kernel 5 %)
__device__ __forceinline__ float origin_of(const LevelConsts &k, float lo)
{
    return __uint_as_float(__float_as_uint(lo) & k.keep);
}
__device__ __forceinline__ LevelConsts level_consts(const GridConsts &gc, int lv)
{
    LevelConsts k;
    k.c = gc.bits[0]; k.qf = gc.qmaxf[0]; k.th = gc.thr[0];
#pragma unroll
    for (int cc = 1; cc < MAX_CAND; ++cc)
        if (lv == cc) { k.c = gc.bits[cc]; k.qf = gc.qmaxf[cc]; k.th = gc.thr[cc]; }
    k.qmax = (unsigned int)k.qf;
    k.keep = k.c ? 0xffffffffu : 0u;
    return k;
}

// One row of one lane group: raw = the lane's 8 bf16 weights.  Returns the lane's 8 codes,
// code e in bits [e*c, (e+1)*c); scl / mn are the row's scale and minimum (same in all lanes
// of the group).  Even lanes divide qmax / R, odd lanes R / qmax.
template <int LPG>
__device__ __forceinline__ unsigned long long quant_pack_row(const uint4 &raw, const LevelConsts &k, bool odd,
                                                             float &scl, float &mn)
{
    float w[8];
    unpack8(raw, w);
    mn = fminf(fminf(fminf(w[0], w[1]), fminf(w[2], w[3])), fminf(fminf(w[4], w[5]), fminf(w[6], w[7])));
    float mx = fmaxf(fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])), fmaxf(fmaxf(w[4], w[5]), fmaxf(w[6], w[7])));
    mn = group_allreduce<LPG>(mn, OpMin{});
    mx = group_allreduce<LPG>(mx, OpMax{});
    const float R = mx - mn;
    mn = origin_of(k, mn);                           // pruned block: origin 0 (both quotients are 0 by its threshold)
    float inv;
    if (LPG >= 2) {
        float v = (odd ? R : k.qf) / (odd ? k.qf : R);
        if (R < k.th) v = 0.0f;
        inv = group_bcast<LPG, 0>(v);
        scl = group_bcast<LPG, 1 % LPG>(v);
    } else {
        inv = k.qf / R; scl = R / k.qf;
        if (R < k.th) { inv = 0.0f; scl = 0.0f; }
    }
    // q = rint(y) for 0 <= y < 2^22 sits in the low mantissa bits of y + 1.5 * 2^23 (round to
    // nearest even, as rintf); y <= qmax * (1 + 2^-22) here, so rint(y) <= qmax and the mask only
    // guards the neighbours' bits against non-finite input.  4 codes fit in 32 bits (c <= 8).
    uint32_t half[2];
#pragma unroll
    for (int hq = 0; hq < 2; ++hq) {
        uint32_t acc = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float y = (w[4 * hq + e] - mn) * inv;
            const uint32_t q = __float_as_uint(y + 12582912.0f) & k.qmax;
            acc |= q << (e * k.c);
        }
        half[hq] = acc;
    }
    const unsigned long long word = (unsigned long long)half[0] | ((unsigned long long)half[1] << (4 * k.c));
    return word;
}

// RS rows of one lane group at once (raw[rs] = the lane's 8 weights of row rs), LPG >= 2 * RS: the
// 2 * RS grid quotients are spread over the lanes of the group (lane 2*rs: qmax / R of row rs,
// lane 2*rs + 1: R / qmax), so the rows share ONE division sequence instead of paying one each.
// Same results as quant_pack_row row by row.
template <int LPG, int RS>
__device__ __forceinline__ void quant_pack_rows(const uint4 (&raw)[RS], const LevelConsts &k, int lig,
                                                unsigned long long (&word)[RS], float (&scl)[RS], float (&mn)[RS])
{
    static_assert(LPG >= 2 * RS, "one lane per quotient");
    float w[RS][8], R[RS];
#pragma unroll
    for (int rs = 0; rs < RS; ++rs) {
        unpack8(raw[rs], w[rs]);
        float lo = fminf(fminf(fminf(w[rs][0], w[rs][1]), fminf(w[rs][2], w[rs][3])),
                         fminf(fminf(w[rs][4], w[rs][5]), fminf(w[rs][6], w[rs][7])));
        float hi = fmaxf(fmaxf(fmaxf(w[rs][0], w[rs][1]), fmaxf(w[rs][2], w[rs][3])),
                         fmaxf(fmaxf(w[rs][4], w[rs][5]), fmaxf(w[rs][6], w[rs][7])));
        lo = group_allreduce<LPG>(lo, OpMin{});
        hi = group_allreduce<LPG>(hi, OpMax{});
        mn[rs] = origin_of(k, lo);                   // pruned block: origin 0 (both quotients are 0 by its threshold)
        R[rs] = hi - lo;
    }
    const int qi = lig & (2 * RS - 1);               // lanes beyond 2*RS repeat a quotient; nobody reads theirs
    float Rsel = R[0];
#pragma unroll
    for (int rs = 1; rs < RS; ++rs)
        if ((qi >> 1) == rs) Rsel = R[rs];
    const bool odd = (qi & 1) != 0;
    float v = (odd ? Rsel : k.qf) / (odd ? k.qf : Rsel);        // IEEE correctly rounded
    if (Rsel < k.th) v = 0.0f;
    static_for<0, RS>([&](auto irs) {
        constexpr int rs = decltype(irs)::value;
        const float inv = group_bcast<LPG, 2 * rs>(v);
        scl[rs] = group_bcast<LPG, 2 * rs + 1>(v);
        uint32_t half[2];
#pragma unroll
        for (int hq = 0; hq < 2; ++hq) {
            uint32_t acc = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float y = (w[rs][4 * hq + e] - mn[rs]) * inv;
                const uint32_t q = __float_as_uint(y + 12582912.0f) & k.qmax;   // see quant_pack_row
                acc |= q << (e * k.c);
            }
            half[hq] = acc;
        }
        word[rs] = (unsigned long long)half[0] | ((unsigned long long)half[1] << (4 * k.c));
    });
}

// ORs the lane's c bytes (c <= 8, held in `word`) into a zeroed LDS strip at byte offset `off` of
// the row that starts at LDS address `row` (4-byte aligned): at most three 32-bit words, the third
// only when c > 4 (`wide`).  No byte-wise stores, no branches.
typedef __attribute__((address_space(3))) uint32_t lds_u32;
__device__ __forceinline__ void or_code_bytes(uint32_t row, int off, unsigned long long word, bool wide)
{
    const int sh = (off & 3) * 8;
    const uint32_t a = row + (uint32_t)(off & ~3);
    const unsigned long long t = word << sh;
    __hip_atomic_fetch_or((lds_u32 *)a, (uint32_t)t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_or((lds_u32 *)(a + 4u), (uint32_t)(t >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (wide) {
        const uint32_t top = sh ? (uint32_t)(word >> (64 - sh)) : 0u;
        __hip_atomic_fetch_or((lds_u32 *)(a + 8u), top, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// the lane's c bytes (c <= 8) of a row's code stream, low byte first; written one by one with
// fixed shifts (a counted loop here gets vectorised into something far more expensive)
template <class BytePtr>
__device__ __forceinline__ void store_code_bytes(BytePtr mine, unsigned long long word, int c)
{
#pragma unroll
    for (int t = 0; t < 8; ++t)
        if (t < c) mine[t] = (unsigned char)(word >> (8 * t));
}

}  // namespace sbits
