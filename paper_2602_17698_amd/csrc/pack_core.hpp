// Arithmetic core of the packing stage: re-quantization of one block row at the block's chosen
// bitwidth (paper Sec. 5 "Implementation": asymmetric min-max round-to-nearest grid, group =
// one block row) and the little-endian bit string of a lane's 8 codes.  Shared by the kernel
// that reads reordered weights and by the one that reorders on the fly.
#pragma once

#include "sbits_device.hpp"

namespace sbits {

// bitwidth, qmax and the finite-quotient threshold of candidate `lv`
struct LevelConsts {
    int c;
    float qf, th;
    unsigned int qmax;
};
__device__ __forceinline__ LevelConsts level_consts(const GridConsts &gc, int lv)
{
    LevelConsts k;
    k.c = gc.bits[0]; k.qf = gc.qmaxf[0]; k.th = gc.thr[0];
#pragma unroll
    for (int cc = 1; cc < 8; ++cc)
        if (lv == cc) { k.c = gc.bits[cc]; k.qf = gc.qmaxf[cc]; k.th = gc.thr[cc]; }
    k.qmax = (unsigned int)k.qf;
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
