// Arithmetic core of the dynamic-sensitivity surrogates (paper App. "choice of sensitivity
// statistics"): per block at its current bitwidth b,
//   s_up   = sum g * (w - what)        what = fmaf(q, scale, min): the dequantized weight
//   s_down = 2^-b * sum |g * what|
// This header holds the per-row part: the lane's partial sums of both terms over its 8 elements
// (left to right, a = fmaf(g, w - what, a) and a = a + |g * what|).
#pragma once

#include "pack_core.hpp"
#include "sbits_device.hpp"

namespace sbits {

// NI rows ("items"), each owned by the caller's lane group and quantized at its own level k[j];
// weights w[j][0..7] (bf16 values as floats), gradients g[j][0..7].  LPG >= 2 * NI: lane 2j of the group divides
// qmax_j / R_j, lane 2j + 1 divides R_j / qmax_j, so the items share one division sequence.
// out[j][0] = the s_up partial, out[j][1] = the s_down partial (before the 2^-b factor).
template <int LPG, int NI>
__device__ __forceinline__ void surrogate_round(const float (&w)[NI][8], const float (&g)[NI][8],
                                                const LevelConsts (&k)[NI], int lig, float (&out)[NI][2])
{
    static_assert(LPG >= 2 * NI, "one lane per quotient");
    float mn[NI], R[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        float lo = fminf(fminf(fminf(w[j][0], w[j][1]), fminf(w[j][2], w[j][3])),
                         fminf(fminf(w[j][4], w[j][5]), fminf(w[j][6], w[j][7])));
        float hi = fmaxf(fmaxf(fmaxf(w[j][0], w[j][1]), fmaxf(w[j][2], w[j][3])),
                         fmaxf(fmaxf(w[j][4], w[j][5]), fmaxf(w[j][6], w[j][7])));
        lo = group_allreduce<LPG>(lo, OpMin{});
        hi = group_allreduce<LPG>(hi, OpMax{});
        mn[j] = origin_of(k[j], lo);                 // pruned block: what = 0 (origin 0, both quotients 0)
        R[j] = hi - lo;
    }
    const int qi = lig & (2 * NI - 1);               // lanes beyond 2*NI repeat a quotient; nobody reads theirs
    float Rsel = R[0], qf = k[0].qf, th = k[0].th;
#pragma unroll
    for (int j = 1; j < NI; ++j)
        if ((qi >> 1) == j) { Rsel = R[j]; qf = k[j].qf; th = k[j].th; }
    const bool odd = (qi & 1) != 0;
    float v = (odd ? Rsel : qf) / (odd ? qf : Rsel);            // IEEE correctly rounded
    if (Rsel < th) v = 0.0f;
    static_for<0, NI>([&](auto ij) {
        constexpr int j = decltype(ij)::value;
        const float inv = group_bcast<LPG, 2 * j>(v);
        const float scl = group_bcast<LPG, 2 * j + 1>(v);
        float up = 0.0f, dn = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float q = rintf((w[j][e] - mn[j]) * inv);      // 0 <= q <= qmax (see quant_pack_row)
            const float what = fmaf(q, scl, mn[j]);
            up = fmaf(g[j][e], w[j][e] - what, up);
            dn = dn + fabsf(g[j][e] * what);
        }
        out[j][0] = up;
        out[j][1] = dn;
    });
}

}  // namespace sbits
