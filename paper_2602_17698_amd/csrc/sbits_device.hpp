// Device helpers for gfx950: cross-lane exchange inside a lane group, the
// quantization-grid constants and the bf16 unpack.  A "lane group" is LPG
// adjacent lanes (LPG a power of two, 1..64) that together own one
// quantization group of LPG*8 consecutive weights.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace sbits {

// compile-time loop: f(std::integral_constant<int, I>) for I = I0 .. N-1
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}


// ---- DPP within a row of 16 lanes ------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    // every control used here reads a valid lane, so neither "old" nor bound_ctrl matters;
    // bound_ctrl = 1 spares the initialisation of the destination and lets the compiler
    // fold the move into the instruction that consumes it
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

constexpr int DPP_XOR1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int DPP_MIRROR = 0x140;       // lane i <-> 15-i inside each 16 lanes
constexpr int DPP_BCAST0 = 0x150;       // row_newbcast:0 (+n for lane n of the row)

// Butterfly all-reduce over the LPG lanes of a group.  The exchange pattern is
// an adjacent-pair tree (lanes 2j,2j+1, then pairs of pairs, ...): after the
// quad steps all lanes of a quad agree, so the mirror steps pair quads and
// halves exactly as xor 4 / xor 8 would.  Every lane ends with the same bits.
template <int LPG, class Op>
__device__ __forceinline__ float group_allreduce(float v, Op op)
{
    if (LPG >= 2)  v = op(v, dpp_mov<DPP_XOR1>(v));
    if (LPG >= 4)  v = op(v, dpp_mov<DPP_XOR2>(v));
    if (LPG >= 8)  v = op(v, dpp_mov<DPP_HALF_MIRROR>(v));
    if (LPG >= 16) v = op(v, dpp_mov<DPP_MIRROR>(v));
    if (LPG >= 32) v = op(v, __shfl_xor(v, 16));
    if (LPG >= 64) v = op(v, __shfl_xor(v, 32));
    return v;
}

struct OpAdd { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMin { __device__ __forceinline__ float operator()(float a, float b) const { return fminf(a, b); } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };

// value held by lane J of the caller's lane group
template <int LPG, int J>
__device__ __forceinline__ float group_bcast(float v)
{
    if (LPG == 1) return v;
    if (LPG == 16) return dpp_mov<DPP_BCAST0 + (J & 15)>(v);
    const int lane = (int)(threadIdx.x & 63);
    return __shfl(v, (lane & ~(LPG - 1)) + J);
}

// ---- loads through a pointer that is known to be global memory ------------------
// (pointers read from a descriptor are generic for the compiler; saying "global" gives
// global_load instead of flat_load)
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 gload_f4(const void *p)
{
    const f32x4_t v = *(const __attribute__((address_space(1))) f32x4_t *)p;
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 gload_u4(const void *p)
{
    const u32x4_t v = *(const __attribute__((address_space(1))) u32x4_t *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- batched launches: one descriptor per matrix of the plan -------------------
struct MatDesc {
    const uint16_t *w;        // original weights (bf16) and sensitivities, caller's pointers
    const float *s;
    int64_t rows, cols, ld_w, ld_s;
    int64_t elem_off;         // element offset of the dense reordered copy in the concatenated arrays
    int64_t block_base;       // first global block id
    int64_t row_off, col_off; // offsets into the concatenated row / column permutations
    int nbr, nbc;             // block grid
    int nseg, nband;          // score partials: 512-column segments, 256-row bands
    int64_t rowpart_off, colpart_off;   // offsets of this matrix's score partials
};

// largest i with wg_start[i] <= wg  (wg_start has n + 1 ascending entries, wg_start[0] = 0)
__device__ __forceinline__ int find_matrix(const int *__restrict__ wg_start, int n, int wg)
{
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (wg_start[mid] <= wg) lo = mid; else hi = mid;
    }
    return lo;
}

// ---- quantization grid constants, one set per candidate ---------------------
// Candidate bitwidths are 0 .. 8, ascending: at most MAX_CAND of them.  0 bits = the block is pruned
// (paper Sec. 3): stored value 0, no codes; its entry has qmax 0 and an infinite threshold, which
// makes both grid quotients 0 wherever a level's constants are used (the origin is forced to 0 there).
constexpr int MAX_CAND = 9;
struct GridConsts {
    float qmaxf[MAX_CAND];   // 2^c - 1
    float thr[MAX_CAND];     // smallest range R for which qmax / R is finite
    int   bits[MAX_CAND];
};

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// 8 consecutive bf16 (one 128-bit load) -> 8 floats, element order preserved
__device__ __forceinline__ void unpack8(const uint4 &p, float (&w)[8])
{
    w[0] = bf16_lo(p.x); w[1] = bf16_hi(p.x);
    w[2] = bf16_lo(p.y); w[3] = bf16_hi(p.y);
    w[4] = bf16_lo(p.z); w[5] = bf16_hi(p.z);
    w[6] = bf16_lo(p.w); w[7] = bf16_hi(p.w);
}

}  // namespace sbits
