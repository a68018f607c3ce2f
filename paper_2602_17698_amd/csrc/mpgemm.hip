// Product of a small batch of activations with the stored mixed-precision weights (paper Sec. 5.3
// "Inference Kernel": dequantization fused into the matrix product, at the granularity of the
// precision blocks, one bitwidth per tile, no divergence inside a wave):
//
//     y[b][i] = sum_j What[i][j] * x[b][j],      What[i][j] = q[i][j] * scale[i][J] + zero[i][J]
//
// for one matrix of the plan, read straight from the packed stream of sbits_pack (blocks in global
// order, rows of a block one after the other, LSB-first codes, scale / zero per block row).
//
// The sum over a block row's n columns splits as  scale * (sum_j q x) + zero * (sum_j x):
// the matrix cores multiply the integer codes (exact in bf16) with x, a second product with
// an all-ones operand gives sum_j x in the same register layout, and two fp32 FMAs per output and
// block apply the row's scale and zero.  For bitwidths below 8 the codes enter as bf16 128 + q
// (the code OR-ed into the mantissa of 128.0: no integer-to-float conversion), and the offset is
// folded into the zero term: zero' = zero - 128 * scale.
//
// Mapping (v_mfma_f32_16x16x32_bf16: A = x, 16 batch rows; B = What^T, 16 output channels; K = 32):
//   lane l supplies channel i = l % 16 and the K-quarter g = l / 16 of a block row: its n / 4 codes
//   are n * c / 32 consecutive bytes of the stream; the wave's 16 rows x n codes are one contiguous
//   run.  A workgroup of 16 waves covers 128 rows (4 row groups of 32 = 2 channel tiles each) x 16
//   block columns (4 waves per row group, 4 blocks per wave, two or three of them in flight in a ring
//   of register slots); the x slice of those columns sits in LDS.  Block columns beyond the first 16
//   go to further workgroups (grid.y), whose partial sums a second kernel adds in a fixed order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sbits_internal.hpp"

namespace sbits {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4v_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x3_t __attribute__((ext_vector_type(3)));

constexpr int MG_WAVES = 16, MG_THREADS = MG_WAVES * 64;
constexpr int MG_RG = 4;                 // row groups (32 rows) per workgroup
constexpr int MG_JL = 4;                 // waves per row group, each on its own block columns
constexpr int MG_NBLK = 4;               // blocks per wave
constexpr int MG_SPAN = MG_JL * MG_NBLK; // block columns per workgroup

struct MpArgs {
    const uint8_t *codes;
    const float *scale, *zero;
    const uint8_t *level;
    const int64_t *byte_off;
    const uint16_t *x;                   // bf16 [batch][ld_x]
    float *out;                          // y [batch][R] (n_split == 1) or partials [n_split][batch][R]
    int64_t block_base, ld_x;
    int R, C, m, nbc, batch, n_split;
    int bits[MAX_CAND];
};

__device__ __forceinline__ bf16x8_t as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    u32x4_t v;
    v.x = a; v.y = b; v.z = c; v.w = d;
    return __builtin_bit_cast(bf16x8_t, v);
}

// The lane's codes of one block row quarter: C dwords (C = 0: an absent block, nothing needed).
// Always exactly two load instructions, whatever C is: the first brings min(C, 4) dwords, the second
// the rest or, if there is no rest, dword 0 once more into r[7] (kept alive by the consumer).  With
// the same number of loads on every path the compiler can count the loads still in flight, and a
// block's product waits for its own codes only, not for those of the blocks behind it.
template <int C>
__device__ __forceinline__ void load_codes(const uint8_t *p, uint32_t (&r)[8])
{
    const __attribute__((address_space(1))) uint32_t *q = (const __attribute__((address_space(1))) uint32_t *)p;
    constexpr int A = C == 0 ? 1 : (C < 4 ? C : 4);
    if constexpr (A == 1) r[0] = q[0];
    else if constexpr (A == 2) { const u32x2_t v = *(const __attribute__((address_space(1))) u32x2_t *)q; r[0] = v.x; r[1] = v.y; }
    else if constexpr (A == 3) { const u32x3_t v = *(const __attribute__((address_space(1))) u32x3_t *)q; r[0] = v.x; r[1] = v.y; r[2] = v.z; }
    else { const u32x4_t v = *(const __attribute__((address_space(1))) u32x4_t *)q; r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w; }
    if constexpr (C <= 4) { r[7] = __builtin_nontemporal_load(q); }
    else if constexpr (C == 5) r[4] = q[4];
    else if constexpr (C == 6) { const u32x2_t v = *(const __attribute__((address_space(1))) u32x2_t *)(q + 4); r[4] = v.x; r[5] = v.y; }
    else if constexpr (C == 7) { const u32x3_t v = *(const __attribute__((address_space(1))) u32x3_t *)(q + 4); r[4] = v.x; r[5] = v.y; r[6] = v.z; }
    else { const u32x4_t v = *(const __attribute__((address_space(1))) u32x4_t *)(q + 4); r[4] = v.x; r[5] = v.y; r[6] = v.z; r[7] = v.w; }
}

// code e (0 .. 8 * words - 1) of the lane's LSB-first stream, C bits
template <int C>
__device__ __forceinline__ uint32_t code_at(const uint32_t (&r)[8], int e)
{
    const int bit = e * C, idx = bit >> 5, sh = bit & 31;
    uint32_t v = r[idx] >> sh;
    if (sh + C > 32) v |= r[idx + 1] << (32 - sh);
    return v & ((1u << C) - 1u);
}

// B operand of step `st`: the lane's codes 8 * st .. 8 * st + 7 as bf16, in stream order.
// C < 8: 128 + q (the code in the mantissa of 128.0);  C == 8: q itself (converted).
template <int C>
__device__ __forceinline__ bf16x8_t operand(const uint32_t (&r)[8], int st)
{
    uint32_t w[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t q0 = code_at<C>(r, 8 * st + 2 * p), q1 = code_at<C>(r, 8 * st + 2 * p + 1);
        if constexpr (C < 8) {
            w[p] = 0x43004300u | q0 | (q1 << 16);
        } else {
            const uint32_t f0 = __float_as_uint((float)q0), f1 = __float_as_uint((float)q1);   // <= 8 significant bits
            w[p] = (f0 >> 16) | (f1 & 0xffff0000u);
        }
    }
    return as_bf16x8(w[0], w[1], w[2], w[3]);
}

// ---- pair order (bitwidths 1, 2, 4): a 32-bit word holds two codes 16 bits apart, so one AND-OR
// turns  (w >> s) & mask  into the bf16 pair (128 + q_a, 128 + q_b) with b - a = 16 / C codes.
// The operand then holds the lane's codes in the order a0, b0, a1, b1, ...; x is put into the
// same order with byte permutes (x_operand; shared by both channel tiles).
//   C = 4: step st, pair p: codes (8 st + p,        8 st + p + 4)     word st,      shift 4 p
//   C = 2: step st, pair p: codes (16 d + 4 h + p,  ... + 8)          word d,       shift 2 (4 h + p),  st = 2 d + h
//   C = 1: step st, pair p: codes (4 st + p,        4 st + p + 16)    word 0,       shift 4 st + p      (32 codes per lane only)
template <int C, int KL>
struct PairOrder {
    static constexpr bool value = C == 4 || C == 2 || (C == 1 && KL == 32);
};

template <int C>
__device__ __forceinline__ bf16x8_t operand_pairs(const uint32_t (&r)[8], int st)
{
    uint32_t w[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if constexpr (C == 4) w[p] = ((r[st] >> (4 * p)) & 0x000f000fu) | 0x43004300u;
        else if constexpr (C == 2) w[p] = ((r[st >> 1] >> (2 * (4 * (st & 1) + p))) & 0x00030003u) | 0x43004300u;
        else w[p] = ((r[0] >> (4 * st + p)) & 0x00010001u) | 0x43004300u;
    }
    return as_bf16x8(w[0], w[1], w[2], w[3]);
}

// x operand of step st, read from the lane's 2 * KL bytes of the staged slice (natural order in LDS).
// Stream order: the step's 16 bytes as they are.  Pair order of bitwidth C: the two elements of pair
// p sit in the same half of two words 16 / C codes apart, fetched as two 8-byte reads and merged
// with byte permutes.
template <int C, bool PAIRS>
__device__ __forceinline__ bf16x8_t x_operand(const unsigned char *xl, int st)
{
    if constexpr (!PAIRS) {
        return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(xl + 16 * st));
    } else {
        int ea, gap;                                  // first element of pair 0; distance to its partner
        if constexpr (C == 4) { ea = 8 * st; gap = 4; }
        else if constexpr (C == 2) { ea = 16 * (st >> 1) + 4 * (st & 1); gap = 8; }
        else { ea = 4 * st; gap = 16; }
        // pairs p = 0..3 use elements ea + p and ea + p + gap: words (ea >> 1) + {0, 1} and the same + gap / 2
        const u32x2_t wa = *reinterpret_cast<const u32x2_t *>(xl + 2 * ea);
        const u32x2_t wb = *reinterpret_cast<const u32x2_t *>(xl + 2 * (ea + gap));
        uint32_t w[4];
        w[0] = __builtin_amdgcn_perm(wb.x, wa.x, 0x05040100u);
        w[1] = __builtin_amdgcn_perm(wb.x, wa.x, 0x07060302u);
        w[2] = __builtin_amdgcn_perm(wb.y, wa.y, 0x05040100u);
        w[3] = __builtin_amdgcn_perm(wb.y, wa.y, 0x07060302u);
        return as_bf16x8(w[0], w[1], w[2], w[3]);
    }
}

// One block: loads were issued before (cw, sc, ze); multiply and add into acc.
template <int C, int N_COLS, int NB>
__device__ __forceinline__ void block_product(const uint32_t (&cw)[2][8], const float (&sc)[2], const float (&ze)[2],
                                              const unsigned char *const (&xl)[NB], f32x4v_t (&acc)[2][NB])
{
    constexpr int STEPS = N_COLS / 32;
    constexpr bool PAIRS = PairOrder<C, N_COLS / 4>::value;
    if constexpr (C <= 4 && N_COLS == 128) asm volatile("" :: "v"(cw[0][7]), "v"(cw[1][7]));   // the second load of load_codes
    const bf16x8_t ones = as_bf16x8(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
    f32x4v_t d[2][NB], d1[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        d1[nb] = f32x4v_t{0.0f, 0.0f, 0.0f, 0.0f};
        d[0][nb] = d1[nb];
        d[1][nb] = d1[nb];
    }
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
        bf16x8_t b0, b1;
        if constexpr (PAIRS) { b0 = operand_pairs<C>(cw[0], st); b1 = operand_pairs<C>(cw[1], st); }
        else { b0 = operand<C>(cw[0], st); b1 = operand<C>(cw[1], st); }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const bf16x8_t xa = x_operand<C, PAIRS>(xl[nb], st);
            d[0][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, b0, d[0][nb], 0, 0, 0);
            d[1][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, b1, d[1][nb], 0, 0, 0);
            d1[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, ones, d1[nb], 0, 0, 0);
        }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const float zz = C < 8 ? fmaf(-128.0f, sc[t], ze[t]) : ze[t];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[t][nb][r] = fmaf(sc[t], d[t][nb][r], fmaf(zz, d1[nb][r], acc[t][nb][r]));
    }
}

// Codes, scales and zeros of block T of a wave -> register slot S; the same number of load
// instructions whatever the block.  c = 0: a block column beyond the matrix, or a pruned block (0 bits:
// no codes, contributes nothing); its dummy loads read the first dword of the scales, which always
// exists, and the clamped block's scales.  (A macro: through a function the slots end up in scratch memory.)
#define MG_REQUEST(T, S)                                                                                          \
    do {                                                                                                          \
        const int c_ = cbits[T];                                                                                  \
        const uint8_t *pb_ = c_ ? a.codes + (int64_t)(((uint64_t)off_hi[T] << 32) | off_lo[T])                    \
                                : reinterpret_cast<const uint8_t *>(a.scale);                                     \
        const float *ps_ = a.scale + blk[T] * a.m + rin, *pz_ = a.zero + blk[T] * a.m + rin;                      \
        _Pragma("unroll") for (int tl = 0; tl < 2; ++tl) {                                                        \
            const uint8_t *p_ = pb_ + (lane_units + (uint32_t)(tl * 16 * (N_COLS / 8))) * (uint32_t)c_;           \
            sc[S][tl] = ps_[16 * tl + li];                                                                        \
            ze[S][tl] = pz_[16 * tl + li];                                                                        \
            if constexpr (KL == 32) {                                                                             \
                switch (c_) {                                                                                     \
                case 0: load_codes<0>(p_, cw[S][tl]); break;                                                      \
                case 1: load_codes<1>(p_, cw[S][tl]); break;                                                      \
                case 2: load_codes<2>(p_, cw[S][tl]); break;                                                      \
                case 3: load_codes<3>(p_, cw[S][tl]); break;                                                      \
                case 4: load_codes<4>(p_, cw[S][tl]); break;                                                      \
                case 5: load_codes<5>(p_, cw[S][tl]); break;                                                      \
                case 6: load_codes<6>(p_, cw[S][tl]); break;                                                      \
                case 7: load_codes<7>(p_, cw[S][tl]); break;                                                      \
                default: load_codes<8>(p_, cw[S][tl]); break;                                                     \
                }                                                                                                 \
            } else {                                                                                              \
                /* 2 * c bytes: 16-bit halves (the stream is only 2-byte aligned here) */                         \
                const __attribute__((address_space(1))) uint16_t *h_ =                                            \
                    (const __attribute__((address_space(1))) uint16_t *)p_;                                       \
                _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                     \
                    if (i < c_)                                                                                   \
                        cw[S][tl][i >> 1] = (i & 1) ? (cw[S][tl][i >> 1] | ((uint32_t)h_[i] << 16)) : (uint32_t)h_[i]; \
            }                                                                                                     \
        }                                                                                                         \
    } while (0)

template <int N_COLS, int NB>
__global__ __launch_bounds__(MG_THREADS)
void mp_gemm_kernel(MpArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int KL = N_COLS / 4, STEPS = N_COLS / 32;
    constexpr int SLICE = MG_SPAN * N_COLS;                    // x columns per workgroup
    constexpr int PITCH = SLICE * 2 + 16;                      // bytes per batch row in LDS (+16: spreads the rows over the banks)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: the bookkeeping below stays scalar
    const int rg = wave & (MG_RG - 1), jl = wave >> 2;
    const int li = lane & 15, g = lane >> 4;
    const int col0 = blockIdx.y * SLICE;                       // first x column of the slice
    const int J0 = blockIdx.y * MG_SPAN;

    // ---- this wave's blocks: all metadata loads first (they head the longest dependency chain);
    // a block column beyond the matrix reads the last one's metadata and is skipped later
    const int row0 = blockIdx.x * (MG_RG * 32) + rg * 32;      // first of the wave's 32 rows
    const bool rows_ok = row0 < a.R;                           // (R is a multiple of 32)
    const int I = rows_ok ? row0 / a.m : 0, rin = rows_ok ? row0 - I * a.m : 0;
    // PF blocks of codes are in flight at a time (a ring of PF register slots, refilled after each
    // block): three with one batch tile (measured: 15.0 us against 15.3 with two and 16.3 with all four
    // requested at once, whose first block then arrives late), two with two batch tiles (registers)
    constexpr int PF = NB == 1 ? 3 : 2;
    int cbits[MG_NBLK];
    uint32_t cw[PF][2][8];
    float sc[PF][2], ze[PF][2];
    int64_t blk[MG_NBLK];
    uint32_t lvl_v[MG_NBLK];
    int64_t boff_v[MG_NBLK];
#pragma unroll
    for (int t = 0; t < MG_NBLK; ++t) {
        const int J = J0 + jl + MG_JL * t;
        blk[t] = a.block_base + (int64_t)I * a.nbc + (J < a.nbc ? J : a.nbc - 1);
        lvl_v[t] = a.level[blk[t]];
        boff_v[t] = a.byte_off[blk[t]];
    }
    // ---- x slice: requested together with the metadata (rows beyond the batch and columns beyond C read
    // as zero) and in LDS by the time the metadata has arrived
    constexpr int XCH = 16 * NB * (SLICE / 8) / MG_THREADS;    // 16-byte pieces per thread
    static_assert(16 * NB * (SLICE / 8) % MG_THREADS == 0, "whole pieces per thread");
    u32x4_t xs[XCH];
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
        const int q = tid + i * MG_THREADS;
        const int b = q / (SLICE / 8), ch = q - b * (SLICE / 8);
        const int bc = b < a.batch ? b : a.batch - 1;                               // in bounds; zeroed below
        const int cc = col0 + ch * 8 < a.C ? col0 + ch * 8 : 0;
        xs[i] = *(const __attribute__((address_space(1))) u32x4_t *)(a.x + (int64_t)bc * a.ld_x + cc);
    }

#pragma unroll
    for (int i = 0; i < XCH; ++i) {
        const int q = tid + i * MG_THREADS;
        const int b = q / (SLICE / 8), ch = q - b * (SLICE / 8);
        const bool ok = b < a.batch && col0 + ch * 8 < a.C;
        u32x4_t v = xs[i];
        v.x = ok ? v.x : 0u; v.y = ok ? v.y : 0u; v.z = ok ? v.z : 0u; v.w = ok ? v.w : 0u;
        *reinterpret_cast<u32x4_t *>(smem + (size_t)b * PITCH + ch * 16) = v;
    }
    // (no global load is in flight here but the metadata: the codes are requested after the barrier)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the x slice is in LDS
    const uint32_t lane_units = (uint32_t)((rin + li) * (N_COLS / 8) + g * (KL / 8));   // x c = the lane's byte offset in the block
    // the blocks' bitwidths and stream offsets as scalars
    uint32_t off_lo[MG_NBLK], off_hi[MG_NBLK];
#pragma unroll
    for (int t = 0; t < MG_NBLK; ++t) {
        const int J = J0 + jl + MG_JL * t;
        const int lv = __builtin_amdgcn_readfirstlane((int)lvl_v[t]);
        int c = a.bits[0];
#pragma unroll
        for (int k = 1; k < MAX_CAND; ++k) c = lv == k ? a.bits[k] : c;
        cbits[t] = (rows_ok && J < a.nbc) ? c : 0;
        off_lo[t] = __builtin_amdgcn_readfirstlane((uint32_t)boff_v[t]);
        off_hi[t] = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)boff_v[t] >> 32));
    }
#pragma unroll
    for (int t = 0; t < PF; ++t) MG_REQUEST(t, t);

    f32x4v_t acc[2][NB];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[t][nb] = f32x4v_t{0.0f, 0.0f, 0.0f, 0.0f};

#pragma unroll
    for (int t = 0; t < MG_NBLK; ++t) {
        const int c = cbits[t];
        const int Jl = jl + MG_JL * t;                         // block column inside the slice
        const unsigned char *xa[NB];                           // the lane's x values of this block column (LDS, natural order)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            xa[nb] = smem + (size_t)(16 * nb + li) * PITCH + (size_t)(Jl * N_COLS + g * KL) * 2;
        if (c != 0) switch (c) {                               // (0: no such block column, or a pruned block)
        case 1: block_product<1, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        case 2: block_product<2, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        case 3: block_product<3, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        case 4: block_product<4, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        case 5: block_product<5, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        case 6: block_product<6, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        case 7: block_product<7, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        default: block_product<8, N_COLS, NB>(cw[t % PF], sc[t % PF], ze[t % PF], xa, acc); break;
        }
        if (t + PF < MG_NBLK) MG_REQUEST((t + PF) % MG_NBLK, t % PF);   // the slot is free again
    }

    // ---- the four waves of a row group add up (fixed order), wave jl = 0 stores
    __syncthreads();                                           // every wave is done with the x slice
    float *red = reinterpret_cast<float *>(smem);              // [wave][tile][nb][r][lane]
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                red[(((wave * 2 + t) * NB + nb) * 4 + r) * 64 + lane] = acc[t][nb][r];
    __syncthreads();
    if (jl != 0 || !rows_ok) return;
    float *dst = a.out + (int64_t)blockIdx.y * a.batch * a.R;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[t][nb][r];
#pragma unroll
                for (int j = 1; j < MG_JL; ++j)
                    v = v + red[((((rg + MG_RG * j) * 2 + t) * NB + nb) * 4 + r) * 64 + lane];
                const int b = 16 * nb + 4 * g + r;             // D layout: row 4 * (lane / 16) + r, column lane % 16
                if (b < a.batch) dst[(int64_t)b * a.R + row0 + 16 * t + li] = v;
            }
}

// y = sum over the column splits of the partials, split 0 first
__global__ __launch_bounds__(256)
void mp_gemm_finish_kernel(const float *__restrict__ part, int64_t n, int n_split, float *__restrict__ y)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float v = part[i];
    for (int s = 1; s < n_split; ++s) v = v + part[(int64_t)s * n + i];
    y[i] = v;
}

}  // namespace sbits

using namespace sbits;

int sbits_mp_gemm_splits(int64_t cols, int n) { return (int)((cols / n + MG_SPAN - 1) / MG_SPAN); }

bool sbits_mp_gemm_shapes_ok(const sbits_plan *plan)
{
    return (plan->n == 64 || plan->n == 128) && plan->m % 32 == 0;
}

// partial sums of the largest matrix at the largest batch (32)
size_t sbits_mp_gemm_ws_bytes(const sbits_plan *plan)
{
    if (!sbits_mp_gemm_shapes_ok(plan)) return 0;
    size_t mx = 0;
    for (int i = 0; i < plan->n_mats; ++i) {
        const int s = sbits_mp_gemm_splits(plan->cols[i], plan->n);
        const size_t b = s > 1 ? (size_t)s * 32 * (size_t)plan->rows[i] * 4 : 0;
        if (b > mx) mx = b;
    }
    return sbits_align_up(mx, 256);
}

template <int N_COLS, int NB>
static int launch_mp(sbits_ctx *ctx, const MpArgs &a, dim3 grid)
{
    constexpr size_t x_bytes = (size_t)16 * NB * (MG_SPAN * N_COLS * 2 + 16);
    constexpr size_t red_bytes = (size_t)MG_WAVES * 2 * NB * 4 * 64 * 4;
    constexpr size_t lds = x_bytes > red_bytes ? x_bytes : red_bytes;
    auto *fn = &mp_gemm_kernel<N_COLS, NB>;
    SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds));
    hipLaunchKernelGGL(fn, grid, dim3(MG_THREADS), lds, ctx->stream, a);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

int sbits_launch_mp_gemm(sbits_plan *plan, int mat, const void *x_bf16, int64_t ld_x, int batch,
                         const uint8_t *level, const int64_t *byte_off, const uint8_t *codes, const float *scale,
                         const float *zero, float *y, void *scratch)
{
    sbits_ctx *ctx = plan->ctx;
    MpArgs a;
    a.codes = codes; a.scale = scale; a.zero = zero; a.level = level; a.byte_off = byte_off;
    a.x = static_cast<const uint16_t *>(x_bf16);
    a.block_base = plan->base[mat]; a.ld_x = ld_x;
    a.R = (int)plan->rows[mat]; a.C = (int)plan->cols[mat]; a.m = plan->m; a.nbc = a.C / plan->n;
    a.batch = batch;
    a.n_split = sbits_mp_gemm_splits(a.C, plan->n);
    for (int c = 0; c < sbits::MAX_CAND; ++c) a.bits[c] = c < plan->K ? plan->bits[c] : plan->bits[plan->K - 1];
    a.out = a.n_split > 1 ? static_cast<float *>(scratch) : y;
    const dim3 grid((unsigned)((a.R + MG_RG * 32 - 1) / (MG_RG * 32)), (unsigned)a.n_split);
    const int nb = batch <= 16 ? 1 : 2;
    int rc;
    if (plan->n == 128) rc = nb == 1 ? launch_mp<128, 1>(ctx, a, grid) : launch_mp<128, 2>(ctx, a, grid);
    else rc = nb == 1 ? launch_mp<64, 1>(ctx, a, grid) : launch_mp<64, 2>(ctx, a, grid);
    if (rc) return rc;
    if (a.n_split > 1) {
        const int64_t n = (int64_t)batch * a.R;
        hipLaunchKernelGGL(mp_gemm_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream,
                           (const float *)scratch, n, a.n_split, y);
        SBITS_HIP(ctx, hipGetLastError());
    }
    return SBITS_OK;
}
