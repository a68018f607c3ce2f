// The stored matrix back as numbers (paper Sec. 5.3: codes with one bitwidth per tile, scale and
// zero per block row): What[i][j] = fmaf(code, scale, zero), in the reordered coordinates the stream
// was packed in, as fp32 (exact: this is the format's definition of the stored value) or rounded to
// bf16 (nearest even).  A utility beside the inference product: for evaluating a quantized model
// with ordinary dense kernels, and for checking.  Write-bound: c / 8 bytes read, 4 (or 2) written
// per weight.
//
// One lane per run of 8 codes of a block row (c bytes of the stream, at any byte alignment): three
// aligned dwords cover them, a funnel shift lines them up, eight field extractions follow; the lanes
// of a wave write 2 KiB (fp32) of one row contiguously.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sbits_internal.hpp"

namespace sbits {

struct DequantArgs {
    const uint8_t *codes;
    const float *scale, *zero;
    const uint8_t *level;
    const int64_t *byte_off;
    void *out;
    int64_t block_base, ld_out;
    int R, C, m, n, nbc;
    int bits[MAX_CAND];
};

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;           // finite input (the format stores finite values)
}

template <bool BF16>
__global__ __launch_bounds__(256)
void dequant_kernel(DequantArgs a)
{
    const int jc = (int)(blockIdx.x * 256 + threadIdx.x);     // run of 8 columns
    const int i = (int)blockIdx.y;                            // row
    if (jc * 8 >= a.C) return;
    const int I = i / a.m, r = i - I * a.m;
    const int J = (jc * 8) / a.n, cin = jc * 8 - J * a.n;
    const int64_t blk = a.block_base + (int64_t)I * a.nbc + J;
    int lv = a.level[blk];
    int c = a.bits[0];
#pragma unroll
    for (int k = 1; k < MAX_CAND; ++k) c = lv == k ? a.bits[k] : c;
    // the run's c bytes and the aligned dwords around them (the stream ends on a multiple of 8 bytes
    // from a 16-byte aligned base, so a dword that holds one of the run's bytes lies inside it)
    const uint8_t *p = a.codes + a.byte_off[blk] + ((int64_t)r * a.n + cin) / 8 * c;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(p);
    const uint32_t *q = reinterpret_cast<const uint32_t *>(pa & ~(uintptr_t)3);
    const int sh = (int)(pa & 3) * 8;
    const int need = (int)(pa & 3) + c;                       // bytes from q[0] on
    const uint32_t w0 = c ? q[0] : 0u;                        // (a pruned block has no codes: its value is zero[] = 0)
    const uint32_t w1 = need > 4 ? q[1] : 0u;
    const uint32_t w2 = need > 8 ? q[2] : 0u;
    const unsigned long long lo64 = ((unsigned long long)w1 << 32) | w0;
    unsigned long long win = lo64 >> sh;
    if (sh) win |= (unsigned long long)w2 << (64 - sh);
    const float s = a.scale[blk * a.m + r], z = a.zero[blk * a.m + r];
    const unsigned long long mask = (1ull << c) - 1ull;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = fmaf((float)(uint32_t)((win >> (e * c)) & mask), s, z);
    if constexpr (BF16) {
        uint16_t *o = static_cast<uint16_t *>(a.out) + (int64_t)i * a.ld_out + (int64_t)jc * 8;
        u32x4_t t;
        t.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16); t.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
        t.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16); t.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
        __builtin_nontemporal_store(t, (__attribute__((address_space(1))) u32x4_t *)o);
    } else {
        float *o = static_cast<float *>(a.out) + (int64_t)i * a.ld_out + (int64_t)jc * 8;
        const f32x4_t lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
        __builtin_nontemporal_store(lo, (__attribute__((address_space(1))) f32x4_t *)o);
        __builtin_nontemporal_store(hi, (__attribute__((address_space(1))) f32x4_t *)(o + 4));
    }
}

}  // namespace sbits

using namespace sbits;

int sbits_launch_dequant(sbits_plan *plan, int mat, const uint8_t *level, const int64_t *byte_off,
                         const uint8_t *codes, const float *scale, const float *zero, void *out, int64_t ld_out,
                         int out_bf16)
{
    sbits_ctx *ctx = plan->ctx;
    DequantArgs a;
    a.codes = codes; a.scale = scale; a.zero = zero; a.level = level; a.byte_off = byte_off;
    a.out = out; a.block_base = plan->base[mat]; a.ld_out = ld_out;
    a.R = (int)plan->rows[mat]; a.C = (int)plan->cols[mat]; a.m = plan->m; a.n = plan->n; a.nbc = a.C / plan->n;
    for (int c = 0; c < sbits::MAX_CAND; ++c) a.bits[c] = c < plan->K ? plan->bits[c] : plan->bits[plan->K - 1];
    const dim3 grid((unsigned)((a.C / 8 + 255) / 256), (unsigned)a.R);
    if (out_bf16) hipLaunchKernelGGL(dequant_kernel<true>, grid, dim3(256), 0, ctx->stream, a);
    else hipLaunchKernelGGL(dequant_kernel<false>, grid, dim3(256), 0, ctx->stream, a);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}
