// Storage: byte offsets of the blocks and bit-packing of the chosen codes
// (one bitwidth per block, paper Sec. 5.3 "Inference Kernel").
//
// offsets : byte_off[i] = sum_{i' < i} m*n*c[level[i']]/8 (exclusive scan, int64).
// pack    : re-quantizes each block row at the block's bitwidth with the same
//           round-to-nearest grid as the cost table and writes the codes LSB
//           first: element e of the block (row-major) occupies bits
//           [e*c, (e+1)*c) of the block's little-endian bit stream.  A lane owns
//           8 consecutive weights = exactly c bytes of the stream; the lanes of
//           a row stage their bytes in LDS and the row is written out as dwords.
#include "sbits_device.hpp"
#include "sbits_internal.hpp"

void sbits_fill_grid_consts(const int32_t *bits, int K, sbits::GridConsts *gc);

namespace sbits {

// ---- offsets --------------------------------------------------------------------
constexpr int OF_THREADS = 256;
constexpr int OF_ITEMS = 8;
constexpr int OF_TILE = OF_THREADS * OF_ITEMS;

struct BitsTab { int bits[8]; };

__device__ __forceinline__ long long block_exclusive_scan(long long v, long long *total)
{
    __shared__ long long wsum[OF_THREADS / 64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    long long inc = v;
    for (int off = 1; off < 64; off <<= 1) {
        const long long t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    long long base = 0, tot = 0;
    for (int w = 0; w < OF_THREADS / 64; ++w) {
        if (w < wv) base += wsum[w];
        tot += wsum[w];
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(OF_THREADS)
void tile_sum_kernel(const uint8_t *__restrict__ level, long long N, long long Mdiv8, BitsTab bt,
                     long long *__restrict__ tilesum)
{
    const long long i0 = (long long)blockIdx.x * OF_TILE + (long long)threadIdx.x * OF_ITEMS;
    long long s = 0;
    for (int e = 0; e < OF_ITEMS; ++e)
        if (i0 + e < N) s += Mdiv8 * bt.bits[level[i0 + e] & 7];
    long long tot;
    block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) tilesum[blockIdx.x] = tot;
}

// one workgroup: exclusive scan of the tile sums in place
__global__ __launch_bounds__(OF_THREADS)
void scan_tiles_kernel(long long *tilesum, long long ntiles)
{
    long long carry = 0;
    for (long long t0 = 0; t0 < ntiles; t0 += OF_THREADS) {
        const long long t = t0 + threadIdx.x;
        const long long v = t < ntiles ? tilesum[t] : 0;
        long long tot;
        const long long ex = block_exclusive_scan(v, &tot);
        if (t < ntiles) tilesum[t] = carry + ex;
        carry += tot;
    }
}

__global__ __launch_bounds__(OF_THREADS)
void tile_scan_kernel(const uint8_t *__restrict__ level, long long N, long long Mdiv8, BitsTab bt,
                      const long long *__restrict__ tilebase, int64_t *__restrict__ byte_off)
{
    const long long i0 = (long long)blockIdx.x * OF_TILE + (long long)threadIdx.x * OF_ITEMS;
    long long v[OF_ITEMS], s = 0;
    for (int e = 0; e < OF_ITEMS; ++e) {
        v[e] = (i0 + e < N) ? Mdiv8 * bt.bits[level[i0 + e] & 7] : 0;
        s += v[e];
    }
    long long tot;
    long long acc = tilebase[blockIdx.x] + block_exclusive_scan(s, &tot);
    for (int e = 0; e < OF_ITEMS; ++e) {
        if (i0 + e < N) byte_off[i0 + e] = acc;
        acc += v[e];
        if (i0 + e == N - 1) byte_off[N] = acc;
    }
}

// ---- pack -------------------------------------------------------------------------
constexpr int PK_THREADS = 256;

template <int LPG>
__global__ __launch_bounds__(PK_THREADS)
void pack_kernel(const uint16_t *__restrict__ W, int64_t C, int m, int nbc, int64_t nrows_total,
                 const uint8_t *__restrict__ level, const int64_t *__restrict__ byte_off,
                 int64_t block_base, uint8_t *__restrict__ codes, float *__restrict__ scale,
                 float *__restrict__ zero, GridConsts gc)
{
    constexpr int GPW = PK_THREADS / LPG;            // block rows per workgroup
    __shared__ __align__(16) uint8_t stage[PK_THREADS * 8];
    const int tid = threadIdx.x;
    const int g = tid / LPG, lig = tid % LPG;

    // global row id over (block, row in block): rows of one block are consecutive
    int64_t rid = (int64_t)blockIdx.x * GPW + g;
    const bool valid = rid < nrows_total;
    if (!valid) rid = nrows_total - 1;
    const int64_t blk = rid / m;
    const int r = (int)(rid - blk * m);
    const int64_t I = blk / nbc, J = blk - I * nbc;
    const int64_t gb = block_base + blk;
    const int lv = level[gb];
    int c = gc.bits[0];
    float qf = gc.qmaxf[0], th = gc.thr[0];
#pragma unroll
    for (int cc = 1; cc < 8; ++cc)
        if (lv == cc) { c = gc.bits[cc]; qf = gc.qmaxf[cc]; th = gc.thr[cc]; }

    const int64_t off = (I * m + r) * C + J * (LPG * 8) + lig * 8;
    const uint4 wp = *reinterpret_cast<const uint4 *>(W + off);
    float w[8];
    unpack8(wp, w);
    float mn = fminf(fminf(fminf(w[0], w[1]), fminf(w[2], w[3])), fminf(fminf(w[4], w[5]), fminf(w[6], w[7])));
    float mx = fmaxf(fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])), fmaxf(fmaxf(w[4], w[5]), fmaxf(w[6], w[7])));
    mn = group_allreduce<LPG>(mn, OpMin{});
    mx = group_allreduce<LPG>(mx, OpMax{});
    const float R = mx - mn;
    float inv = qf / R, scl = R / qf;
    if (R < th) { inv = 0.0f; scl = 0.0f; }

    unsigned long long word = 0;
    const unsigned int qmax = (unsigned int)qf;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float t = rintf((w[e] - mn) * inv);
        unsigned int q = (unsigned int)(int)t;
        q = q > qmax ? qmax : q;
        word |= (unsigned long long)q << (e * c);
    }
    // each group has a fixed slot of LPG*8 bytes; the row's LPG*c bytes sit at its start
    uint8_t *mine = stage + (size_t)g * LPG * 8 + (size_t)lig * c;
    for (int t = 0; t < c; ++t) mine[t] = (uint8_t)(word >> (8 * t));
    __syncthreads();
    if (valid) {
        const int row_bytes = LPG * c;
        uint8_t *dst = codes + byte_off[gb] + (int64_t)r * row_bytes;
        const uint8_t *src = stage + (size_t)g * LPG * 8;
        if ((row_bytes & 3) == 0) {
            for (int d = lig; d < row_bytes / 4; d += LPG)
                reinterpret_cast<uint32_t *>(dst)[d] = reinterpret_cast<const uint32_t *>(src)[d];
        } else {
            for (int d = lig; d < row_bytes; d += LPG) dst[d] = src[d];
        }
        if (lig == 0) {
            scale[gb * m + r] = scl;
            zero[gb * m + r] = mn + 0.0f;
        }
    }
}

template <int LPG>
static int launch_pack_l(sbits_ctx *ctx, const uint16_t *W, int64_t C, int m, int nbc, int64_t nblocks,
                         const uint8_t *level, const int64_t *byte_off, int64_t block_base,
                         uint8_t *codes, float *scale, float *zero, const GridConsts &gc)
{
    constexpr int GPW = PK_THREADS / LPG;
    const int64_t nrows = nblocks * m;
    const int64_t nwg = (nrows + GPW - 1) / GPW;
    if (nwg > 0x7fffffff) return SBITS_ERR_BAD_SHAPE;
    hipLaunchKernelGGL((pack_kernel<LPG>), dim3((unsigned)nwg), dim3(PK_THREADS), 0, ctx->stream,
                       W, C, m, nbc, nrows, level, byte_off, block_base, codes, scale, zero, gc);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

}  // namespace sbits

using namespace sbits;

size_t sbits_offsets_ws_bytes(int64_t N)
{
    const int64_t ntiles = (N + OF_TILE - 1) / OF_TILE;
    return sbits_align_up((size_t)ntiles * 8, 256);
}

int sbits_launch_offsets(sbits_ctx *ctx, const uint8_t *level, int64_t N, int m, int n,
                         const int32_t *bits, int K, int64_t *byte_off, void *ws)
{
    BitsTab bt;
    for (int c = 0; c < 8; ++c) bt.bits[c] = c < K ? bits[c] : bits[K - 1];
    const long long Mdiv8 = (long long)m * n / 8;
    const int64_t ntiles = (N + OF_TILE - 1) / OF_TILE;
    long long *tiles = static_cast<long long *>(ws);
    hipLaunchKernelGGL(tile_sum_kernel, dim3((unsigned)ntiles), dim3(OF_THREADS), 0, ctx->stream,
                       level, (long long)N, Mdiv8, bt, tiles);
    hipLaunchKernelGGL(scan_tiles_kernel, dim3(1), dim3(OF_THREADS), 0, ctx->stream, tiles, (long long)ntiles);
    hipLaunchKernelGGL(tile_scan_kernel, dim3((unsigned)ntiles), dim3(OF_THREADS), 0, ctx->stream,
                       level, (long long)N, Mdiv8, bt, tiles, byte_off);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

int sbits_launch_pack(sbits_ctx *ctx, const void *Wp, int64_t R, int64_t C, int m, int n,
                      const int32_t *bits, int K, const uint8_t *level, const int64_t *byte_off,
                      int64_t block_base, uint8_t *codes, float *scale, float *zero)
{
    GridConsts gc;
    sbits_fill_grid_consts(bits, K, &gc);
    const int nbc = (int)(C / n);
    const int64_t nblocks = (R / m) * (C / n);
    const uint16_t *W = static_cast<const uint16_t *>(Wp);
    switch (n / 8) {
    case 1:  return launch_pack_l<1>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    case 2:  return launch_pack_l<2>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    case 4:  return launch_pack_l<4>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    case 8:  return launch_pack_l<8>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    case 16: return launch_pack_l<16>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    case 32: return launch_pack_l<32>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    case 64: return launch_pack_l<64>(ctx, W, C, m, nbc, nblocks, level, byte_off, block_base, codes, scale, zero, gc);
    }
    return SBITS_ERR_BAD_SHAPE;
}
