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
#include <string.h>

#include <mutex>

#include "pack_core.hpp"
#include "sbits_device.hpp"
#include "sbits_internal.hpp"

void sbits_fill_grid_consts(const int32_t *bits, int K, sbits::GridConsts *gc);

namespace sbits {

// ---- offsets --------------------------------------------------------------------
constexpr int OF_THREADS = 256;
constexpr int OF_ITEMS = 8;
constexpr int OF_TILE = OF_THREADS * OF_ITEMS;

struct BitsTab { int bits[MAX_CAND]; };
// (a level beyond the table, which no valid input holds, reads its last entry)
__device__ __forceinline__ int tab_bits(const BitsTab &bt, int lv) { return bt.bits[lv < MAX_CAND ? lv : MAX_CAND - 1]; }

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
        if (i0 + e < N) s += Mdiv8 * tab_bits(bt, level[i0 + e]);
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
        v[e] = (i0 + e < N) ? Mdiv8 * tab_bits(bt, level[i0 + e]) : 0;
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

// Geometry as in the cost kernel: the GW = 64/LPG lane groups of a wave sit on BX adjacent
// blocks of one block row (contiguous reads), the four waves (and the remaining OW groups of a
// wave) take different octets.  A workgroup is one step of one unit; each lane group packs one
// octet (8 rows) of one block, staged in LDS and written out as one contiguous run.
template <int LPG>
struct PackGeom {
    static constexpr int GW = 64 / LPG;
    static constexpr int BX = GW < 8 ? GW : 8;
    static constexpr int OW = GW / BX;
    static constexpr int OS = 4 * OW;
    static int blocks_per_unit(int m) { const int opb = m / 8; return opb >= OS ? BX : BX * (OS / opb); }
    static int steps(int m) { const int opb = m / 8; return opb >= OS ? opb / OS : 1; }
};

template <int LPG>
__global__ __launch_bounds__(PK_THREADS)
void pack_kernel(const MatDesc *__restrict__ descs, MatDesc one, const int *__restrict__ wg_start, int n_mats,
                 const uint16_t *__restrict__ W, int m, const uint8_t *__restrict__ level,
                 const int64_t *__restrict__ byte_off, uint8_t *__restrict__ codes, float *__restrict__ scale,
                 float *__restrict__ zero, GridConsts gc)
{
    using G = PackGeom<LPG>;
    constexpr int BX = G::BX, OS = G::OS, NG = PK_THREADS / LPG;
    __shared__ __align__(16) uint8_t stage[NG][8 * LPG * 8];     // per group: 8 rows x LPG*c bytes (c <= 8)

    const int mat = descs ? find_matrix(wg_start, n_mats, (int)blockIdx.x) : 0;
    const MatDesc d = descs ? descs[mat] : one;
    const int lid = (int)blockIdx.x - (descs ? wg_start[mat] : 0);
    const int opb = m >> 3;
    const int bpu = opb >= OS ? BX : BX * (OS / opb);
    const int steps = opb >= OS ? opb / OS : 1;
    const int upr = (d.nbc + bpu - 1) / bpu;
    const int I = lid / (upr * steps);
    const int rem = lid - I * (upr * steps);
    const int U = rem / steps, p = rem - U * steps;

    const int tid = threadIdx.x;
    const int lig = tid % LPG;
    const int g = tid / LPG;
    const int gw = (tid & 63) / LPG;
    const int slot = (tid >> 6) * G::OW + gw / BX;
    const int bl = (gw % BX) + (opb >= OS ? 0 : BX * (slot / opb));
    const int o = (opb >= OS ? slot : slot % opb) + p * OS;
    const int J = U * bpu + bl;
    const bool valid = J < d.nbc;
    const int Jc = valid ? J : d.nbc - 1;
    const int64_t gb = d.block_base + (int64_t)I * d.nbc + Jc;   // global block id
    const LevelConsts lk = level_consts(gc, level[gb]);
    const int c = lk.c;

    const uint16_t *__restrict__ src = W + d.elem_off + ((int64_t)I * m + (int64_t)o * 8) * d.cols +
                                       (int64_t)Jc * (LPG * 8) + lig * 8;
    uint4 raw[8];
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) raw[rr] = *reinterpret_cast<const uint4 *>(src + (int64_t)rr * d.cols);

    const int row_bytes = LPG * c;
    const bool odd = (lig & 1) != 0;                 // even lanes divide qmax/R, odd lanes R/qmax
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        float scl, mn;
        const unsigned long long word = quant_pack_row<LPG>(raw[rr], lk, odd, scl, mn);
        uint8_t *mine = &stage[g][rr * row_bytes + lig * c];
        store_code_bytes(mine, word, c);
        if (valid && lig == 0) {
            const int64_t ri = gb * m + o * 8 + rr;
            scale[ri] = scl;
            zero[ri] = mn + 0.0f;
        }
    }
    __syncthreads();
    if (valid) {
        // the octet's 8 rows are consecutive in the block's stream: one run of 8*row_bytes bytes
        uint8_t *dst = codes + byte_off[gb] + (int64_t)o * 8 * row_bytes;
        const int nbytes = 8 * row_bytes;            // a multiple of 8
        const uint32_t *s32 = reinterpret_cast<const uint32_t *>(&stage[g][0]);
        uint32_t *d32 = reinterpret_cast<uint32_t *>(dst);
        for (int k = lig; k < nbytes / 4; k += LPG) d32[k] = s32[k];
    }
}

struct PackLaunch {
    const MatDesc *descs;
    MatDesc one;
    const int *wg_start;
    int n_mats;
    int64_t total_wg;
    const uint16_t *W;
    int m;
    const uint8_t *level;
    const int64_t *byte_off;
    uint8_t *codes;
    float *scale, *zero;
    GridConsts gc;
};

template <int LPG>
static int launch_pack_l(sbits_ctx *ctx, const PackLaunch &a)
{
    if (a.total_wg > 0x7fffffff) return SBITS_ERR_BAD_SHAPE;
    if (a.total_wg == 0) return SBITS_OK;
    hipLaunchKernelGGL((pack_kernel<LPG>), dim3((unsigned)a.total_wg), dim3(PK_THREADS), 0, ctx->stream,
                       a.descs, a.one, a.wg_start, a.n_mats, a.W, a.m, a.level, a.byte_off, a.codes, a.scale,
                       a.zero, a.gc);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

static int launch_pack(int n, sbits_ctx *ctx, const PackLaunch &a)
{
    switch (n / 8) {
    case 1:  return launch_pack_l<1>(ctx, a);
    case 2:  return launch_pack_l<2>(ctx, a);
    case 4:  return launch_pack_l<4>(ctx, a);
    case 8:  return launch_pack_l<8>(ctx, a);
    case 16: return launch_pack_l<16>(ctx, a);
    case 32: return launch_pack_l<32>(ctx, a);
    case 64: return launch_pack_l<64>(ctx, a);
    }
    return SBITS_ERR_BAD_SHAPE;
}

static int64_t pack_wgs(int m, int n, int nbr, int nbc)
{
    int bpu = 1, st = 1;
    switch (n / 8) {
    case 1:  bpu = PackGeom<1>::blocks_per_unit(m);  st = PackGeom<1>::steps(m); break;
    case 2:  bpu = PackGeom<2>::blocks_per_unit(m);  st = PackGeom<2>::steps(m); break;
    case 4:  bpu = PackGeom<4>::blocks_per_unit(m);  st = PackGeom<4>::steps(m); break;
    case 8:  bpu = PackGeom<8>::blocks_per_unit(m);  st = PackGeom<8>::steps(m); break;
    case 16: bpu = PackGeom<16>::blocks_per_unit(m); st = PackGeom<16>::steps(m); break;
    case 32: bpu = PackGeom<32>::blocks_per_unit(m); st = PackGeom<32>::steps(m); break;
    case 64: bpu = PackGeom<64>::blocks_per_unit(m); st = PackGeom<64>::steps(m); break;
    }
    return (int64_t)nbr * ((nbc + bpu - 1) / bpu) * st;
}

}  // namespace sbits

using namespace sbits;

size_t sbits_offsets_ws_bytes(int64_t N)
{
    const int64_t ntiles = (N + OF_TILE - 1) / OF_TILE;
    return sbits_align_up((size_t)ntiles * 8, 256);
}

// ---- offsets without a caller workspace ---------------------------------------------
// The tile sums of the scan in a fixed device array instead of the caller's workspace, for
// callers that cannot allocate one.  Each GPU holds its own copy of the array at its own
// address; the address is looked up once per device (with that device current) and kept.
static __device__ __align__(256) long long scratch[SBITS_OFFSETS_STATIC_MAX_BLOCKS / OF_TILE];
static_assert(SBITS_OFFSETS_STATIC_MAX_BLOCKS % OF_TILE == 0, "whole tiles");

constexpr int OF_MAX_DEVICES = 64;
static std::mutex g_scratch_lock;
static long long *g_scratch_ptr[OF_MAX_DEVICES];     // device address of scratch[], per device ordinal

// Device address of this GPU's scratch array (ctx->device must be the current device).
int sbits_offsets_static_setup(sbits_ctx *ctx)
{
    if (ctx->device < 0 || ctx->device >= OF_MAX_DEVICES) return SBITS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[ctx->device]) {
        long long *ptr = nullptr;
        SBITS_HIP(ctx, hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) return SBITS_ERR_HIP;
        g_scratch_ptr[ctx->device] = ptr;
    }
    return SBITS_OK;
}

int sbits_launch_offsets_static(sbits_ctx *ctx, const uint8_t *level, int64_t N, int m, int n,
                                const int32_t *bits, int K, int64_t *byte_off)
{
    if (N > SBITS_OFFSETS_STATIC_MAX_BLOCKS) return SBITS_ERR_WORKSPACE;
    if (ctx->device < 0 || ctx->device >= OF_MAX_DEVICES) return SBITS_ERR_HIP;
    long long *ptr;
    {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        ptr = g_scratch_ptr[ctx->device];
    }
    if (!ptr) return SBITS_ERR_HIP;                  // sbits_create resolves it; never the array's host-side name
    // every tile sum in use is written by the first kernel before the others read it: nothing to clear
    return sbits_launch_offsets(ctx, level, N, m, n, bits, K, byte_off, ptr);
}

int sbits_launch_offsets(sbits_ctx *ctx, const uint8_t *level, int64_t N, int m, int n,
                         const int32_t *bits, int K, int64_t *byte_off, void *ws)
{
    BitsTab bt;
    for (int c = 0; c < sbits::MAX_CAND; ++c) bt.bits[c] = c < K ? bits[c] : bits[K - 1];
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
    PackLaunch a;
    memset(&a, 0, sizeof a);
    sbits_fill_grid_consts(bits, K, &a.gc);
    a.one.rows = R; a.one.cols = C; a.one.nbr = (int)(R / m); a.one.nbc = (int)(C / n);
    a.one.block_base = block_base;
    a.n_mats = 1;
    a.total_wg = pack_wgs(m, n, a.one.nbr, a.one.nbc);
    a.W = static_cast<const uint16_t *>(Wp);
    a.m = m;
    a.level = level; a.byte_off = byte_off; a.codes = codes; a.scale = scale; a.zero = zero;
    return launch_pack(n, ctx, a);
}

// all matrices of the plan in one launch; the descriptor table is already in the workspace head
int sbits_launch_pack_all(sbits_plan *plan, const void *w_re, const uint8_t *level, const int64_t *byte_off,
                          uint8_t *codes, float *scale, float *zero, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    PackLaunch a;
    memset(&a, 0, sizeof a);
    sbits_fill_grid_consts(plan->bits, plan->K, &a.gc);
    if (plan->pack_wg_start.empty()) {
        int64_t tot = 0;
        for (int i = 0; i < plan->n_mats; ++i) {
            plan->pack_wg_start.push_back((int)tot);
            tot += pack_wgs(plan->m, plan->n, plan->descs[i].nbr, plan->descs[i].nbc);
            if (tot > 0x7fffffff) { plan->pack_wg_start.clear(); return SBITS_ERR_BAD_SHAPE; }
        }
        plan->pack_wg_start.push_back((int)tot);
    }
    int *d_pre = sbits_prefix_ptr(plan, ws, 2);
    SBITS_HIP(ctx, hipMemcpyAsync(d_pre, plan->pack_wg_start.data(), plan->pack_wg_start.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    a.descs = sbits_desc_ptr(ws);
    a.wg_start = d_pre;
    a.n_mats = plan->n_mats;
    a.total_wg = plan->pack_wg_start.back();
    a.W = static_cast<const uint16_t *>(w_re);
    a.m = plan->m;
    a.level = level; a.byte_off = byte_off; a.codes = codes; a.scale = scale; a.zero = zero;
    return launch_pack(plan->n, ctx, a);
}
