// Reorder-gather fused with the block x bitwidth cost table: the original weights (bf16) and
// sensitivities (fp32) are read ONCE, permuted on the fly and scored; the reordered weights are
// written back only if the caller asks for them (the packing stage reads the originals too).  The
// reordered sensitivities never reach HBM.
//
// Operation: the same as gather followed by the cost table (paper Sec. 4.2 "bi-directional
// channel reordering" applied to W and S, then Sec. 5 "Implementation": per-block-row
// round-to-nearest grids for every candidate bitwidth), with the same fixed summation order,
// so the table equals the two-pass result bit for bit.
//
// Mapping.  A workgroup owns a run of octets (8 output rows each) of one matrix, all columns.
// Per step it has RS source rows (the rows row_perm names) brought into LDS by direct
// global-to-LDS loads (no registers in between), then every lane picks the 8 source columns of
// each of its CPL output chunks (chunk = 8 consecutive output columns; LPG adjacent lanes = one
// quantization group) out of LDS and scores them while the next step's rows are on their way.
// The levels of the octet's row tree are compile-time positions of an unrolled run of steps; at
// the end of an octet the group's lanes are reduced and the octet's partial sum goes to
// part[octet of the matrix][block column][candidate]; a second, tiny kernel runs the tree over the
// octets of each block.
#include <string.h>

#include <vector>

#include "cost_core.hpp"
#include "pack_core.hpp"
#include "surrogate_core.hpp"
#include "sbits_device.hpp"
#include "sbits_internal.hpp"

void sbits_fill_grid_consts(const int32_t *bits, int K, sbits::GridConsts *gc);

namespace sbits {

constexpr int FU_OPU = 16;                          // octets per workgroup at most (128 output rows); fewer for small classes
constexpr int FU_MAX_COLS = 16384;                  // widest row the cost kernel stages (2048 chunks: bf16 + fp32 row in LDS)
constexpr int FU_PACK_MAX_COLS = 32768;             // widest row the packing kernel stages (bf16 row only)

__device__ __forceinline__ int funi(int v) { return __builtin_amdgcn_readfirstlane(v); }

typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef __attribute__((address_space(3))) float lds_f32;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load in flight, which would expose the latency of the rows being prefetched into registers.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- rows into LDS without passing through registers -------------------------------------
// A wave-wide direct load (16 bytes per lane) writes one contiguous KiB of LDS, "a piece".  The
// RS source rows of a step are laid out piece by piece with the rows interleaved:
//   weights        piece p (columns 512p ..) of row r at  Wb + (p * RS + r) * 1024
//   sensitivities  piece p (columns 256p ..) of row r at  Sb + (p * RS + r) * 1024,  Sb = Wb + nW * RS * 1024
// so one address register per element serves every row of the step (row r = offset r * 1024 of the
// LDS instruction).  The loads carry the non-temporal hint: without it the same loop streams 12 %
// slower.  Lanes past a row's end repeat its last 16 bytes (into the padding of the last piece).
__device__ __forceinline__ void load_row_pieces(const char *wrow, const char *srow, int nW, int nS, uint32_t wbytes,
                                                uint32_t sbytes, uint32_t Wb, uint32_t Sb, int RSr, int rs, int wave,
                                                int nwv, int lane, bool do_w = true, bool do_s = true)
{
    const uint32_t l16 = (uint32_t)lane * 16u;
    for (int p = wave; do_w && p < nW; p += nwv) {
        const uint32_t off = min((uint32_t)p * 1024u + l16, wbytes - 16u);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wrow + off),
                                         (__attribute__((address_space(3))) void *)(Wb + (uint32_t)(p * RSr + rs) * 1024u),
                                         16, 0, 2);
    }
    for (int p = wave; do_s && p < nS; p += nwv) {
        const uint32_t off = min((uint32_t)p * 1024u + l16, sbytes - 16u);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(srow + off),
                                         (__attribute__((address_space(3))) void *)(Sb + (uint32_t)(p * RSr + rs) * 1024u),
                                         16, 0, 2);
    }
}

// bytes of LDS a step needs: rs rows of cols bf16 weights and (with_s) fp32 sensitivities, in whole pieces
static inline size_t staged_step_bytes(int64_t cols, int rs, bool with_s)
{
    const size_t nW = (size_t)(2 * cols + 1023) / 1024, nS = with_s ? (size_t)(4 * cols + 1023) / 1024 : 0;
    return (nW + nS) * (size_t)rs * 1024;
}

// One element out of the staged rows: the weight (bf16) is loaded into the upper half of a register
// (d16_hi).  On a GPU whose memories run with error correction (the target id says "sramecc+"; every
// MI355X does) such a load writes the whole register, zeros below: the register then holds the weight
// as a float, no conversion instruction needed.  (Without error correction the lower half would keep
// its old contents: the library refuses the one-pass route on such a device.)  The compiler does not
// see these loads' completion: lds_gather_wait() below stands between them and the first use.
template <int OFF>
__device__ __forceinline__ void lds_w_hi(float &w, uint32_t addr)
{
    asm volatile("ds_read_u16_d16_hi %0, %1 offset:%2" : "=v"(w) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_s(float &s, uint32_t addr)
{
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(s) : "v"(addr), "n"(OFF) : "memory");
}
__device__ __forceinline__ void lds_gather_wait(float (&w)[8])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7])
                 :: "memory");
}
__device__ __forceinline__ void lds_gather_wait(float (&w)[8], float (&s)[8])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7]),
                   "+v"(s[0]), "+v"(s[1]), "+v"(s[2]), "+v"(s[3]), "+v"(s[4]), "+v"(s[5]), "+v"(s[6]), "+v"(s[7])
                 :: "memory");
}

// Launched with T = the smallest multiple of 64 threads whose CPL chunks per lane cover a row
// (T <= TMAX), so that rows whose chunk count is no power of two leave no lanes idle.
// SUR = false: the block x bitwidth cost table (K candidates per block; with Z0 the first of them is
//              "0 bits", the pruned block, and gc holds the other K - 1 grids).
// SUR = true : the dynamic-sensitivity surrogates (K = 2 sums per block, at the block's current
//              level[]; the "sensitivity" input is the gradient; gc holds every candidate).
// Steps: RS rows each.  Per step: wait for the rows (this wave's loads, then everybody's: barrier),
// pick the lane's elements out of LDS, barrier (the buffer is free), request the next step's rows,
// score.  U = 8 / RS (RS = 2) or 2 (RS = 1) steps are unrolled so that the rows' positions in the
// octet's adjacent-pair tree are compile-time constants.
// Who talks to global memory: a wave that waits for its row loads (vmcnt 0) would also wait for any
// store it has issued, and a store's acknowledgement under this read load takes far longer than a
// load (the octet sums, 16 bytes per block, cost 12 % of the kernel's time that way).  So all waves
// but the last request rows and never store; the octet sums go through a small LDS table and the
// last wave, which requests nothing and never waits for vector memory, writes them out one step later.
// (A workgroup of a single wave does both.)
// SLATE (one row per step, cost table only): the sensitivities are read out of LDS while the first half
// of the arithmetic runs.  Order of a step: weights out of LDS, barrier, request the next row's weights;
// sensitivities requested from LDS (ordinary loads: the compiler places the wait at their first use),
// minimum / range / divisions / x meanwhile; barrier, request the next row's sensitivities; candidates.
// With one workgroup per CU (rows of 8192 elements and more) nobody else would fill the time the LDS
// needs for the gather.
// WPIPE (a refinement of SLATE; the parameter is the distance of the buffers in bytes, 0 = off): two buffers for
// the row of weights, a fixed distance apart (an immediate offset of the LDS reads; at least a row of weights).  The weights of row r + 1 are in LDS a step early, and a lane picks its elements of them out of
// LDS while it runs the second half of row r's arithmetic: no phase of a step is LDS reads alone, and a step
// has two barriers instead of three.
template <int LPG, int K, int CPL, int RS, int TMAX, int MINW, bool SUR, bool Z0, bool SLATE = false, int WPIPE = 0>
__global__ __launch_bounds__(TMAX, MINW)
void gather_cost_kernel(const MatDesc *__restrict__ descs, const int *__restrict__ members,
                        const int *__restrict__ wg_start, int n_members,
                        const int32_t *__restrict__ row_perm, const int32_t *__restrict__ col_perm, int m,
                        uint16_t *__restrict__ w_re_all, float *__restrict__ part, GridConsts gc,
                        const uint8_t *__restrict__ level, int kstride, int koff, int opu)
{
    // kstride, koff: the K sums of an octet go to part[..][koff .. koff + K) of kstride values (a launch
    // may cover a subset of the candidates)
    static_assert(!SUR || (K == 2 && !Z0), "two sums per block");
    static_assert(RS == 1 || RS == 2, "rows per step");
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int rowsrc[FU_OPU * 8];
    constexpr int NIT = RS * CPL;                    // rows x chunks scored per step
    using DP = DivPlan<LPG, K - Z0>;
    constexpr int NG = NIT > 2 ? 2 : NIT;            // items scored together
    constexpr int NI = SUR ? NG : (DP::RP < NG ? DP::RP : NG);   // of which NI share a round of divisions
    constexpr int U = RS == 2 ? 4 : 2;               // steps unrolled: B = U * RS rows with static tree positions
    constexpr int B = U * RS;
    constexpr bool SDER = RS == 1 && CPL >= 2;       // sensitivity address derived from the weight's (saves registers)
    static_assert(NIT % NG == 0 && NG % NI == 0, "step shape");
    static_assert(!SLATE || (RS == 1 && !SUR && SDER && NIT == NG), "late sensitivities: one row, one group of items");
    static_assert(!WPIPE || SLATE, "the weights' pipeline is a form of the slate step");
    constexpr uint32_t WBUF = (uint32_t)WPIPE;       // distance of the two weight buffers

    const int tid = (int)threadIdx.x;
    const int T = (int)blockDim.x;                   // a multiple of 64, at most TMAX
    const int lane = tid & 63, wave = funi(tid >> 6), nwv = T >> 6;
    const int lig = tid % LPG;
    const int mem = funi(find_matrix(wg_start, n_members, (int)blockIdx.x));
    const MatDesc &d = descs[funi(members[mem])];
    const int R = funi((int)d.rows), C = funi((int)d.cols) & ~7;   // (a multiple of the block width anyway)
    const int nbc = funi(d.nbc);
    const int opb = m >> 3;
    const int oct0 = ((int)blockIdx.x - funi(wg_start[mem])) * opu;
    const int noct = min(opu, (R >> 3) - oct0);
    const int32_t *__restrict__ rp = row_perm + d.row_off;
    const int32_t *__restrict__ cp = col_perm + d.col_off;
    const char *const Wg = reinterpret_cast<const char *>(d.w);
    const char *const Sg = reinterpret_cast<const char *>(d.s);
    const int64_t pitch_w = d.ld_w * 2, pitch_s = d.ld_s * 4;

    const uint32_t wbytes = 2u * (uint32_t)C, sbytes = 4u * (uint32_t)C;
    const int nW = (int)((wbytes + 1023u) >> 10), nS = (int)((sbytes + 1023u) >> 10);
    const uint32_t Wb = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint32_t Sb = WPIPE ? Wb + 2u * WBUF : Wb + (uint32_t)(nW * RS) * 1024u;
    float *const otab = reinterpret_cast<float *>(smem + (WPIPE ? (size_t)2 * WBUF + (size_t)nS * 1024
                                                                : (size_t)(nW + nS) * RS * 1024));   // [nbc][K] octet sums
    const int nld = nwv > 1 ? nwv - 1 : 1;           // waves that request rows
    const bool loader = wave < nld, storer = wave == nwv - 1;

    DP dp;
    dp.init(gc, lig);

    // source rows of the run (a permutation never trips the clamp; it keeps a bad one in bounds)
    for (int i = tid; i < noct * 8; i += T) {
        int sr = rp[oct0 * 8 + i];
        rowsrc[i] = sr < 0 ? 0 : (sr >= R ? R - 1 : sr);
    }

    // LDS addresses of the source columns of this lane's chunks (fixed for the whole run), row 0 of a step
    const int nchunk = C >> 3;
    uint32_t aw[CPL][8], as[SDER ? 1 : CPL][SDER ? 1 : 8];
    bool valid[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int chunk = tid + T * c;
        valid[c] = chunk < nchunk;
        const int cb = valid[c] ? chunk * 8 : 0;
        const int4 a = *reinterpret_cast<const int4 *>(cp + cb);
        const int4 b = *reinterpret_cast<const int4 *>(cp + cb + 4);
        const int t[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t sc = (uint32_t)(t[e] < 0 ? 0 : (t[e] >= C ? C - 1 : t[e]));
            aw[c][e] = Wb + (((sc >> 9) * (uint32_t)RS) << 10) + ((sc & 511u) << 1);
            if constexpr (!SDER) as[c][e] = Sb + (((sc >> 8) * (uint32_t)RS) << 10) + ((sc & 255u) << 2);
        }
    }
    const uint32_t sder = Sb - 2u * Wb;              // SDER: sensitivity address = 2 * weight address + sder
    __syncthreads();

    const int nrows = noct * 8, nrows_m1 = nrows - 1;
    // the source rows of the step that starts at `row` (read from LDS before any direct load or gather
    // read is in flight: the wait for them would otherwise wait for those as well)
    struct Rows { int sr[RS]; };
    auto source_rows = [&](int row) {
        Rows r;
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            int v = rowsrc[min(row + rs, nrows_m1)];
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v));           // here, not behind the gather reads issued later
            r.sr[rs] = funi(v);
        }
        return r;
    };
    auto request = [&](const Rows &r, bool do_w = true, bool do_s = true, uint32_t wbuf = 0u) {
        if (!loader) return;
#pragma unroll
        for (int rs = 0; rs < RS; ++rs)
            load_row_pieces(Wg + (int64_t)r.sr[rs] * pitch_w, Sg + (int64_t)r.sr[rs] * pitch_s, nW, nS, wbytes, sbytes,
                            Wb + wbuf, Sb, RS, rs, wave, nld, lane, do_w, do_s);
    };
    // the last wave writes the octet sums of octet `og` (in otab since the previous barrier) to part[]
    int pend_og = -1;
    auto flush = [&]() {
        if (pend_og < 0) return;
        if (storer) {
            // part: per matrix [octet of the matrix][block column][candidate], so that an octet's sums are one
            // contiguous run of whole cache lines (short writes scattered over many lines cost the read stream
            // far more than their bytes)
            float *row = part + ((d.block_base * opb + (int64_t)pend_og * nbc) * kstride + koff);
            for (int J = lane; J < nbc; J += 64) {
#pragma unroll
                for (int k = 0; k < K; ++k) row[J * kstride + k] = otab[J * K + k];
            }
        }
        pend_og = -1;
    };

    float t2[CPL][K], t3[CPL][K];                    // upper levels of the octet's row tree (B < 8 only)
    uint16_t *const wout = w_re_all + d.elem_off;
    LevelConsts lk[SUR ? CPL : 1];                   // SUR: the current grid of each chunk's block
    int curI = -1;

    // a lane's 8 reordered weights of output row orow, chunk c, as bf16 (the optional W' output)
    auto store_reordered = [&](const float (&w)[8], int orow, int c) {
        u32x4_t sv;
        sv.x = (__float_as_uint(w[0]) >> 16) | __float_as_uint(w[1]);
        sv.y = (__float_as_uint(w[2]) >> 16) | __float_as_uint(w[3]);
        sv.z = (__float_as_uint(w[4]) >> 16) | __float_as_uint(w[5]);
        sv.w = (__float_as_uint(w[6]) >> 16) | __float_as_uint(w[7]);
        __builtin_nontemporal_store(sv, (__attribute__((address_space(1))) u32x4_t *)(
                                            wout + (int64_t)orow * C + (int64_t)(tid + T * c) * 8));
    };

    // SLATE: one step (one row) for a wave that owns NV chunks per lane: NIT, or 1 for the last waves of a
    // workgroup whose second chunks lie past the row's end (they then skip that chunk's reads and arithmetic
    // instead of running them on nothing: with rows of 1792 chunks on 16 waves every SIMD gets 7 chunk-waves)
    constexpr bool SOLO_OK = SLATE && CPL == 2;
    const bool solo = SOLO_OK && wave * 64 + T >= nchunk;
    auto slate_step = [&](auto iu, auto inv, int row, const Rows &next, float (&t1)[CPL][K], float (&s2)[CPL][K],
                          float (&s3)[CPL][K], float (&last)[CPL][K]) {
        constexpr int u = decltype(iu)::value, NV = decltype(inv)::value;
        constexpr int NIv = DP::RP < NV ? DP::RP : NV;               // items per round of divisions
        float wv[NV][8], gs[NV][8];
        static_for<0, NV>([&](auto iit) {
            constexpr int it = decltype(iit)::value;
#pragma unroll
            for (int e = 0; e < 8; ++e) lds_w_hi<0>(wv[it][e], aw[it][e]);
        });
        static_for<0, NV>([&](auto iit) { lds_gather_wait(wv[decltype(iit)::value]); });
        asm volatile("s_barrier" ::: "memory");                      // everybody has its weights: that buffer is free
#pragma unroll
        for (int it = 0; it < NV; ++it)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t a;
                asm("v_lshl_add_u32 %0, %1, 1, %2" : "=v"(a) : "v"(aw[it][e]), "s"(sder));
                gs[it][e] = *(const lds_f32 *)a;
            }
        if (row + RS < nrows) request(next, true, false);
        __builtin_amdgcn_sched_barrier(0);
        if (w_re_all) {
#pragma unroll
            for (int it = 0; it < NV; ++it)
                if (valid[it]) store_reordered(wv[it], oct0 * 8 + row, it);
        }
        // first halves of all rounds, then the sensitivities' barrier
        float xs[NV][8], vals[NV / NIv][DP::NS];
#pragma unroll
        for (int i0 = 0; i0 < NV; i0 += NIv) {
            float w[NIv][8], x[NIv][8];
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) w[j][e] = wv[i0 + j][e];
            quant_cost_prep<LPG, K, NIv, Z0>(w, dp, x, vals[i0 / NIv]);
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) xs[i0 + j][e] = x[j][e];
        }
        // (the first halves' results are operands so that their arithmetic stays above the barrier)
#pragma unroll
        for (int r = 0; r < NV / NIv; ++r)
#pragma unroll
            for (int t = 0; t < DP::NS; ++t) asm volatile("" : "+v"(vals[r][t]));
#pragma unroll
        for (int it = 0; it < NV; ++it)
            asm volatile("" : "+v"(xs[it][0]), "+v"(xs[it][1]), "+v"(xs[it][2]), "+v"(xs[it][3]),
                              "+v"(xs[it][4]), "+v"(xs[it][5]), "+v"(xs[it][6]), "+v"(xs[it][7]));
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // everybody has its sensitivities
        if (row + RS < nrows) request(next, false, true);
#pragma unroll
        for (int i0 = 0; i0 < NV; i0 += NIv) {
            float w[NIv][8], x[NIv][8], sv[NIv][8], out[NIv][K];
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) { w[j][e] = wv[i0 + j][e]; x[j][e] = xs[i0 + j][e]; sv[j][e] = gs[i0 + j][e]; }
            quant_cost_finish<LPG, K, NIv, Z0, true>(w, x, vals[i0 / NIv], sv, out);
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int k = 0; k < K; ++k) asm volatile("" : "+v"(out[j][k]));     // (see the note in the other path)
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int k = 0; k < K; ++k)
                    last[i0 + j][k] = octet_tree_push(out[j][k], u, t1[i0 + j][k], s2[i0 + j][k], s3[i0 + j][k]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // WPIPE: the lane's weights of the current row (parity u of the unrolled pair) and of the next one
    float wvp[WPIPE ? 2 : 1][NIT][8];
    auto wpipe_step = [&](auto iu, auto inv, int row, const Rows &next, const Rows &next2, float (&t1)[CPL][K],
                          float (&s2)[CPL][K], float (&s3)[CPL][K], float (&last)[CPL][K]) {
        constexpr int u = decltype(iu)::value, NV = decltype(inv)::value;
        constexpr int NIv = DP::RP < NV ? DP::RP : NV;               // items per round of divisions
        constexpr int un = WPIPE ? (u ^ 1) : 0;
        float gs[NV][8];
        // the row's sensitivities out of LDS while the first half of the arithmetic runs
#pragma unroll
        for (int it = 0; it < NV; ++it)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t a;
                asm("v_lshl_add_u32 %0, %1, 1, %2" : "=v"(a) : "v"(aw[it][e]), "s"(sder));
                lds_s<0>(gs[it][e], a);
            }
        if (w_re_all) {
#pragma unroll
            for (int it = 0; it < NV; ++it)
                if (valid[it]) store_reordered(wvp[u & (WPIPE ? 1 : 0)][it], oct0 * 8 + row, it);
        }
        float xs[NV][8], vals[NV / NIv][DP::NS];
#pragma unroll
        for (int i0 = 0; i0 < NV; i0 += NIv) {
            float w[NIv][8], x[NIv][8];
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) w[j][e] = wvp[u & (WPIPE ? 1 : 0)][i0 + j][e];
            quant_cost_prep<LPG, K, NIv, Z0>(w, dp, x, vals[i0 / NIv]);
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) xs[i0 + j][e] = x[j][e];
        }
#pragma unroll
        for (int r = 0; r < NV / NIv; ++r)
#pragma unroll
            for (int t = 0; t < DP::NS; ++t) asm volatile("" : "+v"(vals[r][t]));
#pragma unroll
        for (int it = 0; it < NV; ++it)
            asm volatile("" : "+v"(xs[it][0]), "+v"(xs[it][1]), "+v"(xs[it][2]), "+v"(xs[it][3]),
                              "+v"(xs[it][4]), "+v"(xs[it][5]), "+v"(xs[it][6]), "+v"(xs[it][7]));
        static_for<0, NV>([&](auto iit) { lds_gather_wait(gs[decltype(iit)::value]); });
        asm volatile("s_barrier" ::: "memory");                      // everybody has its sensitivities: that buffer is free
        if (row + 2 < nrows) request(next2, true, false, (uint32_t)u * WBUF);   // weights of row r + 2 -> the buffer row r left
        if (row + 1 < nrows) request(next, false, true);                          // sensitivities of row r + 1
        if (row + 1 < nrows) {
            static_for<0, NV>([&](auto iit) {
                constexpr int it = decltype(iit)::value;
#pragma unroll
                for (int e = 0; e < 8; ++e) lds_w_hi<un * WBUF>(wvp[un][it][e], aw[it][e]);
            });
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i0 = 0; i0 < NV; i0 += NIv) {
            float w[NIv][8], x[NIv][8], sv[NIv][8], out[NIv][K];
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) { w[j][e] = wvp[u & (WPIPE ? 1 : 0)][i0 + j][e]; x[j][e] = xs[i0 + j][e]; sv[j][e] = gs[i0 + j][e]; }
            quant_cost_finish<LPG, K, NIv, Z0, true>(w, x, vals[i0 / NIv], sv, out);
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int k = 0; k < K; ++k) asm volatile("" : "+v"(out[j][k]));
#pragma unroll
            for (int j = 0; j < NIv; ++j)
#pragma unroll
                for (int k = 0; k < K; ++k)
                    last[i0 + j][k] = octet_tree_push(out[j][k], u, t1[i0 + j][k], s2[i0 + j][k], s3[i0 + j][k]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (row + 1 < nrows) static_for<0, NV>([&](auto iit) { lds_gather_wait(wvp[un][decltype(iit)::value]); });
    };

    request(source_rows(0));
    if constexpr (WPIPE) {
        request(source_rows(1), true, false, WBUF);                  // (nrows >= 8)
        if (loader) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        static_for<0, NIT>([&](auto iit) {
            constexpr int it = decltype(iit)::value;
#pragma unroll
            for (int e = 0; e < 8; ++e) lds_w_hi<0>(wvp[0][it][e], aw[it][e]);
        });
        static_for<0, NIT>([&](auto iit) { lds_gather_wait(wvp[0][decltype(iit)::value]); });
    }
    for (int row0 = 0; row0 < nrows; row0 += B) {
        float t1[CPL][K], s2[CPL][K], s3[CPL][K];    // static levels inside the unrolled rows
        float last[CPL][K];
        static_for<0, U>([&](auto iu) {
            constexpr int u = decltype(iu)::value;
            const int row = row0 + u * RS;           // first row of the step inside the run
            __builtin_amdgcn_sched_barrier(0);                       // (the previous step's arithmetic stays above)
            if (loader) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this wave's share of the step's rows
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");    // everybody's: the rows are in LDS
            flush();
            const Rows next = source_rows(row + RS);                 // (clamped past the end; not requested then)
            if constexpr (SUR) {
                const int Inow = (oct0 + (row >> 3)) / opb;          // block row of this step
                if (Inow != curI) {
                    curI = Inow;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        const int J = min((tid + T * c) / LPG, nbc - 1);
                        lk[c] = level_consts(gc, level[d.block_base + (int64_t)Inow * nbc + J]);
                    }
                }
            }
            if constexpr (WPIPE) {
                const Rows next2 = source_rows(row + 2);
                if (SOLO_OK && solo) wpipe_step(iu, std::integral_constant<int, 1>{}, row, next, next2, t1, s2, s3, last);
                else wpipe_step(iu, std::integral_constant<int, NIT>{}, row, next, next2, t1, s2, s3, last);
                return;
            }
            if constexpr (SLATE) {
                if (SOLO_OK && solo) slate_step(iu, std::integral_constant<int, 1>{}, row, next, t1, s2, s3, last);
                else slate_step(iu, std::integral_constant<int, NIT>{}, row, next, t1, s2, s3, last);
                return;
            }
            // items (item = rs * CPL + c): all LDS reads of the step
            float wv[NIT][8], gs[NIT][8];
            static_for<0, NIT>([&](auto iit) {
                constexpr int it = decltype(iit)::value;
                constexpr int rs = it / CPL, c = it % CPL;
#pragma unroll
                for (int e = 0; e < 8; ++e) lds_w_hi<rs * 1024>(wv[it][e], aw[c][e]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if constexpr (SDER) {
                        uint32_t a;
                        asm volatile("v_lshl_add_u32 %0, %1, 1, %2" : "=v"(a) : "v"(aw[c][e]), "s"(sder));
                        lds_s<rs * 1024>(gs[it][e], a);
                    } else {
                        lds_s<rs * 1024>(gs[it][e], as[c][e]);
                    }
                }
            });
            static_for<0, NIT>([&](auto iit) { lds_gather_wait(wv[decltype(iit)::value], gs[decltype(iit)::value]); });
            asm volatile("s_barrier" ::: "memory");                  // everybody has read: the buffer is free
            if (row + RS < nrows) request(next);
            __builtin_amdgcn_sched_barrier(0);

#pragma unroll
            for (int g0 = 0; g0 < NIT; g0 += NG) {
                if (w_re_all) {
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        const int rs = (g0 + g) / CPL, c = (g0 + g) % CPL;
                        if (valid[c]) store_reordered(wv[g0 + g], oct0 * 8 + row + rs, c);
                    }
                }
#pragma unroll
                for (int i0 = 0; i0 < NG; i0 += NI) {
                    float w[NI][8], s[NI][8], out[NI][K];
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int e = 0; e < 8; ++e) { w[j][e] = wv[g0 + i0 + j][e]; s[j][e] = gs[g0 + i0 + j][e]; }
                    if constexpr (SUR) {
                        LevelConsts lr[NI];
#pragma unroll
                        for (int j = 0; j < NI; ++j) lr[j] = lk[(g0 + i0 + j) % CPL];
                        surrogate_round<LPG, NI>(w, s, lr, lig, out);
                    } else {
                        quant_cost_round_f<LPG, K, NI, Z0, true>(w, s, dp, out);
                    }
                    // The sums are used by a later step's tree addition only: without an opaque use here the
                    // optimizer sinks the whole arithmetic below the next step's barriers and LDS reads
                    // (and has to keep copies of every input for it).
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int k = 0; k < K; ++k) asm volatile("" : "+v"(out[j][k]));
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        const int rs = (g0 + i0 + j) / CPL, c = (g0 + i0 + j) % CPL;
                        const int rr = u * RS + rs;                  // the row's place among the unrolled rows (compile time)
#pragma unroll
                        for (int k = 0; k < K; ++k) last[c][k] = octet_tree_push(out[j][k], rr, t1[c][k], s2[c][k], s3[c][k]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        });
        if constexpr (B < 8) {                       // the unrolled rows' sum enters the tree's upper levels
            static_assert(B == 2, "pairs of rows");
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                if (c > 0 && solo) continue;
#pragma unroll
                for (int k = 0; k < K; ++k)
                    last[c][k] = octet_tree_push_pair_rt(last[c][k], (row0 >> 1) & 3, t2[c][k], t3[c][k]);
            }
        }

        if (((row0 + B) & 7) == 0) {                 // an octet is complete: lanes of the group, then out
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                if (c > 0 && solo) continue;
                float v[K];
#pragma unroll
                for (int k = 0; k < K; ++k) v[k] = group_allreduce<LPG>(last[c][k], OpAdd{});
                if (lig == 0 && valid[c]) {
                    const int J = (tid + T * c) / LPG;
#pragma unroll
                    for (int k = 0; k < K; ++k) otab[J * K + k] = v[k];
                }
            }
            pend_og = oct0 + (row0 >> 3);            // written out after the next barrier
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    flush();
}

// adjacent-pair tree over n <= 8 values p[0], p[stride], ... (n a power of two)
__device__ __forceinline__ float tree_upto8(const float *__restrict__ p, int64_t stride, int n)
{
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = i < n ? p[i * stride] : 0.0f;
    if (n == 1) return v[0];
    if (n == 2) return v[0] + v[1];
    if (n == 4) return (v[0] + v[1]) + (v[2] + v[3]);
    return ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
}

// Where the octet sums of global block b start in part[] (layout per matrix: [octet][block column][sum], ks sums
// per entry) and the distance between consecutive octets of the block.  The matrix is found by bisection over the
// descriptors' first block ids.
__device__ __forceinline__ const float *block_partials(const float *__restrict__ part, const MatDesc *__restrict__ descs,
                                                       int n_mats, int64_t b, int opb, int ks, int64_t *stride)
{
    int lo = 0, hi = n_mats;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (descs[mid].block_base <= b) lo = mid; else hi = mid;
    }
    const int64_t base = descs[lo].block_base;
    const int nbc = descs[lo].nbc;
    const int64_t bl = b - base;
    const int64_t I = bl / nbc, J = bl - I * nbc;
    *stride = (int64_t)nbc * ks;
    return part + (base * opb + I * opb * nbc + J) * ks;
}

// cost[b][c] = adjacent-pair tree over the opb octet partials of block b (opb a power of two <= 128)
__global__ __launch_bounds__(256)
void octet_finish_kernel(const float *__restrict__ part, const MatDesc *__restrict__ descs, int n_mats, int64_t NK,
                         int K, int opb, float *__restrict__ cost)
{
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= NK) return;
    const int64_t b = q / K;
    const int c = (int)(q - b * K);
    int64_t so;                                      // distance between the block's consecutive octets
    const float *p = block_partials(part, descs, n_mats, b, opb, K, &so) + c;
    if (opb <= 8) {
        cost[q] = tree_upto8(p, so, opb);
        return;
    }
    float t1 = 0.0f, t2 = 0.0f, t3 = 0.0f, t4 = 0.0f, v = 0.0f;
    const int ng = opb >> 3;                         // 2 .. 16 groups of 8 octets
    for (int g = 0; g < ng; ++g) {
        v = tree_upto8(p + (int64_t)g * 8 * so, so, 8);
        if (g & 1) {
            v = t1 + v;
            if (g & 2) {
                v = t2 + v;
                if (g & 4) {
                    v = t3 + v;
                    if (g & 8) v = t4 + v;
                    else t4 = v;
                } else {
                    t3 = v;
                }
            } else {
                t2 = v;
            }
        } else {
            t1 = v;
        }
    }
    cost[q] = v;
}

// ================================================================ gather + pack
// The packing stage on the ORIGINAL weights: a workgroup owns a run of octets of one matrix,
// stages RS source rows per step in LDS like the kernel above (weights only), and every lane
// re-quantizes its chunks at the bitwidth chosen for their block.  The codes of a lane group's
// RS rows are consecutive in the block's stream: they are collected in a per-group LDS strip
// (written and read by lanes of one wave only) and leave as 32-bit words.
// T threads per workgroup; launch bounds ask for 4 waves per SIMD (two workgroups of 512 or one
// of 1024 per CU), which the kernel's ~120 registers allow.
template <int LPG, int CPL, int RS, int TMAX>
__global__ __launch_bounds__(TMAX, 4)
void gather_pack_kernel(const MatDesc *__restrict__ descs, const int *__restrict__ members,
                        const int *__restrict__ wg_start, int n_members,
                        const int32_t *__restrict__ row_perm, const int32_t *__restrict__ col_perm, int m,
                        const uint8_t *__restrict__ level, const int64_t *__restrict__ byte_off,
                        uint8_t *__restrict__ codes, float *__restrict__ scale, float *__restrict__ zero,
                        GridConsts gc, int cmax, int opu)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int rowsrc[FU_OPU * 8];
    constexpr int NIT = RS * CPL;
    static_assert(8 % RS == 0, "step shape");

    const int tid = (int)threadIdx.x;
    const int T = (int)blockDim.x;                   // a multiple of 64, at most TMAX
    const int lig = tid % LPG;
    const int mem = funi(find_matrix(wg_start, n_members, (int)blockIdx.x));
    const MatDesc &d = descs[funi(members[mem])];
    const int R = funi((int)d.rows), C = funi((int)d.cols) & ~7;
    const int nbc = funi(d.nbc);
    const int opb = m >> 3;
    const int oct0 = ((int)blockIdx.x - funi(wg_start[mem])) * opu;
    const int noct = min(opu, (R >> 3) - oct0);
    const int32_t *__restrict__ rp = row_perm + d.row_off;
    const int32_t *__restrict__ cp = col_perm + d.col_off;
    const char *const Wg = reinterpret_cast<const char *>(d.w);
    const int64_t pitch_w = d.ld_w * 2;
    const int64_t block_base = d.block_base;

    // LDS: weights [RS][C] bf16, then one strip of RS * LPG * cmax bytes per (lane group, chunk)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    // (+8: a lane's third word may lie past its row; it is zero there, but has to be addressable)
    const int strip = RS * LPG * cmax + 8;
    const uint32_t strips = lds0 + (uint32_t)RS * (uint32_t)C * 2u;
    for (int c = 0; c < CPL; ++c) {                  // every group zeroes its own strips
        const uint32_t s0 = strips + (uint32_t)((tid / LPG) + (T / LPG) * c) * (uint32_t)strip;
        for (int k = lig; k < strip / 4; k += LPG) *(lds_u32 *)(s0 + 4u * (uint32_t)k) = 0u;
    }

    for (int i = tid; i < noct * 8; i += T) {
        int sr = rp[oct0 * 8 + i];
        rowsrc[i] = sr < 0 ? 0 : (sr >= R ? R - 1 : sr);
    }
    const int nchunk = C >> 3;
    int ci[CPL][8];
    bool valid[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int chunk = tid + T * c;
        valid[c] = chunk < nchunk;
        const int cb = valid[c] ? chunk * 8 : 0;
        const int4 a = *reinterpret_cast<const int4 *>(cp + cb);
        const int4 b = *reinterpret_cast<const int4 *>(cp + cb + 4);
        const int t[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) ci[c][e] = 2 * (t[e] < 0 ? 0 : (t[e] >= C ? C - 1 : t[e]));
    }
    __syncthreads();

    uint32_t offw[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) offw[c] = (uint32_t)min(tid + T * c, nchunk - 1) * 16u;
    uint4 pw[RS][CPL];
    auto prefetch = [&](int row) {
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) {
            const int sr = funi(rowsrc[row + rs]);
            const char *wrow = Wg + (int64_t)sr * pitch_w;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const u32x4_t v = __builtin_nontemporal_load(
                    (const __attribute__((address_space(1))) u32x4_t *)(wrow + offw[c]));
                pw[rs][c] = make_uint4(v.x, v.y, v.z, v.w);
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int rs = 0; rs < RS; ++rs)
#pragma unroll
            for (int c = 0; c < CPL; ++c)
                *reinterpret_cast<uint4 *>(smem + (size_t)rs * C * 2 + offw[c]) = pw[rs][c];
    };

    // per chunk: the block it falls in (fixed column, block row changes every opb octets)
    int curI = -1;
    LevelConsts lk[CPL];
    int64_t gb[CPL];
    uint8_t *dst[CPL];
    const int nsteps = noct * (8 / RS);

    prefetch(0);
    for (int st = 0; st < nsteps; ++st) {
        stage();
        lds_barrier();
        if (st + 1 < nsteps) prefetch((st + 1) * RS);

        const int row = st * RS;
        const int og = oct0 + (row >> 3);
        const int I = og / opb;
        const int rib = (og - I * opb) * 8 + (row & 7);         // first row of the step inside its block
        if (I != curI) {
            curI = I;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int J = min((tid + T * c) / LPG, nbc - 1);
                gb[c] = block_base + (int64_t)I * nbc + J;
                lk[c] = level_consts(gc, level[gb[c]]);
                dst[c] = codes + byte_off[gb[c]];
            }
        }

        uint4 gw[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int rs = it / CPL, c = it % CPL;
            uint32_t wbase = lds0 + (uint32_t)rs * (uint32_t)C * 2u;
            asm volatile("" : "+s"(wbase));          // keeps the 8 sums below out of loop-invariant registers
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = *(const lds_u16 *)(wbase + (uint32_t)ci[c][e]);
            gw[it] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        }
        lds_barrier();                               // the rows may be overwritten from here on

#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const int cb = lk[c].c;
            const int row_bytes = LPG * cb;
            const uint32_t strip0 = strips + (uint32_t)((tid / LPG) + (T / LPG) * c) * (uint32_t)strip;
            uint4 raw[RS];
#pragma unroll
            for (int rs = 0; rs < RS; ++rs) raw[rs] = gw[rs * CPL + c];
            unsigned long long word[RS];
            float scl[RS], mn[RS];
            quant_pack_rows<LPG, RS>(raw, lk[c], lig, word, scl, mn);
#pragma unroll
            for (int rs = 0; rs < RS; ++rs)
                or_code_bytes(strip0 + (uint32_t)(rs * row_bytes), lig * cb, word[rs], cmax > 4);
            if (valid[c] && lig == 0) {
                // RS consecutive rows of one block: one vector store each (rib is a multiple of RS)
                const int64_t ri = gb[c] * m + rib;
                float zr[RS];
#pragma unroll
                for (int rs = 0; rs < RS; ++rs) zr[rs] = mn[rs] + 0.0f;
                if constexpr (RS == 4) {
                    *reinterpret_cast<float4 *>(scale + ri) = make_float4(scl[0], scl[1], scl[2], scl[3]);
                    *reinterpret_cast<float4 *>(zero + ri) = make_float4(zr[0], zr[1], zr[2], zr[3]);
                } else if constexpr (RS == 2) {
                    *reinterpret_cast<float2 *>(scale + ri) = make_float2(scl[0], scl[1]);
                    *reinterpret_cast<float2 *>(zero + ri) = make_float2(zr[0], zr[1]);
                } else {
#pragma unroll
                    for (int rs = 0; rs < RS; ++rs) { scale[ri + rs] = scl[rs]; zero[ri + rs] = zr[rs]; }
                }
            }
            // the strip is private to this lane group (one wave): LDS keeps a wave's operations in order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (valid[c]) {
                const int nwords = RS * row_bytes / 4;           // row_bytes is a multiple of 8
                uint32_t *d32 = reinterpret_cast<uint32_t *>(dst[c] + (int64_t)rib * row_bytes);
                for (int k = lig; k < nwords; k += LPG) {
                    lds_u32 *sp = (lds_u32 *)(strip0 + 4u * (uint32_t)k);
                    d32[k] = *sp;
                    *sp = 0u;                                    // zero again for the next step's ORs
                }
            } else {
                for (int k = lig; k < RS * row_bytes / 4; k += LPG) *(lds_u32 *)(strip0 + 4u * (uint32_t)k) = 0u;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// surrogates: s_up[b] = tree over the octets of sum 0, s_down[b] = 2^-bits * tree over those of sum 1
__global__ __launch_bounds__(256)
void surrogate_finish_kernel(const float *__restrict__ part, const MatDesc *__restrict__ descs, int n_mats, int64_t N,
                             int opb, const uint8_t *__restrict__ level, GridConsts gc, float *__restrict__ s_up,
                             float *__restrict__ s_down)
{
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= 2 * N) return;
    const int64_t b = q >> 1;
    const int which = (int)(q & 1);
    int64_t so;
    const float *p = block_partials(part, descs, n_mats, b, opb, 2, &so) + which;
    float v;
    if (opb <= 8) {
        v = tree_upto8(p, so, opb);
    } else {
        float t1 = 0.0f, t2 = 0.0f, t3 = 0.0f, t4 = 0.0f;
        v = 0.0f;
        const int ng = opb >> 3;
        for (int g = 0; g < ng; ++g) {
            v = tree_upto8(p + (int64_t)g * 8 * so, so, 8);
            if (g & 1) {
                v = t1 + v;
                if (g & 2) {
                    v = t2 + v;
                    if (g & 4) {
                        v = t3 + v;
                        if (g & 8) v = t4 + v;
                        else t4 = v;
                    } else {
                        t3 = v;
                    }
                } else {
                    t2 = v;
                }
            } else {
                t1 = v;
            }
        }
    }
    if (which == 0) {
        s_up[b] = v;
    } else {
        int bits = gc.bits[0];
#pragma unroll
        for (int cc = 1; cc < MAX_CAND; ++cc)
            if (level[b] == cc) bits = gc.bits[cc];
        s_down[b] = ldexpf(v, -bits);
    }
}

struct FusedLaunch {
    const MatDesc *descs;
    const int *members, *wg_start;
    int n_members, total_wg;
    const int32_t *row_perm, *col_perm;
    int m;
    uint16_t *w_re;
    float *part;
    GridConsts gc;
    int64_t cols;
    const uint8_t *level;     // surrogates only
    int kstride, koff;        // where the launch's sums go among the block's (see the kernel)
    int opu;                  // octets per workgroup of this class
};

// threads per workgroup: the chunks of a row spread over CPL per lane, rounded up to whole waves
static int fused_threads(int64_t cols, int cpl, int tmax)
{
    const int64_t need = ((cols / 8 + cpl - 1) / cpl + 63) / 64 * 64;
    return (int)(need < 64 ? 64 : (need > tmax ? tmax : need));
}

template <int LPG, int K, int CPL, int RS, int TMAX, int MINW, bool SUR, bool Z0, bool SLATE = false, int WPIPE = 0>
static int launch_fused_g(sbits_ctx *ctx, const FusedLaunch &a)
{
    int T = fused_threads(a.cols, CPL, TMAX);
    if (SLATE && T > 256) T = (T + 255) / 256 * 256 <= TMAX ? (T + 255) / 256 * 256 : T;   // whole rounds of the four SIMDs
    auto *fn = &gather_cost_kernel<LPG, K, CPL, RS, TMAX, MINW, SUR, Z0, SLATE, WPIPE>;
    SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 159 * 1024));
    const size_t lds = (WPIPE ? (size_t)2 * WPIPE + staged_step_bytes(a.cols, RS, true) - staged_step_bytes(a.cols, RS, false)
                              : staged_step_bytes(a.cols, RS, true)) +
                       (size_t)(a.cols / (LPG * 8)) * K * 4;                               // rows + octet sums
    hipLaunchKernelGGL(fn, dim3((unsigned)a.total_wg), dim3(T), lds, ctx->stream, a.descs, a.members,
                       a.wg_start, a.n_members, a.row_perm, a.col_perm, a.m, a.w_re, a.part, a.gc, a.level, a.kstride,
                       a.koff, a.opu);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

// Instances by row length (chunks of 8 columns) and candidate count:
//   up to 512 chunks : two rows per step; up to four candidates: two chunks per lane in workgroups of up
//                      to 256 threads (three workgroups = 12 waves per CU at up to 168 registers: three
//                      independent barrier groups hide each other's waits better than two of 8 waves);
//                      more candidates: one chunk per lane, up to 512 threads
//   up to 1024       : two chunks per lane, one row per step
//   up to 2048       : the same in workgroups of up to 1024 threads (one per CU: the row takes up to
//                      96 KB of LDS)
template <int LPG, int K, bool Z0>
static int launch_fused_k(sbits_ctx *ctx, const FusedLaunch &a)
{
    const int64_t chunks = a.cols / 8;
    constexpr int MINW = K <= 4 ? 4 : 2;             // waves per SIMD the register budget is set for
    if (chunks <= 512) {
        // (two chunks and two rows per lane where that fits 168 registers without spilling; else one chunk of one
        // row, 62 to 82 registers: three workgroups per CU; measured 2 to 6 % faster than two rows per step there)
        if constexpr (K <= 2 || (K <= 4 && !Z0 && LPG == 16)) return launch_fused_g<LPG, K, 2, 2, 256, 3, false, Z0>(ctx, a);
        // (... as long as it stays within the 80 registers that three workgroups of eight waves leave a lane)
        else if constexpr (LPG == 16 ? (K <= 7 || (K == 8 && !Z0)) : (K <= 5 || (K == 6 && !Z0)))
            return launch_fused_g<LPG, K, 1, 1, 512, 4, false, Z0>(ctx, a);
        else return launch_fused_g<LPG, K, 1, 2, 512, MINW, false, Z0>(ctx, a);
    }
    if (chunks <= 1024) return launch_fused_g<LPG, K, 2, 1, 512, MINW, false, Z0>(ctx, a);
    if (chunks <= 2048) {
        // seven or more candidates: two chunks' state does not fit the 128 registers of a 1024-thread workgroup
        // the slate form; with the weights pipelined where that fits the 128 registers (or nearly: 16 bytes of
        // scratch at five candidates still pay, 24 and more do not)
        if constexpr (LPG == 16 ? K <= 5 : (K <= 2 || (K == 3 && !Z0)))
            return launch_fused_g<LPG, K, 2, 1, 1024, 4, false, Z0, true, 32768>(ctx, a);
        else if constexpr (K <= 5 || (K == 6 && !(Z0 && LPG == 8))) return launch_fused_g<LPG, K, 2, 1, 1024, 4, false, Z0, true>(ctx, a);
        else return launch_fused_g<LPG, K, 2, 1, 1024, 4, false, Z0, false>(ctx, a);
    }
    return SBITS_ERR_BAD_SHAPE;
}

template <int LPG>
static int launch_surrogates_l(sbits_ctx *ctx, const FusedLaunch &a)
{
    const int64_t chunks = a.cols / 8;
    if (chunks <= 512) return launch_fused_g<LPG, 2, 1, 2, 512, 4, true, false>(ctx, a);
    if (chunks <= 1024) return launch_fused_g<LPG, 2, 2, 1, 512, 4, true, false>(ctx, a);
    if (chunks <= 2048) return launch_fused_g<LPG, 2, 2, 1, 1024, 4, true, false>(ctx, a);
    return SBITS_ERR_BAD_SHAPE;
}

// K: the candidates of this launch; z0: the first of them is 0 bits (then 2 <= K <= 9, else 1 <= K <= 8)
template <int LPG>
static int launch_fused_l(int K, bool z0, sbits_ctx *ctx, const FusedLaunch &a)
{
    if (z0) switch (K) {
    case 2: return launch_fused_k<LPG, 2, true>(ctx, a);
    case 3: return launch_fused_k<LPG, 3, true>(ctx, a);
    case 4: return launch_fused_k<LPG, 4, true>(ctx, a);
    case 5: return launch_fused_k<LPG, 5, true>(ctx, a);
    case 6: return launch_fused_k<LPG, 6, true>(ctx, a);
    case 7: return launch_fused_k<LPG, 7, true>(ctx, a);
    case 8: return launch_fused_k<LPG, 8, true>(ctx, a);
    case 9: return launch_fused_k<LPG, 9, true>(ctx, a);
    }
    else switch (K) {
    case 1: return launch_fused_k<LPG, 1, false>(ctx, a);
    case 2: return launch_fused_k<LPG, 2, false>(ctx, a);
    case 3: return launch_fused_k<LPG, 3, false>(ctx, a);
    case 4: return launch_fused_k<LPG, 4, false>(ctx, a);
    case 5: return launch_fused_k<LPG, 5, false>(ctx, a);
    case 6: return launch_fused_k<LPG, 6, false>(ctx, a);
    case 7: return launch_fused_k<LPG, 7, false>(ctx, a);
    case 8: return launch_fused_k<LPG, 8, false>(ctx, a);
    }
    return SBITS_ERR_BAD_BITWIDTHS;
}

struct FusedPackLaunch {
    const MatDesc *descs;
    const int *members, *wg_start;
    int n_members, total_wg;
    const int32_t *row_perm, *col_perm;
    int m;
    const uint8_t *level;
    const int64_t *byte_off;
    uint8_t *codes;
    float *scale, *zero;
    GridConsts gc;
    int cmax;
    int64_t cols;
    int opu;
};

template <int LPG, int CPL, int RS, int TMAX>
static int launch_gpack_g(sbits_ctx *ctx, const FusedPackLaunch &a)
{
    const int T = fused_threads(a.cols, CPL, TMAX);
    auto *fn = &gather_pack_kernel<LPG, CPL, RS, TMAX>;
    SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 159 * 1024));
    const size_t lds = (size_t)RS * a.cols * 2 + (size_t)(CPL * T / LPG) * ((size_t)RS * LPG * a.cmax + 8);
    hipLaunchKernelGGL(fn, dim3((unsigned)a.total_wg), dim3(T), lds, ctx->stream, a.descs, a.members,
                       a.wg_start, a.n_members, a.row_perm, a.col_perm, a.m, a.level, a.byte_off, a.codes, a.scale,
                       a.zero, a.gc, a.cmax, a.opu);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

template <int LPG>
static int launch_gpack_l(sbits_ctx *ctx, const FusedPackLaunch &a)
{
    const int64_t chunks = a.cols / 8;
    if (chunks <= 512) return launch_gpack_g<LPG, 1, 4, 512>(ctx, a);
    if (chunks <= 1024) return launch_gpack_g<LPG, 2, 2, 512>(ctx, a);
    if (chunks <= 2048) return launch_gpack_g<LPG, 2, 2, 1024>(ctx, a);
    if (chunks <= 4096) return launch_gpack_g<LPG, 4, 1, 1024>(ctx, a);
    return SBITS_ERR_BAD_SHAPE;
}

}  // namespace sbits

using namespace sbits;

// shapes the fused kernel takes: 64- or 128-column blocks, rows of at most FU_MAX_COLS elements
// The route is chosen per class of matrices with equal column count.  Rows of up to FU_MAX_COLS
// elements are staged whole (weights and sensitivities) by the one-pass cost kernel; matrices with
// wider rows (up to the plan's limit of 32768) take, one by one, the reorder-gather into a copy in the
// workspace and the cost kernel for reordered matrices.  The packing kernel stages weights only and
// takes every row length.
bool sbits_fused_shapes_ok(const sbits_plan *plan)
{
    if (plan->n != 64 && plan->n != 128) return false;
    return plan->max_cols <= FU_PACK_MAX_COLS;
}
bool sbits_fused_all_staged(const sbits_plan *plan)
{
    return sbits_fused_shapes_ok(plan) && plan->max_cols <= FU_MAX_COLS;
}

static size_t octet_partial_bytes(const sbits_plan *plan)
{
    const size_t per_octet = (size_t)(plan->K > 2 ? plan->K : 2);     // the surrogates keep two sums per block
    return sbits_align_up((size_t)plan->N * (size_t)(plan->m / 8) * per_octet * 4, 256);
}
// octet partials: one float per (block, octet of the block, candidate); then room for the reordered
// copy (bf16, then fp32) of the largest matrix whose rows are too wide to be staged
size_t sbits_fused_ws_bytes(const sbits_plan *plan)
{
    if (!sbits_fused_shapes_ok(plan)) return 0;
    size_t spill = 0;
    for (int i = 0; i < plan->n_mats; ++i) {
        if (plan->cols[i] <= FU_MAX_COLS) continue;
        const size_t el = (size_t)plan->rows[i] * (size_t)plan->cols[i];
        const size_t b = sbits_align_up(el * 2, 256) + sbits_align_up(el * 4, 256);
        if (b > spill) spill = b;
    }
    return octet_partial_bytes(plan) + spill;
}

// The kernels that read sensitivities rely on 16-bit register-half loads filling the other half with
// zeros (the device's target id says "sramecc+").  (That every source row starts on a 16-byte boundary,
// which the row loads need, is a rule of every entry point that takes matrices: checked there.)
bool sbits_fused_layout_ok(const sbits_plan *plan, bool need_s)
{
    return !need_s || plan->ctx->d16_zero_fill;
}

// matrices grouped by column count; members and workgroup prefixes go to slots 3 and 4 of the
// workspace head (the tables depend on shapes only: built once, kept in the plan)
static int fused_classes(sbits_plan *plan, void *ws, int **d_mem, int **d_pre)
{
    sbits_ctx *ctx = plan->ctx;
    if (plan->fused_members.empty()) {
        std::vector<int64_t> classes;
        for (int i = 0; i < plan->n_mats; ++i) {
            bool seen = false;
            for (int64_t c : classes) seen = seen || c == plan->cols[i];
            if (!seen) classes.push_back(plan->cols[i]);
        }
        for (int64_t c : classes) {
            sbits_plan::FusedClass fc;
            fc.cols = c;
            fc.first = (int)plan->fused_members.size();
            fc.pre_first = (int)plan->fused_pre.size();
            fc.n = 0;
            // octets per workgroup: FU_OPU, halved while the class would not even give every CU a few
            // workgroups (one decoder layer of a streamed model is such a plan)
            int opu = FU_OPU;
            auto class_wgs = [&](int o) {
                int64_t t = 0;
                for (int i = 0; i < plan->n_mats; ++i)
                    if (plan->cols[i] == c) t += (plan->rows[i] / 8 + o - 1) / o;
                return t;
            };
            while (opu > 2 && class_wgs(opu) < 2048) opu >>= 1;
            fc.opu = opu;
            int64_t t = 0;
            for (int i = 0; i < plan->n_mats; ++i) {
                if (plan->cols[i] != c) continue;
                plan->fused_members.push_back(i);
                plan->fused_pre.push_back((int)t);
                t += (plan->rows[i] / 8 + opu - 1) / opu;
                ++fc.n;
            }
            if (t > 0x7fffffff) {
                plan->fused_members.clear(); plan->fused_pre.clear(); plan->fused_classes.clear();
                return SBITS_ERR_BAD_SHAPE;
            }
            plan->fused_pre.push_back((int)t);
            plan->fused_classes.push_back(fc);
        }
    }
    *d_mem = sbits_prefix_ptr(plan, ws, 3);
    *d_pre = sbits_prefix_ptr(plan, ws, 4);
    SBITS_HIP(ctx, hipMemcpyAsync(*d_mem, plan->fused_members.data(), plan->fused_members.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(*d_pre, plan->fused_pre.data(), plan->fused_pre.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    return SBITS_OK;
}

// One launch per class of matrices with equal column count (equal LDS need, equal chunks per
// lane); the descriptor table is already in the workspace head.  w_re may be null.
int sbits_launch_gather_cost_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                                 void *w_re, float *cost, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    if (!sbits_fused_shapes_ok(plan) || !sbits_fused_layout_ok(plan, true)) return SBITS_ERR_BAD_SHAPE;
    int *d_mem, *d_pre;
    int rc0 = fused_classes(plan, ws, &d_mem, &d_pre);
    if (rc0) return rc0;
    FusedLaunch a;
    memset(&a, 0, sizeof a);
    a.descs = sbits_desc_ptr(ws);
    a.row_perm = row_perm;
    a.col_perm = col_perm;
    a.m = plan->m;
    a.w_re = static_cast<uint16_t *>(w_re);
    a.part = static_cast<float *>(sbits_scratch(plan, ws));
    for (const sbits_plan::FusedClass &fc : plan->fused_classes) {
        a.members = d_mem + fc.first;
        a.wg_start = d_pre + fc.pre_first;
        a.n_members = fc.n;
        a.total_wg = plan->fused_pre[fc.pre_first + fc.n];
        a.cols = fc.cols;
        a.opu = fc.opu;
        if (a.total_wg == 0 || fc.cols > FU_MAX_COLS) continue;
        const bool z0 = plan->bits[0] == 0;                     // a 0-bit candidate (the first of the list) has no grid
        sbits_fill_grid_consts(plan->bits + z0, plan->K - z0, &a.gc);
        a.kstride = plan->K;
        a.koff = 0;
        const int rc = plan->n == 64 ? launch_fused_l<8>(plan->K, z0, ctx, a) : launch_fused_l<16>(plan->K, z0, ctx, a);
        if (rc) return rc;
    }
    const int64_t NK = plan->N * plan->K;
    if (NK > 0) {
        hipLaunchKernelGGL(octet_finish_kernel, dim3((unsigned)((NK + 255) / 256)), dim3(256), 0, ctx->stream,
                           a.part, a.descs, plan->n_mats, NK, plan->K, plan->m / 8, cost);
        SBITS_HIP(ctx, hipGetLastError());
    }
    // matrices with rows too wide to stage: reordered copy in the workspace, then the cost kernel on it; their
    // rows of the table are written after the tree kernel above (which found nothing of theirs in part[])
    for (int i = 0; i < plan->n_mats; ++i) {
        if (plan->cols[i] <= FU_MAX_COLS) continue;
        const MatDesc &d = plan->descs[i];
        const size_t el = (size_t)plan->rows[i] * (size_t)plan->cols[i];
        char *tmp = static_cast<char *>(sbits_scratch(plan, ws)) + octet_partial_bytes(plan);
        void *w_tmp = w_re ? static_cast<void *>(static_cast<uint16_t *>(w_re) + d.elem_off) : static_cast<void *>(tmp);
        float *s_tmp = reinterpret_cast<float *>(tmp + sbits_align_up(el * 2, 256));
        int rc = sbits_launch_gather(ctx, d.w, d.s, plan->rows[i], plan->cols[i], d.ld_w, d.ld_s, row_perm + d.row_off,
                                     col_perm + d.col_off, w_tmp, s_tmp);
        if (rc) return rc;
        rc = sbits_launch_cost(ctx, w_tmp, s_tmp, plan->rows[i], plan->cols[i], plan->m, plan->n, plan->bits, plan->K,
                               cost + d.block_base * plan->K);
        if (rc) return rc;
    }
    return SBITS_OK;
}

// the packing stage on the original weights, one launch per class
int sbits_launch_gather_pack_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                                 const uint8_t *level, const int64_t *byte_off, uint8_t *codes, float *scale,
                                 float *zero, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    if (!sbits_fused_shapes_ok(plan) || !sbits_fused_layout_ok(plan, false)) return SBITS_ERR_BAD_SHAPE;
    int *d_mem, *d_pre;
    int rc0 = fused_classes(plan, ws, &d_mem, &d_pre);
    if (rc0) return rc0;
    FusedPackLaunch a;
    memset(&a, 0, sizeof a);
    sbits_fill_grid_consts(plan->bits, plan->K, &a.gc);
    a.descs = sbits_desc_ptr(ws);
    a.row_perm = row_perm;
    a.col_perm = col_perm;
    a.m = plan->m;
    a.level = level; a.byte_off = byte_off; a.codes = codes; a.scale = scale; a.zero = zero;
    a.cmax = plan->bits[plan->K - 1];
    for (const sbits_plan::FusedClass &fc : plan->fused_classes) {
        a.members = d_mem + fc.first;
        a.wg_start = d_pre + fc.pre_first;
        a.n_members = fc.n;
        a.total_wg = plan->fused_pre[fc.pre_first + fc.n];
        a.cols = fc.cols;
        a.opu = fc.opu;
        if (a.total_wg == 0) continue;
        const int rc = plan->n == 64 ? launch_gpack_l<8>(ctx, a) : launch_gpack_l<16>(ctx, a);
        if (rc) return rc;
    }
    return SBITS_OK;
}

// dynamic-sensitivity surrogates of all matrices: the one-pass kernel in its second mode, then the
// tree over the octets with the 2^-bits factor of s_down
int sbits_launch_surrogates_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                                const uint8_t *level, float *s_up, float *s_down, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    if (!sbits_fused_all_staged(plan) || !sbits_fused_layout_ok(plan, true)) return SBITS_ERR_BAD_SHAPE;
    int *d_mem, *d_pre;
    int rc0 = fused_classes(plan, ws, &d_mem, &d_pre);
    if (rc0) return rc0;
    FusedLaunch a;
    memset(&a, 0, sizeof a);
    sbits_fill_grid_consts(plan->bits, plan->K, &a.gc);
    a.descs = sbits_desc_ptr(ws);
    a.row_perm = row_perm;
    a.col_perm = col_perm;
    a.m = plan->m;
    a.w_re = nullptr;
    a.part = static_cast<float *>(sbits_scratch(plan, ws));
    a.level = level;
    a.kstride = 2;
    a.koff = 0;
    for (const sbits_plan::FusedClass &fc : plan->fused_classes) {
        a.members = d_mem + fc.first;
        a.wg_start = d_pre + fc.pre_first;
        a.n_members = fc.n;
        a.total_wg = plan->fused_pre[fc.pre_first + fc.n];
        a.cols = fc.cols;
        a.opu = fc.opu;
        if (a.total_wg == 0) continue;
        const int rc = plan->n == 64 ? launch_surrogates_l<8>(ctx, a) : launch_surrogates_l<16>(ctx, a);
        if (rc) return rc;
    }
    if (plan->N > 0) {
        hipLaunchKernelGGL(surrogate_finish_kernel, dim3((unsigned)((2 * plan->N + 255) / 256)), dim3(256), 0,
                           ctx->stream, a.part, a.descs, plan->n_mats, plan->N, plan->m / 8, level, a.gc, s_up, s_down);
        SBITS_HIP(ctx, hipGetLastError());
    }
    return SBITS_OK;
}
