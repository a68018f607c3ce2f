// Bi-directional channel reordering (paper Sec. 4.1): channel scores, argsort,
// and the reorder-gather of weights and sensitivities.  Every kernel serves all
// matrices of a plan in one launch (descriptor table + workgroup prefix) or a
// single matrix whose descriptor travels as a kernel argument.
//
// Scores.  Row score = l1 norm of the row of S, column score = l1 norm of the
// column, each summed in the canonical order: runs of 8 consecutive elements
// left to right from +0, then an adjacent-pair tree over the runs (zero padded
// to a power of two).  One pass over S serves both directions.  A workgroup of
// four waves walks a band of 256 rows over a panel of 4096 columns, row by row
// (16 KiB of consecutive bytes per row); a wave owns two 512-column segments of
// the panel and reads each with two 1 KiB loads, so a run of 8 columns sits in a
// lane pair and the 16 columns of a lane keep their sums in registers for the
// whole band.  The partial trees (per row and 512-column segment; per column
// and 256-row band) go to the workspace and a small kernel finishes them.
//
// Argsort.  Descending by score, ties to the lower index: a stable LSD radix
// sort (4 passes of 8 bits) of the inverted ordered-float keys, one workgroup
// of 16 waves per channel array, all arrays of the plan side by side.
//
// Gather.  out[i][j] = in[rp[i]][cp[j]]: the source row is staged in LDS with
// coalesced 128-bit loads and read out permuted, so global traffic stays
// coalesced in both directions.
#include <string.h>

#include <vector>

#include "sbits_device.hpp"
#include "sbits_internal.hpp"

namespace sbits {

// ================================================================ scores
constexpr int SC_THREADS = 256;
constexpr int SC_ROWS = 256;    // rows per band (32 octets): one workgroup walks a whole band
constexpr int SC_COLS = 512;    // columns per segment: one wave, two 1 KiB loads per row
constexpr int SC_PANEL = 8;     // segments per workgroup: 4 waves x 2 segments = 4096 columns = 16 KiB per row

// rowpart[r][seg]  : tree over the 64 column runs of segment seg (zero beyond C)
// colpart[band][c] : tree over the 32 row runs of band (zero beyond R)
//
// A workgroup reads rows of 16 KiB (its panel of 8 segments) top to bottom, so HBM sees long
// consecutive runs, and every load instruction of a wave covers 1 KiB of consecutive bytes (whole
// cache lines), which is what non-temporal loads need to run at full rate.  Wave w owns segments
// w and w + 4 of the panel.  Inside a segment lane l owns columns 4l..4l+3 and 256+4l..256+4l+3:
// a run of 8 consecutive columns sits in the lane pair (2k, 2k+1).  Column sums stay in registers
// for the whole band (16 columns per lane, a 5-level adjacent-pair tree over the 32 octets).
__global__ __launch_bounds__(SC_THREADS, 2)
void score_partial_kernel(const MatDesc *__restrict__ descs, MatDesc one, const int *__restrict__ wg_start,
                          int n_mats, float *__restrict__ rowpart_all, float *__restrict__ colpart_all)
{
    const int mat = descs ? find_matrix(wg_start, n_mats, (int)blockIdx.x) : 0;
    const MatDesc d = descs ? descs[mat] : one;
    const int lid = (int)blockIdx.x - (descs ? wg_start[mat] : 0);
    const int npanel = (d.nseg + SC_PANEL - 1) / SC_PANEL;
    const int band = lid / npanel, panel = lid - band * npanel;
    const int R = (int)d.rows, C = (int)d.cols;
    const int64_t ld = d.ld_s;
    // the descriptor's pointer is a generic one for the compiler: say that it is global memory
    typedef const char __attribute__((address_space(1))) *gcharp;
    typedef const __attribute__((address_space(1))) f32x4_t *gf4p;
    gcharp Sg = (gcharp)(reinterpret_cast<const char *>(d.s));
    float *__restrict__ rowpart = rowpart_all + d.rowpart_off;
    float *__restrict__ colpart = colpart_all + d.colpart_off;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int seg[2], col0[2][2];
    bool ok[2][2];
    uint32_t voff[2][2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        seg[j] = panel * SC_PANEL + wave + 4 * j;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            col0[j][h] = seg[j] * SC_COLS + h * (SC_COLS / 2) + lane * 4;
            ok[j][h] = col0[j][h] < C;                   // C is a multiple of 8 (4 columns: all in or all out)
            voff[j][h] = (uint32_t)(ok[j][h] ? col0[j][h] : C - 4) * 4u;   // clamped: in bounds, value dropped
        }
    }
    const int rbase = band * SC_ROWS;

    // two rows of the panel per pipeline stage: 8 loads of 16 bytes per lane
    struct Stage { float4 v[2][2][2]; };             // [row][segment][half of the segment]
    auto load_stage = [&](Stage &o, int r0) {
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            int r = rbase + r0 + rr;
            r = r < R ? r : R - 1;                   // rows beyond R are clamped and dropped
            gcharp p = Sg + (int64_t)r * ld * 4;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const f32x4_t t = __builtin_nontemporal_load((gf4p)(p + voff[j][h]));
                    o.v[rr][j][h] = make_float4(t.x, t.y, t.z, t.w);
                }
        }
    };

    // sum of one run of 8 columns held by a lane pair, left to right; both lanes end with it
    auto run_sum = [&](const float (&x)[4]) {
        const float p = ((x[0] + x[1]) + x[2]) + x[3];               // the run's first four (even lane)
        const float start = dpp_mov<0xA0>(p);                         // quad_perm [0,0,2,2]: odd lane <- even lane
        const float q = (((start + x[0]) + x[1]) + x[2]) + x[3];      // odd lane: the whole run
        return dpp_mov<0xF5>(q);                                      // quad_perm [1,1,3,3]: both lanes <- odd lane
    };
    // adjacent-pair tree over the 32 runs held by 64 lanes (lane pairs agree on entry)
    auto tree_runs = [&](float v) {
        v = v + dpp_mov<DPP_XOR2>(v);
        v = v + dpp_mov<DPP_HALF_MIRROR>(v);
        v = v + dpp_mov<DPP_MIRROR>(v);
        v = v + __shfl_xor(v, 16);
        v = v + __shfl_xor(v, 32);
        return v;
    };

    float colrun[16], t1[16], t2[16], t3[16], t4[16], t5[16], col[16];
    auto process = [&](const Stage &cur, int r0) {   // rows r0, r0 + 1 of the band
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int rb = r0 + rr;                  // row inside the band
            const bool rok = rbase + rb < R;
            if ((rb & 7) == 0) {
#pragma unroll
                for (int e = 0; e < 16; ++e) colrun[e] = 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float x[2][4];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const float4 t = cur.v[rr][j][h];
                    const float raw[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        x[h][e] = (ok[j][h] && rok) ? fabsf(raw[e]) : 0.0f;
                        colrun[j * 8 + h * 4 + e] = colrun[j * 8 + h * 4 + e] + x[h][e];   // top to bottom, 8 rows
                    }
                }
                // runs of 8 left to right, then the adjacent-pair tree over the segment's 64 runs
                // (32 in its first 256 columns, 32 in the second)
                const float rs = tree_runs(run_sum(x[0])) + tree_runs(run_sum(x[1]));
                if (lane == 0 && rok && seg[j] < d.nseg) rowpart[(int64_t)(rbase + rb) * d.nseg + seg[j]] = rs;
            }
            if ((rb & 7) == 7) {
                // columns: adjacent-pair tree over the band's 32 octets, fed one octet at a time
                const int oc = rb >> 3;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float v = colrun[e];
                    if (oc & 1) {
                        v = t1[e] + v;
                        if (oc & 2) {
                            v = t2[e] + v;
                            if (oc & 4) {
                                v = t3[e] + v;
                                if (oc & 8) {
                                    v = t4[e] + v;
                                    if (oc & 16) v = t5[e] + v;
                                    else t5[e] = v;
                                } else {
                                    t4[e] = v;
                                }
                            } else {
                                t3[e] = v;
                            }
                        } else {
                            t2[e] = v;
                        }
                    } else {
                        t1[e] = v;
                    }
                    col[e] = v;
                }
            }
        }
    };
    // two buffers in ping-pong: the next two rows are in flight while the current two are summed
    Stage A, B;
    load_stage(A, 0);
#pragma unroll 1
    for (int r0 = 0; r0 < SC_ROWS; r0 += 4) {
        load_stage(B, r0 + 2);
        process(A, r0);
        load_stage(A, r0 + 4 < SC_ROWS ? r0 + 4 : SC_ROWS - 2);   // the last reload is redundant and harmless
        process(B, r0 + 2);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (ok[j][h]) {
                float *dst = colpart + (int64_t)band * C + col0[j][h];
                *reinterpret_cast<float4 *>(dst) = make_float4(col[j * 8 + h * 4], col[j * 8 + h * 4 + 1],
                                                               col[j * 8 + h * 4 + 2], col[j * 8 + h * 4 + 3]);
            }
}

// adjacent-pair tree over 32 leaves x[(i0 + i) * stride], i < 32, zero beyond n
__device__ __forceinline__ float tree32(const float *__restrict__ x, int i0, int n, int64_t stride)
{
    float v[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = (i0 + i < n) ? x[(int64_t)(i0 + i) * stride] : 0.0f;
#pragma unroll
    for (int w = 16; w >= 1; w >>= 1)
#pragma unroll
        for (int i = 0; i < w; ++i) v[i] = v[2 * i] + v[2 * i + 1];
    return v[0];
}

// adjacent-pair tree over n <= 128 leaves, zero padded to a power of two (adding the padding
// is the identity, so trees of 32, 64 and 128 leaves nest)
__device__ __forceinline__ float tree_upto128(const float *__restrict__ x, int n, int64_t stride)
{
    float a = tree32(x, 0, n, stride);
    if (n > 32) a = a + tree32(x, 32, n, stride);
    if (n > 64) {
        float b = tree32(x, 64, n, stride);
        if (n > 96) b = b + tree32(x, 96, n, stride);
        a = a + b;
    }
    return a;
}

// one thread per channel; scores = [rows of matrix 0 | rows of matrix 1 | ... | cols of matrix 0 | ...]
__global__ void score_finish_kernel(const MatDesc *__restrict__ descs, MatDesc one, int n_mats,
                                    int64_t sum_rows, int64_t sum_cols,
                                    const float *__restrict__ rowpart_all, const float *__restrict__ colpart_all,
                                    float *__restrict__ rs_all, float *__restrict__ cs_all)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= sum_rows + sum_cols) return;
    const bool is_row = t < sum_rows;
    const int64_t ch = is_row ? t : t - sum_rows;
    int mat = 0;
    if (descs) {                                     // largest mat with offset <= ch
        int lo = 0, hi = n_mats;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            const int64_t o = is_row ? descs[mid].row_off : descs[mid].col_off;
            if (o <= ch) lo = mid; else hi = mid;
        }
        mat = lo;
    }
    const MatDesc &d = descs ? descs[mat] : one;
    if (is_row) {
        const int64_t r = ch - d.row_off;
        rs_all[ch] = tree_upto128(rowpart_all + d.rowpart_off + r * d.nseg, d.nseg, 1);
    } else {
        const int64_t c = ch - d.col_off;
        cs_all[ch] = tree_upto128(colpart_all + d.colpart_off + c, d.nband, d.cols);
    }
}

// ================================================================ argsort
constexpr int RS_THREADS = 1024;
constexpr int RS_WAVES = RS_THREADS / 64;

__device__ __forceinline__ unsigned int sort_key(float f)
{
    const unsigned int u = __float_as_uint(f + 0.0f);                 // -0 -> +0
    const unsigned int ord = (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // ascending in f
    return ~ord;                                                      // ascending key = descending score
}

// Array a of the launch: a < n_mats -> the rows of matrix a, else the columns of matrix a - n_mats.
// k0/k1/i0/i1 are ping-pong buffers with the same indexing as the score array.
// arr_mode (may be null = all SORT): what to do with array a; arr_segment (with arr_mode): 0 or the
// length of the pieces that are sorted one by one (a permutation that stays inside attention heads).
enum { ARR_SORT = 0, ARR_IDENTITY = 1, ARR_SKIP = 2 };
__global__ __launch_bounds__(RS_THREADS)
void radix_argsort_kernel(const MatDesc *__restrict__ descs, MatDesc one, int n_mats, int64_t sum_rows,
                          const float *__restrict__ scores, unsigned int *__restrict__ k0,
                          unsigned int *__restrict__ k1, unsigned int *__restrict__ i0,
                          unsigned int *__restrict__ i1, int32_t *__restrict__ row_perm,
                          int32_t *__restrict__ col_perm, const int *__restrict__ arr_mode,
                          const int *__restrict__ arr_segment)
{
    __shared__ unsigned int hist[RS_WAVES][256];     // per-wave digit counts, then running offsets
    __shared__ unsigned int total[256];
    const int a = blockIdx.x;
    const bool is_row = a < n_mats;
    const MatDesc &d = descs ? descs[is_row ? a : a - n_mats] : one;
    const int n_all = (int)(is_row ? d.rows : d.cols);
    const int64_t off_all = is_row ? d.row_off : sum_rows + d.col_off;
    int32_t *__restrict__ perm_all = is_row ? row_perm + d.row_off : col_perm + d.col_off;
    const int mode = arr_mode ? arr_mode[a] : ARR_SORT;
    if (mode == ARR_SKIP) return;
    if (mode == ARR_IDENTITY) {
        for (int i = threadIdx.x; i < n_all; i += RS_THREADS) perm_all[i] = i;
        return;
    }
    const int piece = (arr_mode && arr_segment[a] > 0) ? arr_segment[a] : n_all;
    for (int p0 = 0; p0 < n_all; p0 += piece) {      // (uniform over the workgroup)
    const int n = min(piece, n_all - p0);
    const int64_t off = off_all + p0;
    int32_t *__restrict__ perm = perm_all + p0;
    const float *__restrict__ sc = scores + off;
    unsigned int *kb[2] = {k0 + off, k1 + off};
    unsigned int *ib[2] = {i0 + off, i1 + off};

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // each wave owns a contiguous segment (a multiple of 64 long) of the current order
    const int seg = ((n + RS_WAVES - 1) / RS_WAVES + 63) / 64 * 64;
    const int beg = wave * seg, end = min(beg + seg, n);

    for (int i = tid; i < n; i += RS_THREADS) {
        kb[0][i] = sort_key(sc[i]);
        ib[0][i] = (unsigned int)i;
    }
    __syncthreads();

    for (int pass = 0; pass < 4; ++pass) {
        const unsigned int *__restrict__ kin = kb[pass & 1];
        const unsigned int *__restrict__ iin = ib[pass & 1];
        unsigned int *__restrict__ kout = kb[(pass + 1) & 1];
        unsigned int *__restrict__ iout = ib[(pass + 1) & 1];
        const int shift = 8 * pass;

        for (int b = lane; b < 256; b += 64) hist[wave][b] = 0;
        __syncthreads();
        for (int i = beg + lane; i < end; i += 64) atomicAdd(&hist[wave][(kin[i] >> shift) & 255u], 1u);
        __syncthreads();
        // offsets in (digit, wave) order: first the per-digit totals and the per-wave prefix inside a digit
        if (tid < 256) {
            unsigned int run = 0;
            for (int w = 0; w < RS_WAVES; ++w) {
                const unsigned int c = hist[w][tid];
                hist[w][tid] = run;
                run += c;
            }
            total[tid] = run;
        }
        __syncthreads();
        if (wave == 0) {                             // exclusive scan of the 256 totals by one wave
            unsigned int v[4], s = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { v[j] = total[lane * 4 + j]; s += v[j]; }
            unsigned int inc = s;
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned int t = __shfl_up(inc, o);
                if (lane >= o) inc += t;
            }
            unsigned int ex = inc - s;
#pragma unroll
            for (int j = 0; j < 4; ++j) { total[lane * 4 + j] = ex; ex += v[j]; }
        }
        __syncthreads();
        for (int b = lane; b < 256; b += 64) hist[wave][b] += total[b];
        __syncthreads();
        // stable scatter: the wave walks its segment in order, 64 elements at a time
        for (int i = beg + lane; i - lane < end; i += 64) {
            const bool valid = i < end;
            const unsigned int key = valid ? kin[i] : 0u;
            const unsigned int idx = valid ? iin[i] : 0u;
            const unsigned int dg = (key >> shift) & 255u;
            unsigned long long same = __ballot(valid);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const unsigned long long bal = __ballot((dg >> b) & 1u);
                same &= ((dg >> b) & 1u) ? bal : ~bal;
            }
            const unsigned long long lt = (1ull << lane) - 1ull;
            const unsigned int rank = __popcll(same & lt);
            if (valid) {
                const unsigned int base = hist[wave][dg];
                const unsigned int dst = base + rank;
                if (pass == 3) perm[dst] = (int32_t)idx + p0;
                else { kout[dst] = key; iout[dst] = idx; }
                if (rank == 0) hist[wave][dg] = base + __popcll(same);
            }
        }
        __syncthreads();
    }
    }
}

// ---- coupled reordering (paper App. "Channel Reordering": one permutation for all the matrix
// dimensions that carry the same activation; the scores of the coupled dimensions are summed) ----
// Arrays are numbered as in the sort kernel.  arr_next[a]: the next member of a's group, or -1.
// The leader (first member) of a group accumulates, member after member in array order:
//   s[leader][j] = (..(s[leader][j] + s[m1][j]) + s[m2][j]) + ...
// A member with repeat r > 1 is r times as long: each piece of seg channels of the group stands
// for r consecutive pieces of the member (one value head serving r query heads); its r scores of
// channel j are added one after the other, lower piece first.
__global__ __launch_bounds__(256)
void group_sum_kernel(const MatDesc *__restrict__ descs, int n_mats, int64_t sum_rows, float *__restrict__ scores,
                      const int *__restrict__ arr_mode, const int *__restrict__ arr_next,
                      const int *__restrict__ arr_seg, const int *__restrict__ arr_rep)
{
    const int a = blockIdx.y;
    if (arr_mode[a] != ARR_SORT || arr_next[a] < 0) return;      // only leaders with other members
    const bool is_row = a < n_mats;
    const MatDesc &d = descs[is_row ? a : a - n_mats];
    const int n = (int)(is_row ? d.rows : d.cols);
    const int sg = arr_seg[a];
    const int64_t off = is_row ? d.row_off : sum_rows + d.col_off;
    for (int j = (int)(blockIdx.x * blockDim.x + threadIdx.x); j < n; j += (int)(gridDim.x * blockDim.x)) {
        float acc = scores[off + j];
        for (int b = arr_next[a]; b >= 0; b = arr_next[b]) {
            const bool br = b < n_mats;
            const MatDesc &e = descs[br ? b : b - n_mats];
            const float *sb = scores + (br ? e.row_off : sum_rows + e.col_off);
            const int r = arr_rep[b];
            if (r == 1) {
                acc = acc + sb[j];
            } else {                                             // sg > 0 (checked on the host)
                const int64_t base = (int64_t)(j / sg) * r * sg + j % sg;
                for (int t = 0; t < r; ++t) acc = acc + sb[base + (int64_t)t * sg];
            }
        }
        scores[off + j] = acc;
    }
}

// the members of a group take their leader's permutation; a member with repeat r applies the
// permutation of group piece p inside each of its pieces r*p .. r*p + r - 1
__global__ __launch_bounds__(256)
void replicate_perm_kernel(const MatDesc *__restrict__ descs, int n_mats, int32_t *__restrict__ row_perm,
                           int32_t *__restrict__ col_perm, const int *__restrict__ arr_mode,
                           const int *__restrict__ arr_leader, const int *__restrict__ arr_seg,
                           const int *__restrict__ arr_rep)
{
    const int a = blockIdx.y;
    if (arr_mode[a] != ARR_SKIP) return;
    const int l = arr_leader[a];
    const bool ar = a < n_mats, lr = l < n_mats;
    const MatDesc &d = descs[ar ? a : a - n_mats];
    const MatDesc &e = descs[lr ? l : l - n_mats];
    const int n = (int)(ar ? d.rows : d.cols);
    const int r = arr_rep[a], sg = arr_seg[l];
    int32_t *dst = ar ? row_perm + d.row_off : col_perm + d.col_off;
    const int32_t *src = lr ? row_perm + e.row_off : col_perm + e.col_off;
    for (int j = (int)(blockIdx.x * blockDim.x + threadIdx.x); j < n; j += (int)(gridDim.x * blockDim.x)) {
        if (r == 1) {
            dst[j] = src[j];
        } else {
            const int pc = j / sg, dd = j - pc * sg;             // the member's piece and the channel inside it
            const int gbase = (pc / r) * sg;                     // first channel of the group's piece
            dst[j] = pc * sg + (src[gbase + dd] - gbase);
        }
    }
}

// ================================================================ gather
constexpr int GA_THREADS = 512;
constexpr int GA_LDS_TARGET = 48 * 1024;            // rows per workgroup are chosen to fill about this much

// T = uint16_t (bf16) or float.  A workgroup stages rpw consecutive output rows of one matrix
// (their source rows) in LDS and emits them permuted; the column indices are read once per
// column chunk and serve all rpw rows.  A launch covers the matrices of one "class" (equal
// column count, hence equal LDS need): members[] lists them, wg_start[] is their workgroup prefix.
template <class T>
__global__ __launch_bounds__(GA_THREADS)
void gather_kernel(const MatDesc *__restrict__ descs, MatDesc one, const int *__restrict__ members,
                   const int *__restrict__ wg_start, int n_members, int rpw,
                   const int32_t *__restrict__ row_perm, const int32_t *__restrict__ col_perm,
                   T *__restrict__ out_all)
{
    extern __shared__ __align__(16) unsigned char smem[];
    T *rows = reinterpret_cast<T *>(smem);
    constexpr int V = 16 / sizeof(T);               // elements per 128-bit access
    typedef const T __attribute__((address_space(1))) *gtp;

    int mem = 0;
    if (descs) mem = find_matrix(wg_start, n_members, (int)blockIdx.x);
    const MatDesc &d = descs ? descs[members[mem]] : one;
    const int R = (int)d.rows, C = (int)d.cols;
    const int i0 = ((int)blockIdx.x - (descs ? wg_start[mem] : 0)) * rpw;     // first output row
    const int nr = min(rpw, R - i0);
    const T *in = sizeof(T) == 2 ? reinterpret_cast<const T *>(d.w) : reinterpret_cast<const T *>(d.s);
    const int64_t ld = sizeof(T) == 2 ? d.ld_w : d.ld_s;
    const int32_t *__restrict__ rp = row_perm + d.row_off;
    const int32_t *__restrict__ cp = col_perm + d.col_off;

    for (int r = 0; r < nr; ++r) {
        int sr = rp[i0 + r];
        sr = sr < 0 ? 0 : (sr >= R ? R - 1 : sr);   // a permutation never trips this; keeps a bad one in bounds
        const T *src = in + (int64_t)sr * ld;
        T *dstl = rows + (size_t)r * C;
        if ((reinterpret_cast<uintptr_t>(src) & 15) == 0) {
            for (int j = threadIdx.x * V; j < C; j += GA_THREADS * V)
            {
                const u32x4_t v = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4_t *)(src + j));
                *reinterpret_cast<uint4 *>(dstl + j) = make_uint4(v.x, v.y, v.z, v.w);
            }
        } else {
            for (int j = threadIdx.x; j < C; j += GA_THREADS) dstl[j] = *(gtp)(src + j);
        }
    }
    __syncthreads();
    T *dst = out_all + d.elem_off + (int64_t)i0 * C;      // dense output, C % 8 == 0: 16-byte aligned rows
    for (int j = threadIdx.x * V; j < C; j += GA_THREADS * V) {
        int ci[V];
        const int4 c0 = *reinterpret_cast<const int4 *>(cp + j);
        ci[0] = c0.x; ci[1] = c0.y; ci[2] = c0.z; ci[3] = c0.w;
        if constexpr (V == 8) {
            const int4 c1 = *reinterpret_cast<const int4 *>(cp + j + 4);
            ci[4] = c1.x; ci[5] = c1.y; ci[6] = c1.z; ci[7] = c1.w;
        }
        for (int r = 0; r < nr; ++r) {
            const T *srcl = rows + (size_t)r * C;
            T tmp[V];
#pragma unroll
            for (int e = 0; e < V; ++e) tmp[e] = srcl[ci[e]];
            // written once, not read again by this kernel: streamed past the caches
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4_t *>(tmp),
                                        (__attribute__((address_space(1))) u32x4_t *)(dst + (int64_t)r * C + j));
        }
    }
}

static int gather_rows_per_wg(int64_t C, size_t elem)
{
    int64_t r = GA_LDS_TARGET / (C * (int64_t)elem);
    return (int)(r < 1 ? 1 : (r > 8 ? 8 : r));
}

}  // namespace sbits

using namespace sbits;

// ---- workspace of the reorder stage (after the head) ---------------------------------
//   scores [L] | rowpart [RP] | colpart [CP] | k0 [L] | k1 [L] | i0 [L] | i1 [L]
// with L = channels (rows + cols), RP = sum rows*nseg, CP = sum nband*cols.
struct ReorderWs {
    float *scores, *rowpart, *colpart;
    unsigned int *k0, *k1, *i0, *i1;
};

static size_t reorder_ws_layout(void *base, int64_t L, int64_t RP, int64_t CP, ReorderWs *out)
{
    char *p = static_cast<char *>(base);
    size_t b = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + b : nullptr; b += sbits_align_up(bytes, 256); return q; };
    float *scores = reinterpret_cast<float *>(take((size_t)L * 4));
    float *rowpart = reinterpret_cast<float *>(take((size_t)RP * 4));
    float *colpart = reinterpret_cast<float *>(take((size_t)CP * 4));
    unsigned int *k0 = reinterpret_cast<unsigned int *>(take((size_t)L * 4));
    unsigned int *k1 = reinterpret_cast<unsigned int *>(take((size_t)L * 4));
    unsigned int *i0 = reinterpret_cast<unsigned int *>(take((size_t)L * 4));
    unsigned int *i1 = reinterpret_cast<unsigned int *>(take((size_t)L * 4));
    if (out) { out->scores = scores; out->rowpart = rowpart; out->colpart = colpart;
               out->k0 = k0; out->k1 = k1; out->i0 = i0; out->i1 = i1; }
    return b;
}

// workgroups of score_partial_kernel for a matrix with nseg segments and nband bands
int sbits_score_wgs(int nseg, int nband) { return nband * ((nseg + SC_PANEL - 1) / SC_PANEL); }

void sbits_score_geometry(int64_t R, int64_t C, int *nseg, int *nband)
{
    *nseg = (int)((C + SC_COLS - 1) / SC_COLS);
    *nband = (int)((R + SC_ROWS - 1) / SC_ROWS);
}

size_t sbits_reorder_ws_bytes(int64_t L, int64_t RP, int64_t CP)
{
    return reorder_ws_layout(nullptr, L, RP, CP, nullptr);
}

// descriptor of a single matrix with its own (offset-free) layout
static MatDesc single_desc(const void *W, const float *S, int64_t R, int64_t C, int64_t ld_w, int64_t ld_s)
{
    MatDesc d;
    memset(&d, 0, sizeof d);
    d.w = static_cast<const uint16_t *>(W);
    d.s = S;
    d.rows = R; d.cols = C; d.ld_w = ld_w; d.ld_s = ld_s;
    sbits_score_geometry(R, C, &d.nseg, &d.nband);
    return d;
}

static int run_scores(sbits_ctx *ctx, const MatDesc *descs, const MatDesc &one, const int *d_wg_start,
                      int n_mats, int total_wg, int64_t sum_rows, int64_t sum_cols, const ReorderWs &w)
{
    hipLaunchKernelGGL(score_partial_kernel, dim3((unsigned)total_wg), dim3(SC_THREADS), 0, ctx->stream,
                       descs, one, d_wg_start, n_mats, w.rowpart, w.colpart);
    SBITS_HIP(ctx, hipGetLastError());
    const int64_t L = sum_rows + sum_cols;
    hipLaunchKernelGGL(score_finish_kernel, dim3((unsigned)((L + 255) / 256)), dim3(256), 0, ctx->stream,
                       descs, one, n_mats, sum_rows, sum_cols, w.rowpart, w.colpart, w.scores,
                       w.scores + sum_rows);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

// ---- single matrix ----------------------------------------------------------------------
int sbits_launch_scores(sbits_ctx *ctx, const float *S, int64_t R, int64_t C, int64_t ld,
                        float *row_score, float *col_score, void *scratch)
{
    MatDesc one = single_desc(nullptr, S, R, C, C, ld);
    ReorderWs w;
    reorder_ws_layout(scratch, R + C, R * one.nseg, (int64_t)one.nband * C, &w);
    int rc = run_scores(ctx, nullptr, one, nullptr, 1, sbits_score_wgs(one.nseg, one.nband), R, C, w);
    if (rc) return rc;
    if (row_score)
        SBITS_HIP(ctx, hipMemcpyAsync(row_score, w.scores, (size_t)R * 4, hipMemcpyDeviceToDevice, ctx->stream));
    if (col_score)
        SBITS_HIP(ctx, hipMemcpyAsync(col_score, w.scores + R, (size_t)C * 4, hipMemcpyDeviceToDevice, ctx->stream));
    return SBITS_OK;
}

int sbits_launch_reorder(sbits_ctx *ctx, const float *S, int64_t R, int64_t C, int64_t ld,
                         int32_t *row_perm, int32_t *col_perm, void *scratch)
{
    MatDesc one = single_desc(nullptr, S, R, C, C, ld);
    ReorderWs w;
    reorder_ws_layout(scratch, R + C, R * one.nseg, (int64_t)one.nband * C, &w);
    int rc = run_scores(ctx, nullptr, one, nullptr, 1, sbits_score_wgs(one.nseg, one.nband), R, C, w);
    if (rc) return rc;
    hipLaunchKernelGGL(radix_argsort_kernel, dim3(2), dim3(RS_THREADS), 0, ctx->stream,
                       (const MatDesc *)nullptr, one, 1, R, w.scores, w.k0, w.k1, w.i0, w.i1, row_perm, col_perm,
                       (const int *)nullptr, (const int *)nullptr);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

static int gather_attr(sbits_ctx *ctx)
{
    SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gather_kernel<float>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    SBITS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gather_kernel<uint16_t>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    return SBITS_OK;
}

int sbits_launch_gather(sbits_ctx *ctx, const void *W, const float *S, int64_t R, int64_t C,
                        int64_t ld_w, int64_t ld_s, const int32_t *rp, const int32_t *cp,
                        void *w_out, float *s_out)
{
    if ((size_t)C * 4 > 160 * 1024) return SBITS_ERR_BAD_SHAPE;
    int rc = gather_attr(ctx);
    if (rc) return rc;
    MatDesc one = single_desc(W, S, R, C, ld_w, ld_s);
    const int *nul = nullptr;
    if (w_out) {
        const int rpw = gather_rows_per_wg(C, 2);
        hipLaunchKernelGGL(gather_kernel<uint16_t>, dim3((unsigned)((R + rpw - 1) / rpw)), dim3(GA_THREADS),
                           (size_t)rpw * C * 2, ctx->stream, (const MatDesc *)nullptr, one, nul, nul, 1, rpw,
                           rp, cp, static_cast<uint16_t *>(w_out));
        SBITS_HIP(ctx, hipGetLastError());
    }
    if (s_out) {
        const int rpw = gather_rows_per_wg(C, 4);
        hipLaunchKernelGGL(gather_kernel<float>, dim3((unsigned)((R + rpw - 1) / rpw)), dim3(GA_THREADS),
                           (size_t)rpw * C * 4, ctx->stream, (const MatDesc *)nullptr, one, nul, nul, 1, rpw,
                           rp, cp, s_out);
        SBITS_HIP(ctx, hipGetLastError());
    }
    return SBITS_OK;
}

// ---- all matrices of the plan (descriptor table already in the workspace head) ------------
int sbits_launch_reorder_all(sbits_plan *plan, int32_t *row_perm, int32_t *col_perm, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    ReorderWs w;
    reorder_ws_layout(sbits_scratch(plan, ws), plan->sum_rows + plan->sum_cols, plan->sum_rowpart,
                      plan->sum_colpart, &w);
    int *d_pre = sbits_prefix_ptr(plan, ws, 1);
    SBITS_HIP(ctx, hipMemcpyAsync(d_pre, plan->score_wg_start.data(), plan->score_wg_start.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    MatDesc none;
    memset(&none, 0, sizeof none);
    int rc = run_scores(ctx, sbits_desc_ptr(ws), none, d_pre, plan->n_mats, plan->score_wg_start.back(),
                        plan->sum_rows, plan->sum_cols, w);
    if (rc) return rc;
    hipLaunchKernelGGL(radix_argsort_kernel, dim3((unsigned)(2 * plan->n_mats)), dim3(RS_THREADS), 0, ctx->stream,
                       (const MatDesc *)sbits_desc_ptr(ws), none, plan->n_mats, plan->sum_rows, w.scores,
                       w.k0, w.k1, w.i0, w.i1, row_perm, col_perm, (const int *)nullptr, (const int *)nullptr);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

// Host part of the coupled reordering: validates the groups and builds, per array a (rows of matrix
// a, or columns of matrix a - n_mats), what the sort kernel does with it (mode), the piece length
// (seg), the next member of its group (next) and, for non-leaders, the group's first member (leader).
int sbits_coupling_tables(const sbits_plan *plan, const int32_t *row_group, const int32_t *col_group, int n_groups,
                          const int32_t *group_segment, const int32_t *row_repeat, const int32_t *col_repeat,
                          std::vector<int> *mode_, std::vector<int> *seg_, std::vector<int> *next_,
                          std::vector<int> *leader_, std::vector<int> *rep_)
{
    const int nm = plan->n_mats, na = 2 * nm;
    std::vector<int> mode(na), seg(na, 0), next(na, -1), leader(na, -1), rep(na, 1);
    std::vector<int> last(n_groups > 0 ? n_groups : 0, -1);
    std::vector<int> first(last);
    auto len = [&](int a) { return a < nm ? plan->rows[a] : plan->cols[a - nm]; };
    for (int a = 0; a < na; ++a) {
        const int g = a < nm ? row_group[a] : col_group[a - nm];
        const int32_t *rp = a < nm ? row_repeat : col_repeat;
        const int r = rp ? rp[a < nm ? a : a - nm] : 1;
        if (r < 1) return SBITS_ERR_INVALID_ARG;
        if (g == SBITS_DIM_INDEPENDENT || g == SBITS_DIM_FIXED) {
            if (r != 1) return SBITS_ERR_INVALID_ARG;
            mode[a] = g == SBITS_DIM_FIXED ? ARR_IDENTITY : ARR_SORT;
            continue;
        }
        if (g < 0 || g >= n_groups) return SBITS_ERR_INVALID_ARG;
        const int sg = group_segment ? group_segment[g] : 0;
        if (sg < 0) return SBITS_ERR_BAD_SHAPE;
        rep[a] = r;
        if (first[g] < 0) {
            if (r != 1) return SBITS_ERR_INVALID_ARG;              // the first member carries the group's length
            if (sg > 0 && len(a) % sg) return SBITS_ERR_BAD_SHAPE;
            first[g] = last[g] = a;
            mode[a] = ARR_SORT;
            seg[a] = sg;
        } else {
            if (r > 1 && sg == 0) return SBITS_ERR_BAD_SHAPE;     // repeats are repeats of pieces
            if (len(a) != (int64_t)r * len(first[g])) return SBITS_ERR_BAD_SHAPE;   // the same activation
            mode[a] = ARR_SKIP;
            leader[a] = first[g];
            next[last[g]] = a;
            last[g] = a;
        }
    }
    if (mode_) { *mode_ = mode; *seg_ = seg; *next_ = next; *leader_ = leader; *rep_ = rep; }
    return SBITS_OK;
}

// Coupled reordering of all matrices.  group[a] for every array a (rows of matrix a, or columns of
// matrix a - n_mats): SBITS_DIM_INDEPENDENT, SBITS_DIM_FIXED or a group id; segment[g]: 0 or the
// piece length for group g; repeat: pieces of the member per piece of the group.  Tables go to
// slots 6..10 of the workspace head.
int sbits_launch_reorder_coupled_all(sbits_plan *plan, const int32_t *row_group, const int32_t *col_group,
                                     int n_groups, const int32_t *group_segment, const int32_t *row_repeat,
                                     const int32_t *col_repeat, int32_t *row_perm, int32_t *col_perm, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    const int nm = plan->n_mats, na = 2 * nm;
    std::vector<int> mode, seg, next, leader, rep;
    int rcv = sbits_coupling_tables(plan, row_group, col_group, n_groups, group_segment, row_repeat, col_repeat,
                                    &mode, &seg, &next, &leader, &rep);
    if (rcv) return rcv;
    int *d_mode = sbits_prefix_ptr(plan, ws, 6), *d_seg = sbits_prefix_ptr(plan, ws, 7);
    int *d_next = sbits_prefix_ptr(plan, ws, 8), *d_leader = sbits_prefix_ptr(plan, ws, 9);
    int *d_rep = sbits_prefix_ptr(plan, ws, 10);
    SBITS_HIP(ctx, hipMemcpyAsync(d_mode, mode.data(), (size_t)na * 4, hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(d_seg, seg.data(), (size_t)na * 4, hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(d_next, next.data(), (size_t)na * 4, hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(d_leader, leader.data(), (size_t)na * 4, hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(d_rep, rep.data(), (size_t)na * 4, hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipStreamSynchronize(ctx->stream));           // the host vectors go away on return

    ReorderWs w;
    reorder_ws_layout(sbits_scratch(plan, ws), plan->sum_rows + plan->sum_cols, plan->sum_rowpart,
                      plan->sum_colpart, &w);
    int *d_pre = sbits_prefix_ptr(plan, ws, 1);
    SBITS_HIP(ctx, hipMemcpyAsync(d_pre, plan->score_wg_start.data(), plan->score_wg_start.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    MatDesc none;
    memset(&none, 0, sizeof none);
    const MatDesc *descs = sbits_desc_ptr(ws);
    int rc = run_scores(ctx, descs, none, d_pre, nm, plan->score_wg_start.back(), plan->sum_rows, plan->sum_cols, w);
    if (rc) return rc;
    const int64_t maxlen = plan->max_rows > plan->max_cols ? plan->max_rows : plan->max_cols;
    const dim3 g2((unsigned)((maxlen + 255) / 256), (unsigned)na);
    hipLaunchKernelGGL(group_sum_kernel, g2, dim3(256), 0, ctx->stream, descs, nm, plan->sum_rows, w.scores,
                       (const int *)d_mode, (const int *)d_next, (const int *)d_seg, (const int *)d_rep);
    hipLaunchKernelGGL(radix_argsort_kernel, dim3((unsigned)na), dim3(RS_THREADS), 0, ctx->stream, descs, none, nm,
                       plan->sum_rows, w.scores, w.k0, w.k1, w.i0, w.i1, row_perm, col_perm, (const int *)d_mode,
                       (const int *)d_seg);
    hipLaunchKernelGGL(replicate_perm_kernel, g2, dim3(256), 0, ctx->stream, descs, nm, row_perm, col_perm,
                       (const int *)d_mode, (const int *)d_leader, (const int *)d_seg, (const int *)d_rep);
    SBITS_HIP(ctx, hipGetLastError());
    return SBITS_OK;
}

// One launch per class of matrices with equal column count (equal LDS need) and element type.
// The class tables depend on shapes only: built once, kept in the plan, copied per call.
//   slot 3 of the workspace head: members of all classes, class after class
//   slot 4: workgroup prefixes (W), slot 5: workgroup prefixes (S); each class has n_k + 1 entries
int sbits_launch_gather_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                            void *w_re, float *s_re, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    if ((size_t)plan->max_cols * 4 > 160 * 1024) return SBITS_ERR_BAD_SHAPE;
    int rc = gather_attr(ctx);
    if (rc) return rc;
    if (plan->gather_members.empty()) {
        std::vector<int64_t> classes;
        for (int i = 0; i < plan->n_mats; ++i) {
            bool seen = false;
            for (int64_t c : classes) seen = seen || c == plan->cols[i];
            if (!seen) classes.push_back(plan->cols[i]);
        }
        for (int64_t c : classes) {
            sbits_plan::GatherClass gc;
            gc.cols = c;
            gc.first = (int)plan->gather_members.size();
            gc.pre_first = (int)plan->gather_pre_w.size();
            gc.rpw_w = gather_rows_per_wg(c, 2);
            gc.rpw_s = gather_rows_per_wg(c, 4);
            int64_t tw = 0, ts = 0;
            gc.n = 0;
            for (int i = 0; i < plan->n_mats; ++i) {
                if (plan->cols[i] != c) continue;
                plan->gather_members.push_back(i);
                plan->gather_pre_w.push_back((int)tw);
                plan->gather_pre_s.push_back((int)ts);
                tw += (plan->rows[i] + gc.rpw_w - 1) / gc.rpw_w;
                ts += (plan->rows[i] + gc.rpw_s - 1) / gc.rpw_s;
                ++gc.n;
            }
            if (tw > 0x7fffffff || ts > 0x7fffffff) { plan->gather_members.clear(); return SBITS_ERR_BAD_SHAPE; }
            plan->gather_pre_w.push_back((int)tw);
            plan->gather_pre_s.push_back((int)ts);
            plan->gather_classes.push_back(gc);
        }
    }
    int *d_mem = sbits_prefix_ptr(plan, ws, 3);
    int *d_pw = sbits_prefix_ptr(plan, ws, 4);
    int *d_ps = sbits_prefix_ptr(plan, ws, 5);
    SBITS_HIP(ctx, hipMemcpyAsync(d_mem, plan->gather_members.data(), plan->gather_members.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(d_pw, plan->gather_pre_w.data(), plan->gather_pre_w.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipMemcpyAsync(d_ps, plan->gather_pre_s.data(), plan->gather_pre_s.size() * 4,
                                  hipMemcpyHostToDevice, ctx->stream));
    MatDesc none;
    memset(&none, 0, sizeof none);
    const MatDesc *descs = sbits_desc_ptr(ws);
    for (const sbits_plan::GatherClass &gc : plan->gather_classes) {
        if (w_re) {
            const int tot = plan->gather_pre_w[gc.pre_first + gc.n];
            hipLaunchKernelGGL(gather_kernel<uint16_t>, dim3((unsigned)tot), dim3(GA_THREADS),
                               (size_t)gc.rpw_w * gc.cols * 2, ctx->stream, descs, none, d_mem + gc.first,
                               d_pw + gc.pre_first, gc.n, gc.rpw_w, row_perm, col_perm,
                               static_cast<uint16_t *>(w_re));
            SBITS_HIP(ctx, hipGetLastError());
        }
        if (s_re) {
            const int tot = plan->gather_pre_s[gc.pre_first + gc.n];
            hipLaunchKernelGGL(gather_kernel<float>, dim3((unsigned)tot), dim3(GA_THREADS),
                               (size_t)gc.rpw_s * gc.cols * 4, ctx->stream, descs, none, d_mem + gc.first,
                               d_ps + gc.pre_first, gc.n, gc.rpw_s, row_perm, col_perm, s_re);
            SBITS_HIP(ctx, hipGetLastError());
        }
    }
    return SBITS_OK;
}
