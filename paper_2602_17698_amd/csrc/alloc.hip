// Scalable greedy bitwidth search (paper Algorithm 2, relaxed step Eq. 5) on the
// block x bitwidth cost table, run on the device.
//
// Per iteration:
//   gains   : marginal cost change per bit of raising / lowering every block,
//             read off the table at the current levels (Alg. 2 line 5), encoded
//             as 64-bit keys  [ordered value : 32][N-1-index : IB][step bits : 8]
//             so that "larger key" = "earlier in (value, lower index first)".
//   select  : radix descent, 11 bits per pass, over the keys: the longest prefix
//             of the descending order that keeps count <= cnt_max and
//             cumulative step bits <= w_max.  Each pass builds a count/weight
//             histogram of the digits under the decided prefix; the workgroup
//             that finishes last scans the 2048 bins and fixes the next digit.
//   expansion (Alg. 2 lines 6-7)  : top-k raised, capped by the remaining
//             budget and by gain > 0.
//   swap (Alg. 2 lines 9-12)      : top-k/2 raised, bottom-k/2 (outside the
//             raised set) lowered; accepted iff the summed cost change, held in
//             order-independent int64 fixed point, is strictly negative; on
//             rejection k is halved.
// All sums that decide anything are integers, so results do not depend on the
// order in which atomics land.
#include <math.h>
#include <string.h>

#include <vector>

#include "sbits_internal.hpp"

namespace sbits {

constexpr int AL_THREADS = 256;
constexpr int64_t TRACE_CAP = 16384;
#ifndef SEL_DB_BITS
#define SEL_DB_BITS 10                        // (8 .. 12 measured on 426 k blocks: 1.29, 1.19, 1.15, 1.20, 1.48 ms per search)
#endif
constexpr int SEL_DB = SEL_DB_BITS;           // digit bits of the selection's radix descent
constexpr int SEL_BINS = 1 << SEL_DB;
#ifndef SEL_KPT
#define SEL_KPT 16                            // keys per thread of a selection pass ...
#endif
#ifndef SEL_MAXWG
#define SEL_MAXWG 128                         // ... and the most workgroups it uses
#endif

struct SelJob {
    unsigned long long prefix;     // decided high digits, right aligned
    long long cnt_above, w_above;  // totals of the keys above the current bucket
    long long cnt_max, w_max;
    unsigned long long key_min;    // keys below are never selected (0 = ineligible)
    unsigned long long tau;        // result: selected <=> key >= tau
    long long n_sel, w_sel;
    int resolved;
    unsigned int ticket;
    unsigned long long hist[SEL_BINS];   // per bucket: (sum of step widths << 32) | number of keys
};

enum { JOB_E = 0, JOB_U = 1, JOB_D = 2, JOB_U2 = 3, N_JOBS = 4 };
enum { MODE_NONE = 0, MODE_EXPAND = 1, MODE_ACCEPT = 2, MODE_REJECT = 3 };

struct AllocHead {
    long long N, T, k, kmin, used;
    long long lossD, gainU;        // fixed-point sums of the current proposal
    long long cost_fixed, bits_check;
    int K, IB, P, shift;
    int iters, max_iters, expansions, swaps_ok, swaps_rej;
    int done, status, mode;
    unsigned int maxc_bits;
    int bits[MAX_CAND];
    long long prop_up, prop_dn, prop_after;   // the single step on caller-supplied estimates: its result
};
struct AllocState : AllocHead {
    SelJob job[N_JOBS];
};
static_assert(sizeof(AllocHead) % 8 == 0, "the jobs follow the head without padding");

// The start state from a kernel argument: no host buffer has to outlive the call, so nothing waits.
// One workgroup: thread 0 writes the head, all threads clear the selection jobs.
__global__ __launch_bounds__(256)
void set_state_kernel(AllocState *st, AllocHead head)
{
    if (threadIdx.x == 0) *static_cast<AllocHead *>(st) = head;
    unsigned int *j = reinterpret_cast<unsigned int *>(st->job);
    for (unsigned i = threadIdx.x; i < sizeof(st->job) / 4; i += blockDim.x) j[i] = 0u;
}

__device__ __forceinline__ unsigned int ord_f32(float f)
{
    const unsigned int u = __float_as_uint(f + 0.0f);          // -0 -> +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ long long fx(float v, int shift)
{
    const double p2 = __longlong_as_double((long long)(1023 + shift) << 52);
    return __double2ll_rn((double)v * p2);
}

// ---- initialisation -------------------------------------------------------------
__global__ void max_cost_kernel(const float *__restrict__ cost, long long n, AllocState *st)
{
    unsigned int mx = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        const float v = cost[i];
        if (v > 0.0f) mx = max(mx, __float_as_uint(v));
    }
    for (int off = 32; off; off >>= 1) mx = max(mx, (unsigned int)__shfl_xor((int)mx, off));
    // one atomic per workgroup: thousands of them on one address take longer than the reads
    __shared__ unsigned int wmx[AL_THREADS / 64];
    if ((threadIdx.x & 63) == 0) wmx[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) mx = max(mx, wmx[w]);
        if (mx) atomicMax(&st->maxc_bits, mx);
    }
}

__global__ void init_state_kernel(AllocState *st, int ceil_log2_n)
{
    const unsigned int b = st->maxc_bits;
    int shift = 0;
    if (b) {
        const int e = (int)(b >> 23);
        const int ilog = e ? e - 127 : (31 - __clz((int)(b & 0x7fffffu))) - 149;
        shift = 61 - ceil_log2_n - (ilog + 1);
    }
    st->shift = shift;
}

__global__ void fill_level_kernel(uint8_t *level, long long n, uint8_t v)
{
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x)
        level[i] = v;
}

// ---- gains ------------------------------------------------------------------------
__device__ void job_reset(SelJob *j, long long cnt_max, long long w_max, unsigned long long key_min)
{
    j->prefix = 0; j->cnt_above = 0; j->w_above = 0;
    j->cnt_max = cnt_max; j->w_max = w_max; j->key_min = key_min;
    j->tau = ~0ull; j->n_sel = 0; j->w_sel = 0; j->resolved = 0;
}

__global__ __launch_bounds__(AL_THREADS)
void gains_kernel(AllocState *st, const float *__restrict__ cost, const uint8_t *__restrict__ level,
                  unsigned long long *__restrict__ keyU, unsigned long long *__restrict__ keyD)
{
    const long long N = st->N;
    const int K = st->K, IB = st->IB;
    int bits[MAX_CAND];
#pragma unroll
    for (int c = 0; c < MAX_CAND; ++c) bits[c] = st->bits[c];
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x) {
        const int l = level[i];
        const float *c = cost + i * K;
        const float cl = c[l];
        const unsigned long long low = (unsigned long long)(N - 1 - i) << 8;
        unsigned long long ku = 0, kd = 0;
        if (l < K - 1) {
            const int step = bits[l + 1] - bits[l];
            const float g = (cl - c[l + 1]) / (float)step;
            ku = ((unsigned long long)ord_f32(g) << (IB + 8)) | low | (unsigned)step;
        }
        if (l > 0) {
            const int step = bits[l] - bits[l - 1];
            const float g = (c[l - 1] - cl) / (float)step;
            kd = ((unsigned long long)(~ord_f32(g)) << (IB + 8)) | low | (unsigned)step;
        }
        keyU[i] = ku;
        keyD[i] = kd;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const long long slack = st->T - st->used;
        long long h = st->k / 2;
        if (h < 1) h = 1;
        const unsigned long long key_pos = (unsigned long long)0x80000001u << (IB + 8);  // value > +0
        job_reset(&st->job[JOB_E], st->k, slack, key_pos);
        job_reset(&st->job[JOB_U], h, 0x7fffffffffffffffll, 1);
        job_reset(&st->job[JOB_D], h, 0x7fffffffffffffffll, 1);
        st->mode = MODE_NONE;
        st->lossD = 0;
        st->gainU = 0;
    }
}

// ---- one radix-descent pass ---------------------------------------------------------
// excl != null: keys whose partner key excl[i] >= st->job[excl_job].tau are skipped.
__global__ __launch_bounds__(AL_THREADS)
void select_pass_kernel(AllocState *st, int job_id, const unsigned long long *__restrict__ keys,
                        const unsigned long long *__restrict__ excl, int excl_job, int pass)
{
    SelJob *job = &st->job[job_id];
    if (job->resolved) return;                                   // uniform over the grid
    // count and width sum of a bucket share one 64-bit word (count low, widths high; neither can
    // reach 2^32: at most 2^24 keys of width <= 255): one LDS atomic per key instead of two
    __shared__ unsigned long long h64[SEL_BINS];
    unsigned int *const hc = reinterpret_cast<unsigned int *>(h64), *const hw = hc + SEL_BINS;   // the last workgroup's view, later
    __shared__ long long gcnt[AL_THREADS], gwgt[AL_THREADS];
    __shared__ bool is_last;
    for (int b = threadIdx.x; b < SEL_BINS; b += AL_THREADS) h64[b] = 0ull;
    __syncthreads();
    const long long N = st->N;
    const int P = st->P;
    const unsigned long long prefix = job->prefix, key_min = job->key_min;
    const unsigned long long excl_tau = excl ? st->job[excl_job].tau : 0;
    // Digits are cut from the TOP of the 32 + IB significant bits (the last one may be narrower): the
    // first pass then already splits on 11 bits of the value instead of on the few bits that a
    // bottom-aligned cut leaves at the top, and a selection whose boundary bucket holds one key is
    // resolved a pass earlier.
    const int TB = 32 + st->IB;
    const int sh_prefix = TB - SEL_DB * pass;
    const int sh_digit = sh_prefix > SEL_DB ? sh_prefix - SEL_DB : 0;
    const int width = sh_prefix - sh_digit;
    const unsigned int dmask = (1u << width) - 1u;
    const long long stride = (long long)gridDim.x * blockDim.x;
    // all of a thread's keys are requested at once (SEL_KPT loads in flight: one memory latency per pass)
    for (long long i0 = (long long)blockIdx.x * blockDim.x + threadIdx.x; i0 < N; i0 += SEL_KPT * stride) {
        unsigned long long key[SEL_KPT], ex[SEL_KPT];
#pragma unroll
        for (int u = 0; u < SEL_KPT; ++u) {
            const long long i = i0 + u * stride;
            key[u] = i < N ? keys[i] : 0ull;
            ex[u] = (excl && i < N) ? excl[i] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < SEL_KPT; ++u) {
            if (key[u] < key_min) continue;                      // also drops the padding (key 0)
            if (excl && ex[u] >= excl_tau) continue;
            const unsigned long long s = key[u] >> 8;
            const unsigned long long hi = sh_prefix >= 64 ? 0ull : (s >> sh_prefix);
            if (hi != prefix) continue;
            const unsigned int d = (unsigned int)(s >> sh_digit) & dmask;
            atomicAdd(&h64[d], ((key[u] & 255ull) << 32) | 1ull);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < SEL_BINS; b += AL_THREADS)
        if (h64[b]) atomicAdd(&job->hist[b], h64[b]);
    // Everything the workgroups exchange goes through device-scope atomics, which are performed at the
    // point of coherence: waiting for their acknowledgement (vmcnt) orders them before the ticket.  A
    // release fence would also write the L2 back, which costs more than the rest of the pass.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int t = atomicAdd(&job->ticket, 1u);
        is_last = (t == gridDim.x - 1);
    }
    __syncthreads();
    if (!is_last) return;
    // the last workgroup: read the finished histogram, clear it for the next pass; thread t owns
    // the SEL_BINS/256 consecutive bins [t*G, (t+1)*G)
    constexpr int G = SEL_BINS / AL_THREADS;
    long long gc = 0, gw = 0;
    unsigned long long got[G];
#pragma unroll
    for (int j = 0; j < G; ++j)
        got[j] = __hip_atomic_exchange(&job->hist[threadIdx.x * G + j], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // (every thread read its part of h64 before the barriers above: it can be reused as hc / hw)
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int b = threadIdx.x * G + j;
        hc[b] = (unsigned int)got[j];
        hw[b] = (unsigned int)(got[j] >> 32);
        gc += hc[b]; gw += hw[b];
    }
    // suffix sums over the groups (descending order = from the last group down): group t fits whole,
    // given that everything above it does, iff the sums down to t stay in bounds; the sums grow
    // downwards, so the groups that fit are the top ones
    __shared__ int first_fail;
    const int t = threadIdx.x;
    gcnt[t] = gc; gwgt[t] = gw;
    if (t == 0) first_fail = -1;
    __syncthreads();
    for (int off = 1; off < AL_THREADS; off <<= 1) {
        const long long ac = t + off < AL_THREADS ? gcnt[t + off] : 0;
        const long long aw = t + off < AL_THREADS ? gwgt[t + off] : 0;
        __syncthreads();
        gcnt[t] += ac; gwgt[t] += aw;
        __syncthreads();
    }
    {
        const long long c0 = job->cnt_above, w0 = job->w_above;
        if (gc && !(c0 + gcnt[t] <= job->cnt_max && w0 + gwgt[t] <= job->w_max)) atomicMax(&first_fail, t);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        job->ticket = 0;
        long long c = job->cnt_above, w = job->w_above;
        const long long cmax = job->cnt_max, wmax = job->w_max;
        int boundary = -1;
        long long boundary_cnt = 0;
        const int g = first_fail;
        if (g >= 0) {
            if (g + 1 < AL_THREADS) { c += gcnt[g + 1]; w += gwgt[g + 1]; }
            // bin by bin inside the first group that does not fit whole
            for (int b = g * G + G - 1; b >= g * G; --b) {
                const long long bc = hc[b], bw = hw[b];
                if (!bc) continue;
                if (c + bc <= cmax && w + bw <= wmax) { c += bc; w += bw; }
                else { boundary = b; boundary_cnt = bc; break; }
            }
        } else {
            c += gcnt[0]; w += gwgt[0];
        }
        if (boundary < 0) {
            // every key under the prefix fits: the selection ends at the bucket's lower edge
            unsigned long long lo = sh_prefix >= 56 ? 0ull : ((prefix << sh_prefix) << 8);
            job->tau = lo > key_min ? lo : key_min;
            job->n_sel = c; job->w_sel = w; job->resolved = 1;
        } else {
            const unsigned long long np = (prefix << width) | (unsigned long long)boundary;
            job->cnt_above = c; job->w_above = w;
            if (pass == P - 1 || boundary_cnt == 1) {
                // a single key that does not fit (its remaining digits do not matter): select the
                // keys strictly above its bucket
                job->tau = ((np + 1) << sh_digit) << 8;
                job->n_sel = c; job->w_sel = w; job->resolved = 1;
            } else {
                job->prefix = np;
            }
        }
    }
}

// ---- expansion ----------------------------------------------------------------------
__device__ void trace_write(sbits_trace *tr, int it, int kind, long long k, long long n_up, long long n_dn,
                            long long p_up, long long p_dn, long long before, long long after, long long delta)
{
    if (it >= TRACE_CAP) return;
    sbits_trace &t = tr[it];
    t.kind = kind; t.pad_ = 0; t.k = k; t.n_up = n_up; t.n_dn = n_dn; t.p_up = p_up; t.p_dn = p_dn;
    t.bits_before = before; t.bits_after = after; t.delta_fixed = delta;
}

__device__ void finish_iteration(AllocState *st)
{
    st->iters++;
    if (st->k < st->kmin) { st->done = 1; }
    else if (st->iters >= st->max_iters) { st->done = 1; st->status = SBITS_ERR_MAX_ITERS; }
}

__global__ void decide_expand_kernel(AllocState *st, sbits_trace *tr)
{
    const SelJob &e = st->job[JOB_E];
    if (st->T - st->used > 0 && e.n_sel > 0) {
        st->mode = MODE_EXPAND;
        trace_write(tr, st->iters, 0, st->k, e.n_sel, 0, e.n_sel, 0, st->used, st->used + e.w_sel, 0);
        st->used += e.w_sel;
        st->expansions++;
        finish_iteration(st);
    }
}

__global__ __launch_bounds__(AL_THREADS)
void apply_expand_kernel(const AllocState *st, const unsigned long long *__restrict__ keyU,
                         uint8_t *__restrict__ level)
{
    if (st->mode != MODE_EXPAND) return;
    const unsigned long long tau = st->job[JOB_E].tau;
    const long long N = st->N;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x)
        if (keyU[i] >= tau) level[i] = level[i] + 1;
}

// ---- swap -----------------------------------------------------------------------------
// after U and D are known: the raised set is the prefix of U that fits slack + freed bits
__global__ void prep_u2_kernel(AllocState *st)
{
    if (st->mode == MODE_EXPAND) return;          // (single step: the swap jobs were closed by the expansion)
    const SelJob &u = st->job[JOB_U];
    const SelJob &d = st->job[JOB_D];
    long long h = st->k / 2;
    if (h < 1) h = 1;
    const long long w_max = (st->T - st->used) + d.w_sel;
    SelJob *j = &st->job[JOB_U2];
    job_reset(j, h, w_max, 1);
    if (u.w_sel <= w_max) {           // all of U fits
        j->tau = u.tau; j->n_sel = u.n_sel; j->w_sel = u.w_sel; j->resolved = 1;
    }
}

__global__ __launch_bounds__(AL_THREADS)
void eval_swap_kernel(AllocState *st, const float *__restrict__ cost, const uint8_t *__restrict__ level,
                      const unsigned long long *__restrict__ keyU, const unsigned long long *__restrict__ keyD)
{
    __shared__ long long sl[AL_THREADS / 64], sg[AL_THREADS / 64];
    const long long N = st->N;
    const int K = st->K, shift = st->shift;
    const unsigned long long tauU = st->job[JOB_U].tau, tauD = st->job[JOB_D].tau, tauU2 = st->job[JOB_U2].tau;
    long long loss = 0, gain = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x) {
        const unsigned long long ku = keyU[i], kd = keyD[i];
        const bool up = ku >= tauU2;
        const bool dn = kd >= tauD && !(ku >= tauU);
        if (up || dn) {
            const int l = level[i];
            const float *c = cost + i * K;
            if (up) gain += fx(c[l] - c[l + 1], shift);
            if (dn) loss += fx(c[l - 1] - c[l], shift);
        }
    }
    for (int off = 32; off; off >>= 1) {
        loss += __shfl_xor(loss, off);
        gain += __shfl_xor(gain, off);
    }
    const int wv = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sl[wv] = loss; sg[wv] = gain; }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long a = 0, b = 0;
        for (int w = 0; w < AL_THREADS / 64; ++w) { a += sl[w]; b += sg[w]; }
        if (a) atomicAdd((unsigned long long *)&st->lossD, (unsigned long long)a);
        if (b) atomicAdd((unsigned long long *)&st->gainU, (unsigned long long)b);
    }
}

__global__ void decide_swap_kernel(AllocState *st, sbits_trace *tr)
{
    const SelJob &u2 = st->job[JOB_U2];
    const SelJob &d = st->job[JOB_D];
    const long long delta = st->lossD - st->gainU;
    if (u2.n_sel > 0 && d.n_sel > 0 && delta < 0) {
        st->mode = MODE_ACCEPT;
        trace_write(tr, st->iters, 1, st->k, u2.n_sel, d.n_sel, u2.n_sel, d.n_sel, st->used,
                    st->used + u2.w_sel - d.w_sel, delta);
        st->used += u2.w_sel - d.w_sel;
        st->swaps_ok++;
    } else {
        st->mode = MODE_REJECT;
        trace_write(tr, st->iters, 2, st->k, 0, 0, u2.n_sel, d.n_sel, st->used, st->used, delta);
        st->k = st->k / 2;
        st->swaps_rej++;
    }
    finish_iteration(st);
}

__global__ __launch_bounds__(AL_THREADS)
void apply_swap_kernel(const AllocState *st, const unsigned long long *__restrict__ keyU,
                       const unsigned long long *__restrict__ keyD, uint8_t *__restrict__ level)
{
    if (st->mode != MODE_ACCEPT) return;
    const unsigned long long tauU = st->job[JOB_U].tau, tauD = st->job[JOB_D].tau, tauU2 = st->job[JOB_U2].tau;
    const long long N = st->N;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x) {
        const unsigned long long ku = keyU[i], kd = keyD[i];
        if (ku >= tauU2) level[i] = level[i] + 1;
        else if (kd >= tauD && !(ku >= tauU)) level[i] = level[i] - 1;
    }
}

// ---- a single step on caller-supplied estimates (the paper's own loop: s_up / s_down are
// re-estimated from a fresh gradient every iteration, Alg. 2 lines 4-5; the acceptance test of
// lines 11-12 is the caller's, who owns the loss) -------------------------------------------
// keys as in gains_kernel, the values taken as given; the bits in use are summed on the way
__global__ __launch_bounds__(AL_THREADS)
void step_keys_kernel(AllocState *st, const float *__restrict__ s_up, const float *__restrict__ s_down,
                      const uint8_t *__restrict__ level, unsigned long long *__restrict__ keyU,
                      unsigned long long *__restrict__ keyD)
{
    __shared__ long long su[AL_THREADS / 64];
    const long long N = st->N;
    const int K = st->K, IB = st->IB;
    int bits[MAX_CAND];
#pragma unroll
    for (int c = 0; c < MAX_CAND; ++c) bits[c] = st->bits[c];
    long long used = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x) {
        const int l = min((int)level[i], K - 1);
        used += bits[l];
        const unsigned long long low = (unsigned long long)(N - 1 - i) << 8;
        unsigned long long ku = 0, kd = 0;
        if (l < K - 1)
            ku = ((unsigned long long)ord_f32(s_up[i]) << (IB + 8)) | low | (unsigned)(bits[l + 1] - bits[l]);
        if (l > 0)
            kd = ((unsigned long long)(~ord_f32(s_down[i])) << (IB + 8)) | low | (unsigned)(bits[l] - bits[l - 1]);
        keyU[i] = ku;
        keyD[i] = kd;
    }
    for (int off = 32; off; off >>= 1) used += __shfl_xor(used, off);
    if ((threadIdx.x & 63) == 0) su[threadIdx.x >> 6] = used;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long a = 0;
        for (int w = 0; w < AL_THREADS / 64; ++w) a += su[w];
        atomicAdd((unsigned long long *)&st->used, (unsigned long long)a);
    }
}

__global__ void step_jobs_kernel(AllocState *st)
{
    const long long slack = st->T - st->used;
    long long h = st->k / 2;
    if (h < 1) h = 1;
    const unsigned long long key_pos = (unsigned long long)0x80000001u << (st->IB + 8);  // value > +0
    job_reset(&st->job[JOB_E], st->k, slack > 0 ? slack : 0, key_pos);
    job_reset(&st->job[JOB_U], h, 0x7fffffffffffffffll, 1);
    job_reset(&st->job[JOB_D], h, 0x7fffffffffffffffll, 1);
    job_reset(&st->job[JOB_U2], h, 0, 1);
    st->mode = MODE_NONE;
    st->prop_up = st->prop_dn = 0;
    st->prop_after = st->used;
}

// after the expansion's selection: an expansion closes the swap's jobs (their passes return at once)
__global__ void step_decide_expand_kernel(AllocState *st)
{
    const SelJob &e = st->job[JOB_E];
    if (st->T - st->used > 0 && e.n_sel > 0) {
        st->mode = MODE_EXPAND;
        st->prop_up = e.n_sel;
        st->prop_after = st->used + e.w_sel;
        st->job[JOB_U].resolved = st->job[JOB_D].resolved = st->job[JOB_U2].resolved = 1;
    }
}

__global__ void step_decide_swap_kernel(AllocState *st)
{
    if (st->mode == MODE_EXPAND) return;
    const SelJob &u2 = st->job[JOB_U2];
    const SelJob &d = st->job[JOB_D];
    if (u2.n_sel > 0 && d.n_sel > 0) {
        st->mode = MODE_ACCEPT;                    // a proposal: the caller accepts or rejects it
        st->prop_up = u2.n_sel;
        st->prop_dn = d.n_sel;
        st->prop_after = st->used + u2.w_sel - d.w_sel;
    }
}

__global__ __launch_bounds__(AL_THREADS)
void step_apply_kernel(const AllocState *st, const unsigned long long *__restrict__ keyU,
                       const unsigned long long *__restrict__ keyD, const uint8_t *__restrict__ level_in,
                       uint8_t *__restrict__ level_out)
{
    const int mode = st->mode;
    const unsigned long long tauE = st->job[JOB_E].tau;
    const unsigned long long tauU = st->job[JOB_U].tau, tauD = st->job[JOB_D].tau, tauU2 = st->job[JOB_U2].tau;
    const long long N = st->N;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x) {
        const unsigned long long ku = keyU[i], kd = keyD[i];
        int l = level_in[i];
        if (mode == MODE_EXPAND) {
            if (ku >= tauE) ++l;
        } else if (mode == MODE_ACCEPT) {
            if (ku >= tauU2) ++l;
            else if (kd >= tauD && !(ku >= tauU)) --l;
        }
        level_out[i] = (uint8_t)l;
    }
}

// ---- final statistics ---------------------------------------------------------------------
__global__ __launch_bounds__(AL_THREADS)
void final_stats_kernel(AllocState *st, const float *__restrict__ cost, const uint8_t *__restrict__ level)
{
    __shared__ long long sa[AL_THREADS / 64], sb[AL_THREADS / 64];
    const long long N = st->N;
    const int K = st->K, shift = st->shift;
    long long cf = 0, bu = 0;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (long long)gridDim.x * blockDim.x) {
        const int l = level[i];
        cf += fx(cost[i * K + l], shift);
        bu += st->bits[l];
    }
    for (int off = 32; off; off >>= 1) { cf += __shfl_xor(cf, off); bu += __shfl_xor(bu, off); }
    const int wv = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sa[wv] = cf; sb[wv] = bu; }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long a = 0, b = 0;
        for (int w = 0; w < AL_THREADS / 64; ++w) { a += sa[w]; b += sb[w]; }
        atomicAdd((unsigned long long *)&st->cost_fixed, (unsigned long long)a);
        atomicAdd((unsigned long long *)&st->bits_check, (unsigned long long)b);
    }
}

static int ceil_log2_ll(long long v) { int p = 0; while ((1ll << p) < v) ++p; return p; }

}  // namespace sbits

using namespace sbits;

// workspace: AllocState | keyU [N] | keyD [N] | trace [TRACE_CAP]
size_t sbits_alloc_ws_bytes(int64_t N)
{
    size_t b = sbits_align_up(sizeof(AllocState), 256);
    b += 2 * sbits_align_up((size_t)N * 8, 256);
    b += sbits_align_up((size_t)TRACE_CAP * sizeof(sbits_trace), 256);
    return b;
}

int sbits_run_allocate(sbits_plan *plan, const float *cost, double avg_bits,
                       const sbits_params *prm, uint8_t *level, sbits_stats *host_stats,
                       sbits_trace *host_trace, int64_t trace_cap, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    hipStream_t sm = ctx->stream;
    const int64_t N = plan->N;
    const int K = plan->K;
    if (avg_bits < (double)plan->bits[0]) return SBITS_ERR_INFEASIBLE_BUDGET;

    char *p = static_cast<char *>(ws);
    AllocState *st = reinterpret_cast<AllocState *>(p);
    p += sbits_align_up(sizeof(AllocState), 256);
    unsigned long long *keyU = reinterpret_cast<unsigned long long *>(p);
    p += sbits_align_up((size_t)N * 8, 256);
    unsigned long long *keyD = reinterpret_cast<unsigned long long *>(p);
    p += sbits_align_up((size_t)N * 8, 256);
    sbits_trace *tr = reinterpret_cast<sbits_trace *>(p);

    // the per-iteration read-back lands in page-locked memory: a pageable target makes every
    // copy a staged, blocking one
    if (!ctx->pinned) SBITS_HIP(ctx, hipHostMalloc(&ctx->pinned, SBITS_PINNED_BYTES, hipHostMallocDefault));
    static_assert(sizeof(AllocHead) <= SBITS_PINNED_BYTES, "state head must fit the pinned buffer");
    AllocHead *hp = static_cast<AllocHead *>(ctx->pinned);     // the state's head as read back
    AllocHead h;
    memset(&h, 0, sizeof h);
    h.N = N;
    h.T = (long long)floor(avg_bits * (double)N);
    h.k = (long long)floor(prm->gamma0 * (double)N);
    h.kmin = (long long)floor(prm->gammaT * (double)N);
    if (h.k < 1) h.k = 1;
    if (h.kmin < 1) h.kmin = 1;
    h.K = K;
    h.IB = ceil_log2_ll(N) > 0 ? ceil_log2_ll(N) : 1;
    h.P = (32 + h.IB + SEL_DB - 1) / SEL_DB;
    h.max_iters = prm->max_iters;
    for (int c = 0; c < MAX_CAND; ++c) h.bits[c] = c < K ? plan->bits[c] : plan->bits[K - 1];

    const bool all_max = avg_bits >= (double)plan->bits[K - 1];
    int l0 = 0;
    if (all_max) l0 = K - 1;
    else if (prm->init_mode == 0) {
        const double fb = floor(avg_bits);
        for (int l = 0; l < K; ++l) if ((double)plan->bits[l] <= fb) l0 = l;
    }
    h.used = N * (long long)plan->bits[l0];
    if (all_max) h.done = 1;

    const unsigned grid = (unsigned)((N + AL_THREADS - 1) / AL_THREADS < 1024 ? (N + AL_THREADS - 1) / AL_THREADS : 1024);
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(256), 0, sm, st, h);
    hipLaunchKernelGGL(max_cost_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, cost, (long long)(N * K), st);
    hipLaunchKernelGGL(init_state_kernel, dim3(1), dim3(1), 0, sm, st, ceil_log2_ll(N));
    hipLaunchKernelGGL(fill_level_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, level, (long long)N, (uint8_t)l0);
    SBITS_HIP(ctx, hipGetLastError());

    long long used = h.used;
    bool done = all_max;
    const int P = h.P;
    // the selection passes end in one global atomic per non-empty bin and workgroup: few, fat workgroups
    const unsigned sgrid = (unsigned)((N + AL_THREADS * SEL_KPT - 1) / (AL_THREADS * SEL_KPT) < SEL_MAXWG ? (N + AL_THREADS * SEL_KPT - 1) / (AL_THREADS * SEL_KPT) : SEL_MAXWG);
    if (!ctx->readback) SBITS_HIP(ctx, hipEventCreateWithFlags(&ctx->readback, hipEventDisableTiming));
    constexpr size_t HEAD = sizeof(AllocHead);
    // A read-back ends in an event of its own: the host waits for the event, not for the stream, so the
    // work enqueued behind the read-back keeps the device busy during the host's round trip.
    auto read_back = [&]() -> hipError_t {
        hipError_t e = hipMemcpyAsync(hp, st, HEAD, hipMemcpyDeviceToHost, sm);
        return e != hipSuccess ? e : hipEventRecord(ctx->readback, sm);
    };
    auto wait_state = [&]() -> hipError_t {
        hipError_t e = hipEventSynchronize(ctx->readback);
        if (e == hipSuccess) memcpy(&h, hp, HEAD);
        return e;
    };
    auto launch_gains = [&]() {
        hipLaunchKernelGGL(gains_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, st, cost, level, keyU, keyD);
    };
    // One expansion attempt: its selection, decision and application, the read-back of the state, and the
    // keys of whatever iteration comes next (every iteration starts with them, so they are requested
    // before the host knows the outcome: computed once too often after the last iteration, and after an
    // attempt that raised nothing, with the same values).
    auto enqueue_expand = [&]() -> hipError_t {
        for (int ps = 0; ps < P; ++ps)
            hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_E, keyU,
                               (const unsigned long long *)nullptr, 0, ps);
        hipLaunchKernelGGL(decide_expand_kernel, dim3(1), dim3(1), 0, sm, st, tr);
        hipLaunchKernelGGL(apply_expand_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, st, keyU, level);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = read_back();
        launch_gains();
        return e;
    };

    if (!done) launch_gains();
    while (!done) {
        bool expanded = false;
        if (h.T - used > 0) {
            SBITS_HIP(ctx, enqueue_expand());
            SBITS_HIP(ctx, wait_state());
            expanded = h.mode == MODE_EXPAND;
        }
        if (!expanded) {
            for (int ps = 0; ps < P; ++ps)
                hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_U, keyU,
                                   (const unsigned long long *)nullptr, 0, ps);
            for (int ps = 0; ps < P; ++ps)
                hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_D, keyD,
                                   (const unsigned long long *)keyU, (int)JOB_U, ps);
            hipLaunchKernelGGL(prep_u2_kernel, dim3(1), dim3(1), 0, sm, st);
            for (int ps = 0; ps < P; ++ps)
                hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_U2, keyU,
                                   (const unsigned long long *)nullptr, 0, ps);
            hipLaunchKernelGGL(eval_swap_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, st, cost, level, keyU, keyD);
            hipLaunchKernelGGL(decide_swap_kernel, dim3(1), dim3(1), 0, sm, st, tr);
            hipLaunchKernelGGL(apply_swap_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, st, keyU, keyD, level);
            SBITS_HIP(ctx, hipGetLastError());
            SBITS_HIP(ctx, read_back());
            launch_gains();
            SBITS_HIP(ctx, wait_state());
        }
        used = h.used;
        done = h.done != 0;
    }

    hipLaunchKernelGGL(final_stats_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, st, cost, level);
    SBITS_HIP(ctx, hipGetLastError());
    SBITS_HIP(ctx, hipMemcpyAsync(hp, st, sizeof(AllocHead), hipMemcpyDeviceToHost, sm));
    SBITS_HIP(ctx, hipStreamSynchronize(sm));
    memcpy(&h, hp, sizeof(AllocHead));
    if (host_stats) {
        host_stats->iters = h.iters; host_stats->expansions = h.expansions;
        host_stats->swaps_ok = h.swaps_ok; host_stats->swaps_rej = h.swaps_rej;
        host_stats->k_final = h.k; host_stats->bits_used = h.bits_check; host_stats->bits_budget = h.T;
        host_stats->cost_fixed = h.cost_fixed; host_stats->cost_shift = h.shift; host_stats->pad_ = 0;
    }
    if (host_trace && trace_cap > 0 && h.iters > 0) {
        int64_t nrec = h.iters < trace_cap ? h.iters : trace_cap;
        if (nrec > TRACE_CAP) nrec = TRACE_CAP;
        SBITS_HIP(ctx, hipMemcpyAsync(host_trace, tr, (size_t)nrec * sizeof(sbits_trace), hipMemcpyDeviceToHost, sm));
        SBITS_HIP(ctx, hipStreamSynchronize(sm));
    }
    if (h.bits_check != h.used) return SBITS_ERR_INTERNAL;      // the loop's running total and a recount must agree
    return h.status;
}


// One step of Algorithm 2 on caller-supplied estimates.  Workspace as sbits_run_allocate.
int sbits_run_propose(sbits_plan *plan, const float *s_up, const float *s_down, const uint8_t *level_in,
                      double avg_bits, int64_t k, uint8_t *level_out, sbits_proposal *host_out, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    hipStream_t sm = ctx->stream;
    const int64_t N = plan->N;
    const int K = plan->K;

    char *p = static_cast<char *>(ws);
    AllocState *st = reinterpret_cast<AllocState *>(p);
    p += sbits_align_up(sizeof(AllocState), 256);
    unsigned long long *keyU = reinterpret_cast<unsigned long long *>(p);
    p += sbits_align_up((size_t)N * 8, 256);
    unsigned long long *keyD = reinterpret_cast<unsigned long long *>(p);

    if (!ctx->pinned) SBITS_HIP(ctx, hipHostMalloc(&ctx->pinned, SBITS_PINNED_BYTES, hipHostMallocDefault));
    AllocHead *hp = static_cast<AllocHead *>(ctx->pinned);
    AllocHead h;
    memset(&h, 0, sizeof h);
    h.N = N;
    h.T = (long long)floor(avg_bits * (double)N);
    h.k = k;
    h.K = K;
    h.IB = ceil_log2_ll(N) > 0 ? ceil_log2_ll(N) : 1;
    h.P = (32 + h.IB + SEL_DB - 1) / SEL_DB;
    for (int c = 0; c < MAX_CAND; ++c) h.bits[c] = c < K ? plan->bits[c] : plan->bits[K - 1];
    // the start state travels as a kernel argument: nothing to keep alive, nothing to wait for
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(256), 0, sm, st, h);

    const unsigned grid = (unsigned)((N + AL_THREADS - 1) / AL_THREADS < 1024 ? (N + AL_THREADS - 1) / AL_THREADS : 1024);
    const unsigned sgrid = (unsigned)((N + AL_THREADS * SEL_KPT - 1) / (AL_THREADS * SEL_KPT) < SEL_MAXWG ? (N + AL_THREADS * SEL_KPT - 1) / (AL_THREADS * SEL_KPT) : SEL_MAXWG);
    const int P = h.P;
    const unsigned long long *none = nullptr;
    hipLaunchKernelGGL(step_keys_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, st, s_up, s_down, level_in, keyU, keyD);
    hipLaunchKernelGGL(step_jobs_kernel, dim3(1), dim3(1), 0, sm, st);
    for (int ps = 0; ps < P; ++ps)
        hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_E, keyU, none, 0, ps);
    hipLaunchKernelGGL(step_decide_expand_kernel, dim3(1), dim3(1), 0, sm, st);
    for (int ps = 0; ps < P; ++ps)
        hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_U, keyU, none, 0, ps);
    for (int ps = 0; ps < P; ++ps)
        hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_D, keyD,
                           (const unsigned long long *)keyU, (int)JOB_U, ps);
    hipLaunchKernelGGL(prep_u2_kernel, dim3(1), dim3(1), 0, sm, st);
    for (int ps = 0; ps < P; ++ps)
        hipLaunchKernelGGL(select_pass_kernel, dim3(sgrid), dim3(AL_THREADS), 0, sm, st, (int)JOB_U2, keyU, none, 0, ps);
    hipLaunchKernelGGL(step_decide_swap_kernel, dim3(1), dim3(1), 0, sm, st);
    hipLaunchKernelGGL(step_apply_kernel, dim3(grid), dim3(AL_THREADS), 0, sm, (const AllocState *)st,
                       (const unsigned long long *)keyU, (const unsigned long long *)keyD, level_in, level_out);
    SBITS_HIP(ctx, hipGetLastError());
    if (host_out) {
        static_assert(sizeof(AllocHead) <= SBITS_PINNED_BYTES, "state head must fit the pinned buffer");
        SBITS_HIP(ctx, hipMemcpyAsync(hp, st, sizeof(AllocHead), hipMemcpyDeviceToHost, sm));
        SBITS_HIP(ctx, hipStreamSynchronize(sm));
        host_out->kind = hp->mode == MODE_EXPAND ? 1 : hp->mode == MODE_ACCEPT ? 2 : 0;
        host_out->pad_ = 0;
        host_out->n_up = hp->prop_up;
        host_out->n_dn = hp->prop_dn;
        host_out->bits_before = hp->used;
        host_out->bits_after = hp->prop_after;
        host_out->bits_budget = hp->T;
    }
    return SBITS_OK;
}
