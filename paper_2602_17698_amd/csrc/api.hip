// C-ABI entry points of libscalebits: argument validation, plan bookkeeping and
// the sequencing of the kernel stages.  No arithmetic of the method lives here.
#include <math.h>
#include <string.h>

#include <new>

#include "sbits_internal.hpp"

static bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

extern "C" {

const char *sbits_strerror(int status)
{
    switch (status) {
    case SBITS_OK: return "ok";
    case SBITS_ERR_INVALID_ARG: return "invalid argument";
    case SBITS_ERR_BAD_SHAPE: return "unsupported or non-dividing block shape";
    case SBITS_ERR_BAD_BITWIDTHS: return "bad candidate bitwidth list";
    case SBITS_ERR_INFEASIBLE_BUDGET: return "budget below the smallest candidate bitwidth";
    case SBITS_ERR_WORKSPACE: return "workspace (or fixed scratch) too small";
    case SBITS_ERR_MAX_ITERS: return "search stopped by max_iters";
    case SBITS_ERR_HIP: return "HIP runtime error";
    case SBITS_ERR_UNIMPLEMENTED: return "not implemented";
    case SBITS_ERR_CAPACITY: return "output buffer too small";
    case SBITS_ERR_INTERNAL: return "internal consistency check failed";
    }
    return "unknown status";
}

int sbits_create(sbits_ctx **out, int device, void *hip_stream)
{
    if (!out || device < -1) return SBITS_ERR_INVALID_ARG;
    sbits_ctx *c = new (std::nothrow) sbits_ctx;
    if (!c) return SBITS_ERR_INVALID_ARG;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->last_hip = 0;
    c->pinned = nullptr;
    c->readback = nullptr;
    c->d16_zero_fill = true;
    if (device >= 0) {
        hipError_t e = hipSetDevice(device);
        if (e != hipSuccess) { c->last_hip = (int)e; delete c; return SBITS_ERR_HIP; }
        const int rc = sbits_offsets_static_setup(c);     // this device's fixed scratch array, looked up once
        if (rc) { delete c; return rc; }
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) { c->last_hip = (int)e; delete c; return SBITS_ERR_HIP; }
        c->d16_zero_fill = strstr(prop.gcnArchName, "sramecc+") != nullptr;
    }
    *out = c;
    return SBITS_OK;
}

int sbits_destroy(sbits_ctx *ctx)
{
    if (!ctx) return SBITS_ERR_INVALID_ARG;
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    if (ctx->readback) (void)hipEventDestroy(ctx->readback);
    delete ctx;
    return SBITS_OK;
}

int sbits_last_hip_error(const sbits_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

int sbits_plan_create(sbits_ctx *ctx, const int64_t *rows, const int64_t *cols, int n_mats,
                      int block_rows, int block_cols, const int32_t *bitwidths, int n_bits,
                      sbits_plan **out)
{
    if (!ctx || !rows || !cols || n_mats <= 0 || !out || !bitwidths) return SBITS_ERR_INVALID_ARG;
    if (n_bits <= 0 || n_bits > sbits::MAX_CAND) return SBITS_ERR_BAD_BITWIDTHS;
    for (int l = 0; l < n_bits; ++l) {
        if (bitwidths[l] < 0 || bitwidths[l] > 8) return SBITS_ERR_BAD_BITWIDTHS;
        if (l && bitwidths[l] <= bitwidths[l - 1]) return SBITS_ERR_BAD_BITWIDTHS;
    }
    if (bitwidths[n_bits - 1] == 0) return SBITS_ERR_BAD_BITWIDTHS;      // "0 bits" alone is no search space
    if (!is_pow2(block_rows) || !is_pow2(block_cols) || block_rows < 8 || block_rows > 1024 ||
        block_cols < 8 || block_cols > 512)
        return SBITS_ERR_BAD_SHAPE;
    sbits_plan *p = new (std::nothrow) sbits_plan;
    if (!p) return SBITS_ERR_INVALID_ARG;
    p->ctx = ctx;
    p->n_mats = n_mats;
    p->m = block_rows;
    p->n = block_cols;
    p->K = n_bits;
    for (int l = 0; l < sbits::MAX_CAND; ++l) p->bits[l] = l < n_bits ? bitwidths[l] : 0;
    p->N = 0;
    p->max_rows = p->max_cols = 0;
    p->sum_rows = p->sum_cols = p->sum_elems = 0;
    p->sum_rowpart = p->sum_colpart = 0;
    int64_t score_wgs = 0;
    for (int i = 0; i < n_mats; ++i) {
        if (rows[i] <= 0 || cols[i] <= 0 || rows[i] % block_rows || cols[i] % block_cols ||
            rows[i] > 32768 || cols[i] > 32768) {
            delete p;
            return SBITS_ERR_BAD_SHAPE;
        }
        p->rows.push_back(rows[i]);
        p->cols.push_back(cols[i]);
        p->base.push_back(p->N);
        sbits::MatDesc d;
        memset(&d, 0, sizeof d);
        d.rows = rows[i]; d.cols = cols[i]; d.ld_w = d.ld_s = cols[i];
        d.elem_off = p->sum_elems; d.block_base = p->N;
        d.row_off = p->sum_rows; d.col_off = p->sum_cols;
        d.nbr = (int)(rows[i] / block_rows); d.nbc = (int)(cols[i] / block_cols);
        sbits_score_geometry(rows[i], cols[i], &d.nseg, &d.nband);
        d.rowpart_off = p->sum_rowpart; d.colpart_off = p->sum_colpart;
        p->sum_rowpart += rows[i] * d.nseg; p->sum_colpart += (int64_t)d.nband * cols[i];
        p->score_wg_start.push_back((int)score_wgs);
        score_wgs += sbits_score_wgs(d.nseg, d.nband);
        p->descs.push_back(d);
        p->sum_rows += rows[i]; p->sum_cols += cols[i]; p->sum_elems += rows[i] * cols[i];
        p->N += (rows[i] / block_rows) * (cols[i] / block_cols);
        if (rows[i] > p->max_rows) p->max_rows = rows[i];
        if (cols[i] > p->max_cols) p->max_cols = cols[i];
    }
    if (p->N > (1ll << 24) || score_wgs > 0x7fffffff) { delete p; return SBITS_ERR_BAD_SHAPE; }   // index field of the selection keys
    p->score_wg_start.push_back((int)score_wgs);
    size_t ws = sbits_reorder_ws_bytes(p->sum_rows + p->sum_cols, p->sum_rowpart, p->sum_colpart);
    const size_t a = sbits_alloc_ws_bytes(p->N), o = sbits_offsets_ws_bytes(p->N);
    if (a > ws) ws = a;
    if (o > ws) ws = o;
    const size_t f = sbits_fused_ws_bytes(p);
    if (f > ws) ws = f;
    const size_t g = sbits_mp_gemm_ws_bytes(p);
    if (g > ws) ws = g;
    p->head_bytes = sbits_desc_bytes(n_mats) + SBITS_N_PREFIX * sbits_prefix_bytes(n_mats);
    p->ws_bytes = p->head_bytes + ws;
    p->ws_given = ~(size_t)0;                        // not declared: not checked
    p->desc_pinned = nullptr;
    *out = p;
    return SBITS_OK;
}

int sbits_plan_destroy(sbits_plan *plan)
{
    if (!plan) return SBITS_ERR_INVALID_ARG;
    if (plan->desc_pinned) {
        for (int i = 0; i < 2; ++i) {
            if (plan->desc_used[i]) (void)hipEventSynchronize(plan->desc_done[i]);   // no copy may still read the buffers
            (void)hipEventDestroy(plan->desc_done[i]);
        }
        (void)hipHostFree(plan->desc_pinned);
    }
    delete plan;
    return SBITS_OK;
}

int64_t sbits_num_blocks(const sbits_plan *plan, int mat)
{
    if (!plan || mat < -1 || mat >= plan->n_mats) return SBITS_ERR_INVALID_ARG;
    if (mat < 0) return plan->N;
    return (plan->rows[mat] / plan->m) * (plan->cols[mat] / plan->n);
}

int64_t sbits_block_base(const sbits_plan *plan, int mat)
{
    if (!plan || mat < 0 || mat >= plan->n_mats) return SBITS_ERR_INVALID_ARG;
    return plan->base[mat];
}

size_t sbits_workspace_bytes(const sbits_plan *plan) { return plan ? plan->ws_bytes : 0; }

int64_t sbits_codes_bytes_bound(const sbits_plan *plan, double avg_bits)
{
    if (!plan || !(avg_bits >= 0)) return SBITS_ERR_INVALID_ARG;
    double b = avg_bits;
    if (b > plan->bits[plan->K - 1]) b = plan->bits[plan->K - 1];
    const int64_t T = (int64_t)floor(b * (double)plan->N);
    return T * ((int64_t)plan->m * plan->n / 8);
}

static int check_matrix(const sbits_plan *plan, int mat, const sbits_matrix *M, bool need_w, bool need_s)
{
    if (!plan || !M || mat < 0 || mat >= plan->n_mats) return SBITS_ERR_INVALID_ARG;
    if (M->rows != plan->rows[mat] || M->cols != plan->cols[mat]) return SBITS_ERR_BAD_SHAPE;
    if (need_w && (!M->w_bf16 || M->ld_w < M->cols || (M->ld_w % 8) || !aligned16(M->w_bf16)))
        return SBITS_ERR_INVALID_ARG;
    if (need_s && (!M->sens || M->ld_s < M->cols || (M->ld_s % 4) || !aligned16(M->sens)))
        return SBITS_ERR_INVALID_ARG;
    return SBITS_OK;
}

static int need_device(const sbits_plan *plan)
{
    if (plan->ctx->device < 0) return SBITS_ERR_HIP;
    return SBITS_OK;
}

}  // extern "C"

// Copies the descriptor table into the workspace head.  mats == nullptr: shapes only.
// The image a copy reads must not change while the copy is pending: the table is built in one of two
// page-locked buffers of the plan, taken in turns; before a buffer is rewritten the host waits for the
// event recorded behind the copy that last read it (two uploads back: as good as always complete).
int sbits_upload_descs(sbits_plan *plan, const sbits_matrix *mats, void *ws)
{
    sbits_ctx *ctx = plan->ctx;
    const size_t bytes = (size_t)plan->n_mats * sizeof(sbits::MatDesc);
    if (!plan->desc_pinned) {
        SBITS_HIP(ctx, hipHostMalloc(&plan->desc_pinned, 2 * bytes, hipHostMallocDefault));
        for (int i = 0; i < 2; ++i) SBITS_HIP(ctx, hipEventCreateWithFlags(&plan->desc_done[i], hipEventDisableTiming));
        plan->desc_turn = 0;
        plan->desc_used[0] = plan->desc_used[1] = false;
    }
    const int t = plan->desc_turn;
    plan->desc_turn ^= 1;
    if (plan->desc_used[t]) SBITS_HIP(ctx, hipEventSynchronize(plan->desc_done[t]));
    sbits::MatDesc *img = reinterpret_cast<sbits::MatDesc *>(static_cast<char *>(plan->desc_pinned) + (size_t)t * bytes);
    for (int i = 0; i < plan->n_mats; ++i) {
        sbits::MatDesc &d = plan->descs[i];
        if (mats) {
            d.w = static_cast<const uint16_t *>(mats[i].w_bf16);
            d.s = mats[i].sens;
            d.ld_w = mats[i].ld_w;
            d.ld_s = mats[i].ld_s;
        } else {
            d.w = nullptr; d.s = nullptr;
        }
        img[i] = d;
    }
    SBITS_HIP(ctx, hipMemcpyAsync(ws, img, bytes, hipMemcpyHostToDevice, ctx->stream));
    SBITS_HIP(ctx, hipEventRecord(plan->desc_done[t], ctx->stream));
    plan->desc_used[t] = true;
    return SBITS_OK;
}

extern "C" {

static bool ws_ok(const void *ws) { return ws && (reinterpret_cast<uintptr_t>(ws) & 255) == 0; }
// the caller's workspace, if its size was declared (sbits_set_workspace_size), holds what the plan needs
static bool ws_fits(const sbits_plan *plan) { return plan->ws_given >= plan->ws_bytes; }

int sbits_set_workspace_size(sbits_plan *plan, size_t bytes)
{
    if (!plan) return SBITS_ERR_INVALID_ARG;
    plan->ws_given = bytes;
    return bytes >= plan->ws_bytes ? SBITS_OK : SBITS_ERR_WORKSPACE;
}

int sbits_channel_scores(sbits_plan *plan, int mat, const sbits_matrix *M, float *row_score,
                         float *col_score, void *ws)
{
    int rc = check_matrix(plan, mat, M, false, true);
    if (rc) return rc;
    if (!row_score || !col_score || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if ((rc = need_device(plan))) return rc;
    return sbits_launch_scores(plan->ctx, M->sens, M->rows, M->cols, M->ld_s, row_score, col_score,
                               sbits_scratch(plan, ws));
}

int sbits_reorder(sbits_plan *plan, int mat, const sbits_matrix *M, int32_t *row_perm,
                  int32_t *col_perm, void *ws)
{
    int rc = check_matrix(plan, mat, M, false, true);
    if (rc) return rc;
    if (!row_perm || !col_perm || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if ((rc = need_device(plan))) return rc;
    return sbits_launch_reorder(plan->ctx, M->sens, M->rows, M->cols, M->ld_s, row_perm, col_perm,
                                sbits_scratch(plan, ws));
}

static int check_all(const sbits_plan *plan, const sbits_matrix *mats, bool need_w, bool need_s)
{
    if (!plan || !mats) return SBITS_ERR_INVALID_ARG;
    for (int i = 0; i < plan->n_mats; ++i) {
        const int rc = check_matrix(plan, i, &mats[i], need_w, need_s);
        if (rc) return rc;
    }
    return SBITS_OK;
}

int sbits_reorder_all(sbits_plan *plan, const sbits_matrix *mats, int32_t *row_perm, int32_t *col_perm, void *ws)
{
    int rc = check_all(plan, mats, false, true);
    if (rc) return rc;
    if (!row_perm || !col_perm || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if ((rc = need_device(plan))) return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    return sbits_launch_reorder_all(plan, row_perm, col_perm, ws);
}

int sbits_reorder_coupled_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_group,
                              const int32_t *col_group, int n_groups, const int32_t *group_segment,
                              const int32_t *row_repeat, const int32_t *col_repeat, int32_t *row_perm,
                              int32_t *col_perm, void *ws)
{
    int rc = check_all(plan, mats, false, true);
    if (rc) return rc;
    if (!row_group || !col_group || n_groups < 0 || !row_perm || !col_perm || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if ((rc = sbits_coupling_tables(plan, row_group, col_group, n_groups, group_segment, row_repeat, col_repeat,
                                    nullptr, nullptr, nullptr, nullptr, nullptr)))
        return rc;
    if ((rc = need_device(plan))) return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    return sbits_launch_reorder_coupled_all(plan, row_group, col_group, n_groups, group_segment, row_repeat,
                                            col_repeat, row_perm, col_perm, ws);
}

int sbits_gather_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                     const int32_t *col_perm, void *w_re_bf16, float *s_re, void *ws)
{
    int rc = check_all(plan, mats, w_re_bf16 != nullptr, s_re != nullptr);
    if (rc) return rc;
    if (!row_perm || !col_perm || (!w_re_bf16 && !s_re) || !aligned16(col_perm) || !aligned16(w_re_bf16) ||
        !aligned16(s_re) || !ws_ok(ws))
        return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if ((rc = need_device(plan))) return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    return sbits_launch_gather_all(plan, row_perm, col_perm, w_re_bf16, s_re, ws);
}

int sbits_gather(sbits_plan *plan, int mat, const sbits_matrix *M, const int32_t *row_perm,
                 const int32_t *col_perm, void *w_out_bf16, float *s_out)
{
    int rc = check_matrix(plan, mat, M, w_out_bf16 != nullptr, s_out != nullptr);
    if (rc) return rc;
    if (!row_perm || !col_perm || (!w_out_bf16 && !s_out) || !aligned16(col_perm) ||
        !aligned16(w_out_bf16) || !aligned16(s_out))
        return SBITS_ERR_INVALID_ARG;
    if (w_out_bf16 == M->w_bf16 || (const void *)s_out == (const void *)M->sens) return SBITS_ERR_INVALID_ARG;
    if ((rc = need_device(plan))) return rc;
    return sbits_launch_gather(plan->ctx, M->w_bf16, M->sens, M->rows, M->cols, M->ld_w, M->ld_s,
                               row_perm, col_perm, w_out_bf16, s_out);
}

int sbits_cost_table(sbits_plan *plan, int mat, const void *w_re_bf16, const float *s_re, float *cost)
{
    if (!plan || mat < 0 || mat >= plan->n_mats || !w_re_bf16 || !s_re || !cost) return SBITS_ERR_INVALID_ARG;
    if (!aligned16(w_re_bf16) || !aligned16(s_re)) return SBITS_ERR_INVALID_ARG;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_launch_cost(plan->ctx, w_re_bf16, s_re, plan->rows[mat], plan->cols[mat], plan->m, plan->n,
                             plan->bits, plan->K, cost + plan->base[mat] * plan->K);
}

int sbits_cost_table_all(sbits_plan *plan, const void *w_re_bf16, const float *s_re, float *cost, void *ws)
{
    if (!plan || !w_re_bf16 || !s_re || !cost || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!aligned16(w_re_bf16) || !aligned16(s_re)) return SBITS_ERR_INVALID_ARG;
    int rc = need_device(plan);
    if (rc) return rc;
    if ((rc = sbits_upload_descs(plan, nullptr, ws))) return rc;
    return sbits_launch_cost_all(plan, w_re_bf16, s_re, cost, ws);
}

int sbits_gather_cost_supported(const sbits_plan *plan) { return plan && sbits_fused_shapes_ok(plan) ? 1 : 0; }

int sbits_gather_cost_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                          const int32_t *col_perm, void *w_re_bf16, float *cost, void *ws)
{
    int rc = check_all(plan, mats, true, true);
    if (rc) return rc;
    if (!row_perm || !col_perm || !cost || !aligned16(col_perm) || !aligned16(w_re_bf16) || !ws_ok(ws))
        return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!sbits_fused_shapes_ok(plan)) return SBITS_ERR_UNIMPLEMENTED;
    if ((rc = need_device(plan))) return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    if (!sbits_fused_layout_ok(plan, true)) return SBITS_ERR_UNIMPLEMENTED;
    return sbits_launch_gather_cost_all(plan, row_perm, col_perm, w_re_bf16, cost, ws);
}

int sbits_surrogates_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                         const int32_t *col_perm, const uint8_t *level, float *s_up, float *s_down, void *ws)
{
    int rc = check_all(plan, mats, true, true);
    if (rc) return rc;
    if (!row_perm || !col_perm || !level || !s_up || !s_down || !aligned16(col_perm) || !ws_ok(ws))
        return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!sbits_fused_all_staged(plan)) return SBITS_ERR_UNIMPLEMENTED;
    if ((rc = need_device(plan))) return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    if (!sbits_fused_layout_ok(plan, true)) return SBITS_ERR_UNIMPLEMENTED;
    return sbits_launch_surrogates_all(plan, row_perm, col_perm, level, s_up, s_down, ws);
}

int sbits_gather_pack_all(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_perm,
                          const int32_t *col_perm, const uint8_t *level, const int64_t *byte_off,
                          uint8_t *codes, float *scale, float *zero, void *ws)
{
    int rc = check_all(plan, mats, true, false);
    if (rc) return rc;
    if (!row_perm || !col_perm || !level || !byte_off || !codes || !scale || !zero || !aligned16(col_perm) ||
        !ws_ok(ws) || (reinterpret_cast<uintptr_t>(codes) & 7) || !aligned16(scale) || !aligned16(zero))
        return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!sbits_fused_shapes_ok(plan)) return SBITS_ERR_UNIMPLEMENTED;
    if ((rc = need_device(plan))) return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    if (!sbits_fused_layout_ok(plan, false)) return SBITS_ERR_UNIMPLEMENTED;
    return sbits_launch_gather_pack_all(plan, row_perm, col_perm, level, byte_off, codes, scale, zero, ws);
}

int sbits_allocate(sbits_plan *plan, const float *cost, double avg_bits, const sbits_params *params,
                   uint8_t *level, sbits_stats *host_stats, sbits_trace *host_trace, int64_t trace_cap,
                   void *ws)
{
    if (!plan || !cost || !params || !level || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!(params->gamma0 >= 0) || !(params->gammaT >= 0) || params->max_iters < 1 ||
        (params->init_mode != 0 && params->init_mode != 1) || !(avg_bits == avg_bits))
        return SBITS_ERR_INVALID_ARG;
    if (avg_bits < (double)plan->bits[0]) return SBITS_ERR_INFEASIBLE_BUDGET;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_run_allocate(plan, cost, avg_bits, params, level, host_stats, host_trace, trace_cap,
                              sbits_scratch(plan, ws));
}

int sbits_propose(sbits_plan *plan, const float *s_up, const float *s_down, const uint8_t *level_in,
                  double avg_bits, int64_t k, uint8_t *level_out, sbits_proposal *host_out, void *ws)
{
    if (!plan || !s_up || !s_down || !level_in || !level_out || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (k < 1 || !(avg_bits == avg_bits)) return SBITS_ERR_INVALID_ARG;
    if (avg_bits < (double)plan->bits[0]) return SBITS_ERR_INFEASIBLE_BUDGET;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_run_propose(plan, s_up, s_down, level_in, avg_bits, k, level_out, host_out, sbits_scratch(plan, ws));
}

int sbits_dequant(sbits_plan *plan, int mat, const uint8_t *level, const int64_t *byte_off, const uint8_t *codes,
                  const float *scale, const float *zero, void *out, int64_t ld_out, int out_bf16)
{
    if (!plan || mat < 0 || mat >= plan->n_mats || !level || !byte_off || !codes || !scale || !zero || !out)
        return SBITS_ERR_INVALID_ARG;
    if (ld_out < plan->cols[mat] || (ld_out % 8) || !aligned16(out) || !aligned16(codes) ||
        (out_bf16 != 0 && out_bf16 != 1))
        return SBITS_ERR_INVALID_ARG;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_launch_dequant(plan, mat, level, byte_off, codes, scale, zero, out, ld_out, out_bf16);
}

int sbits_mp_gemm(sbits_plan *plan, int mat, const void *x_bf16, int64_t ld_x, int batch, const uint8_t *level,
                  const int64_t *byte_off, const uint8_t *codes, const float *scale, const float *zero, float *y,
                  void *ws)
{
    if (!plan || mat < 0 || mat >= plan->n_mats || !x_bf16 || !level || !byte_off || !codes || !scale || !zero ||
        !y || !ws_ok(ws))
        return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (batch < 1 || ld_x < plan->cols[mat] || (ld_x % 8) || !aligned16(x_bf16) || !aligned16(codes))
        return SBITS_ERR_INVALID_ARG;
    if (!sbits_mp_gemm_shapes_ok(plan)) return SBITS_ERR_UNIMPLEMENTED;
    int rc = need_device(plan);
    if (rc) return rc;
    // 32 rows of x per launch (two batch tiles of the kernel); launches share the scratch in stream order
    for (int b0 = 0; b0 < batch; b0 += 32) {
        const int nb = batch - b0 < 32 ? batch - b0 : 32;
        rc = sbits_launch_mp_gemm(plan, mat, static_cast<const uint16_t *>(x_bf16) + (int64_t)b0 * ld_x, ld_x, nb, level,
                                  byte_off, codes, scale, zero, y + (int64_t)b0 * plan->rows[mat],
                                  sbits_scratch(plan, ws));
        if (rc) return rc;
    }
    return SBITS_OK;
}

int sbits_offsets(sbits_plan *plan, const uint8_t *level, int64_t *byte_off, void *ws)
{
    if (!plan || !level || !byte_off || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_launch_offsets(plan->ctx, level, plan->N, plan->m, plan->n, plan->bits, plan->K, byte_off,
                                sbits_scratch(plan, ws));
}

int sbits_offsets_static(sbits_plan *plan, const uint8_t *level, int64_t *byte_off)
{
    if (!plan || !level || !byte_off) return SBITS_ERR_INVALID_ARG;
    if (plan->N > SBITS_OFFSETS_STATIC_MAX_BLOCKS) return SBITS_ERR_WORKSPACE;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_launch_offsets_static(plan->ctx, level, plan->N, plan->m, plan->n, plan->bits, plan->K, byte_off);
}

int sbits_pack(sbits_plan *plan, int mat, const void *w_re_bf16, const uint8_t *level,
               const int64_t *byte_off, uint8_t *codes, float *scale, float *zero)
{
    if (!plan || mat < 0 || mat >= plan->n_mats || !w_re_bf16 || !level || !byte_off || !codes || !scale || !zero)
        return SBITS_ERR_INVALID_ARG;
    if (!aligned16(w_re_bf16) || !aligned16(codes)) return SBITS_ERR_INVALID_ARG;
    int rc = need_device(plan);
    if (rc) return rc;
    return sbits_launch_pack(plan->ctx, w_re_bf16, plan->rows[mat], plan->cols[mat], plan->m, plan->n,
                             plan->bits, plan->K, level, byte_off, plan->base[mat], codes, scale, zero);
}

int sbits_pack_all(sbits_plan *plan, const void *w_re_bf16, const uint8_t *level, const int64_t *byte_off,
                   uint8_t *codes, float *scale, float *zero, void *ws)
{
    if (!plan || !w_re_bf16 || !level || !byte_off || !codes || !scale || !zero || !ws_ok(ws))
        return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!aligned16(w_re_bf16) || !aligned16(codes)) return SBITS_ERR_INVALID_ARG;
    int rc = need_device(plan);
    if (rc) return rc;
    if ((rc = sbits_upload_descs(plan, nullptr, ws))) return rc;
    return sbits_launch_pack_all(plan, w_re_bf16, level, byte_off, codes, scale, zero, ws);
}

}  // extern "C"

// permutation groups of a coupled search (null row_group: every dimension on its own)
struct Coupling {
    const int32_t *row_group, *col_group, *group_segment, *row_repeat, *col_repeat;
    int n_groups;
};

static int search_impl(sbits_plan *plan, const sbits_matrix *mats, const Coupling &cpl, double avg_bits,
                       const sbits_params *params, const sbits_outputs *out, sbits_stats *host_stats, void *ws)
{
    if (!plan || !mats || !params || !out || !ws_ok(ws)) return SBITS_ERR_INVALID_ARG;
    if (!ws_fits(plan)) return SBITS_ERR_WORKSPACE;
    if (!out->row_perm || !out->col_perm || !out->cost || !out->level || !out->byte_off || !out->scale || !out->zero)
        return SBITS_ERR_INVALID_ARG;
    if (avg_bits < (double)plan->bits[0]) return SBITS_ERR_INFEASIBLE_BUDGET;
    if (out->codes_capacity < sbits_codes_bytes_bound(plan, avg_bits)) return SBITS_ERR_CAPACITY;
    // (a budget of 0 bits prunes every block: no code is ever written, so no buffer is needed)
    if (!out->codes && sbits_codes_bytes_bound(plan, avg_bits) > 0) return SBITS_ERR_INVALID_ARG;
    int rc = need_device(plan);
    if (rc) return rc;
    if ((rc = check_all(plan, mats, true, true))) return rc;
    if (cpl.row_group &&
        (rc = sbits_coupling_tables(plan, cpl.row_group, cpl.col_group, cpl.n_groups, cpl.group_segment, cpl.row_repeat,
                                    cpl.col_repeat, nullptr, nullptr, nullptr, nullptr, nullptr)))
        return rc;
    if ((rc = sbits_upload_descs(plan, mats, ws))) return rc;
    if (cpl.row_group)
        rc = sbits_launch_reorder_coupled_all(plan, cpl.row_group, cpl.col_group, cpl.n_groups, cpl.group_segment,
                                              cpl.row_repeat, cpl.col_repeat, out->row_perm, out->col_perm, ws);
    else
        rc = sbits_launch_reorder_all(plan, out->row_perm, out->col_perm, ws);
    if (rc) return rc;
    const bool one_pass = sbits_fused_shapes_ok(plan) && sbits_fused_layout_ok(plan, true);
    if (one_pass) {
        if ((rc = sbits_launch_gather_cost_all(plan, out->row_perm, out->col_perm, out->w_re_bf16, out->cost, ws)))
            return rc;
    } else {
        if (!out->s_re || !out->w_re_bf16) return SBITS_ERR_INVALID_ARG;
        if ((rc = sbits_launch_gather_all(plan, out->row_perm, out->col_perm, out->w_re_bf16, out->s_re, ws)))
            return rc;
        if ((rc = sbits_launch_cost_all(plan, out->w_re_bf16, out->s_re, out->cost, ws))) return rc;
    }
    rc = sbits_allocate(plan, out->cost, avg_bits, params, out->level, host_stats, nullptr, 0, ws);
    const int alloc_rc = rc;
    if (rc && rc != SBITS_ERR_MAX_ITERS) return rc;
    if ((rc = sbits_offsets(plan, out->level, out->byte_off, ws))) return rc;
    if (one_pass)
        rc = sbits_launch_gather_pack_all(plan, out->row_perm, out->col_perm, out->level, out->byte_off, out->codes,
                                          out->scale, out->zero, ws);
    else
        rc = sbits_launch_pack_all(plan, out->w_re_bf16, out->level, out->byte_off, out->codes, out->scale,
                                   out->zero, ws);
    if (rc) return rc;
    SBITS_HIP(plan->ctx, hipStreamSynchronize(plan->ctx->stream));
    return alloc_rc;
}

extern "C" {

int sbits_search(sbits_plan *plan, const sbits_matrix *mats, double avg_bits, const sbits_params *params,
                 const sbits_outputs *out, sbits_stats *host_stats, void *ws)
{
    const Coupling none = {nullptr, nullptr, nullptr, nullptr, nullptr, 0};
    return search_impl(plan, mats, none, avg_bits, params, out, host_stats, ws);
}

int sbits_search_coupled(sbits_plan *plan, const sbits_matrix *mats, const int32_t *row_group,
                         const int32_t *col_group, int n_groups, const int32_t *group_segment,
                         const int32_t *row_repeat, const int32_t *col_repeat, double avg_bits,
                         const sbits_params *params, const sbits_outputs *out, sbits_stats *host_stats, void *ws)
{
    if (!row_group || !col_group || n_groups < 0) return SBITS_ERR_INVALID_ARG;
    const Coupling cpl = {row_group, col_group, group_segment, row_repeat, col_repeat, n_groups};
    return search_impl(plan, mats, cpl, avg_bits, params, out, host_stats, ws);
}

}  // extern "C"
