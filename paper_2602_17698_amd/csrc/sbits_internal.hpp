// Internal declarations shared by the translation units of libscalebits.
// Host-side plan/context state and the launch entry of every kernel stage.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <vector>

#include "scalebits.h"
#include "sbits_device.hpp"

struct sbits_ctx {
    int device;            // -1: host-only context
    hipStream_t stream;
    int last_hip;
    void *pinned;          // small page-locked host buffer for state read-backs (allocated on first use)
    hipEvent_t readback;   // marks the end of a state read-back in the stream (created on first use)
    bool d16_zero_fill;    // 16-bit loads into a register half write zeros to the other half (target id "sramecc+")
};
constexpr size_t SBITS_PINNED_BYTES = 4096;

struct sbits_plan {
    sbits_ctx *ctx;
    int n_mats;
    std::vector<int64_t> rows, cols, base;   // base[mat] = first global block id
    int m, n, K;
    int32_t bits[sbits::MAX_CAND];           // ascending, within 0 .. 8; 0 = the block is pruned
    int64_t N;                               // total blocks
    int64_t max_rows, max_cols;
    int64_t sum_rows, sum_cols, sum_elems;
    int64_t sum_rowpart, sum_colpart;        // score partials over all matrices
    std::vector<int> score_wg_start;         // workgroup prefixes of the batched launches
    std::vector<int> cost_unit_start;
    std::vector<int> pack_wg_start;
    struct GatherClass { int64_t cols; int first, pre_first, n, rpw_w, rpw_s; };
    std::vector<GatherClass> gather_classes; // matrices grouped by column count
    std::vector<int> gather_members, gather_pre_w, gather_pre_s;
    struct FusedClass { int64_t cols; int first, pre_first, n, opu; };
    std::vector<FusedClass> fused_classes;   // the same grouping for the fused gather + cost launch
    std::vector<int> fused_members, fused_pre;
    std::vector<sbits::MatDesc> descs;       // shape part filled at creation; pointers per call
    size_t head_bytes;                       // workspace head: descriptor table + workgroup prefixes
    size_t ws_bytes;
    size_t ws_given;                         // size of the caller's workspace if declared, else SIZE_MAX
    void *desc_pinned;                       // two page-locked images of the descriptor table (allocated on first upload)
    hipEvent_t desc_done[2];                 // recorded behind the upload that read image i
    bool desc_used[2];
    int desc_turn;
};

// The workspace head holds the per-matrix descriptor table and the small integer tables (workgroup
// prefixes, class members, coupling tables) of the batched launches; stage scratch starts at sbits_scratch(plan, ws).
constexpr int SBITS_N_PREFIX = 11;
static inline size_t sbits_desc_bytes(int n_mats) { return (size_t)((n_mats * sizeof(sbits::MatDesc) + 255) / 256 * 256); }
static inline size_t sbits_prefix_bytes(int n_mats) { return (size_t)((2 * (n_mats + 1) * 4 + 255) / 256 * 256); }
static inline sbits::MatDesc *sbits_desc_ptr(void *ws) { return static_cast<sbits::MatDesc *>(ws); }
static inline int *sbits_prefix_ptr(const sbits_plan *p, void *ws, int slot)
{
    return reinterpret_cast<int *>(static_cast<char *>(ws) + sbits_desc_bytes(p->n_mats) +
                                   (size_t)slot * sbits_prefix_bytes(p->n_mats));
}
static inline void *sbits_scratch(const sbits_plan *p, void *ws) { return static_cast<char *>(ws) + p->head_bytes; }

#define SBITS_HIP(ctx, expr)                                                   \
    do {                                                                       \
        hipError_t e_ = (expr);                                                \
        if (e_ != hipSuccess) { (ctx)->last_hip = (int)e_; return SBITS_ERR_HIP; } \
    } while (0)

static inline size_t sbits_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- stage launchers (each returns an sbits_status) ------------------------

// workspace sizes in bytes
void sbits_score_geometry(int64_t R, int64_t C, int *nseg, int *nband);
int sbits_score_wgs(int nseg, int nband);
size_t sbits_reorder_ws_bytes(int64_t channels, int64_t rowpart, int64_t colpart);
size_t sbits_alloc_ws_bytes(int64_t N);
size_t sbits_offsets_ws_bytes(int64_t N);

int sbits_launch_scores(sbits_ctx *ctx, const float *S, int64_t R, int64_t C, int64_t ld,
                        float *row_score, float *col_score, void *ws);
int sbits_launch_reorder(sbits_ctx *ctx, const float *S, int64_t R, int64_t C, int64_t ld,
                         int32_t *row_perm, int32_t *col_perm, void *scratch);
int sbits_launch_reorder_all(sbits_plan *plan, int32_t *row_perm, int32_t *col_perm, void *ws);
int sbits_coupling_tables(const sbits_plan *plan, const int32_t *row_group, const int32_t *col_group, int n_groups,
                          const int32_t *group_segment, const int32_t *row_repeat, const int32_t *col_repeat,
                          std::vector<int> *mode, std::vector<int> *seg, std::vector<int> *next,
                          std::vector<int> *leader, std::vector<int> *rep);
int sbits_launch_reorder_coupled_all(sbits_plan *plan, const int32_t *row_group, const int32_t *col_group,
                                     int n_groups, const int32_t *group_segment, const int32_t *row_repeat,
                                     const int32_t *col_repeat, int32_t *row_perm, int32_t *col_perm, void *ws);
int sbits_launch_gather_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                            void *w_re, float *s_re, void *ws);
int sbits_launch_pack_all(sbits_plan *plan, const void *w_re, const uint8_t *level, const int64_t *byte_off,
                          uint8_t *codes, float *scale, float *zero, void *ws);
int sbits_launch_gather(sbits_ctx *ctx, const void *W, const float *S, int64_t R, int64_t C,
                        int64_t ld_w, int64_t ld_s, const int32_t *rp, const int32_t *cp,
                        void *w_out, float *s_out);
int sbits_launch_cost(sbits_ctx *ctx, const void *Wp, const float *Sp, int64_t R, int64_t C,
                      int m, int n, const int32_t *bits, int K, float *cost_rows);
// batched over all matrices of the plan (descriptor table already in the workspace head)
int sbits_upload_descs(sbits_plan *plan, const sbits_matrix *mats, void *ws);
int sbits_launch_cost_all(sbits_plan *plan, const void *w_re, const float *s_re, float *cost, void *ws);
// gather fused with the cost table (reads the original matrices once; writes w_re and cost)
bool sbits_fused_shapes_ok(const sbits_plan *plan);
bool sbits_fused_all_staged(const sbits_plan *plan);
bool sbits_fused_layout_ok(const sbits_plan *plan, bool need_s);
size_t sbits_fused_ws_bytes(const sbits_plan *plan);
int sbits_launch_gather_cost_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                                 void *w_re, float *cost, void *ws);
int sbits_launch_surrogates_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                                const uint8_t *level, float *s_up, float *s_down, void *ws);
int sbits_launch_gather_pack_all(sbits_plan *plan, const int32_t *row_perm, const int32_t *col_perm,
                                 const uint8_t *level, const int64_t *byte_off, uint8_t *codes, float *scale,
                                 float *zero, void *ws);
// dequant.hip
int sbits_launch_dequant(sbits_plan *plan, int mat, const uint8_t *level, const int64_t *byte_off,
                         const uint8_t *codes, const float *scale, const float *zero, void *out, int64_t ld_out,
                         int out_bf16);
// mpgemm.hip
bool sbits_mp_gemm_shapes_ok(const sbits_plan *plan);
size_t sbits_mp_gemm_ws_bytes(const sbits_plan *plan);
int sbits_launch_mp_gemm(sbits_plan *plan, int mat, const void *x_bf16, int64_t ld_x, int batch,
                         const uint8_t *level, const int64_t *byte_off, const uint8_t *codes, const float *scale,
                         const float *zero, float *y, void *scratch);
int sbits_run_propose(sbits_plan *plan, const float *s_up, const float *s_down, const uint8_t *level_in,
                      double avg_bits, int64_t k, uint8_t *level_out, sbits_proposal *host_out, void *ws);
int sbits_run_allocate(sbits_plan *plan, const float *cost, double avg_bits,
                       const sbits_params *prm, uint8_t *level, sbits_stats *host_stats,
                       sbits_trace *host_trace, int64_t trace_cap, void *ws);
int sbits_launch_offsets(sbits_ctx *ctx, const uint8_t *level, int64_t N, int m, int n,
                         const int32_t *bits, int K, int64_t *byte_off, void *ws);
int sbits_offsets_static_setup(sbits_ctx *ctx);
int sbits_launch_offsets_static(sbits_ctx *ctx, const uint8_t *level, int64_t N, int m, int n,
                                const int32_t *bits, int K, int64_t *byte_off);
int sbits_launch_pack(sbits_ctx *ctx, const void *Wp, int64_t R, int64_t C, int m, int n,
                      const int32_t *bits, int K, const uint8_t *level, const int64_t *byte_off,
                      int64_t block_base, uint8_t *codes, float *scale, float *zero);
