// Host-side launch interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once
#include <hip/hip_ext.h>

#include "common.hpp"

namespace fastocr {

// Kernel ids mirror fastocr_kernel in fastocr.h (used by the per-kernel timers).
enum KernelId {
    K_SCORE_LOGITS = 0, K_SCORE_FINALIZE = 1, K_TOPK = 2, K_SPARSE_ATTN = 3, K_DENSE_ATTN = 4,
    K_ATTN_COMBINE = 5, K_FOCAL_FUSED = 6, K_COUNT = 7
};

// Per-kernel timing (api.hip): when a timer is enabled for `kernel`, the next launch gets a pair of
// events that the runtime stamps at the kernel's own start and end (hipExtLaunchKernelGGL);
// otherwise both are null and the launch is an ordinary one.
struct TimerEvents { hipEvent_t start, stop; };
TimerEvents timer_events(int kernel);

#define FASTOCR_LAUNCH(KID, KERNEL, GRID, BLOCK, SHMEM, STREAM, ...)                                   \
    do {                                                                                               \
        const ::fastocr::TimerEvents te_ = ::fastocr::timer_events(KID);                               \
        hipExtLaunchKernelGGL((KERNEL), (GRID), (BLOCK), (SHMEM), (STREAM), te_.start, te_.stop, 0,    \
                              __VA_ARGS__);                                                            \
    } while (0)

enum { DT_F32 = 0, DT_BF16 = 1 };

struct Shape {
    KvDev kv;
    BatchDev bv;
    int batch;
    int n_q_heads;
    int dtype;
    bool paged;
    bool vec16;     // every cache row starts 16-byte aligned and head_dim covers whole 16-byte pieces
    bool fast;      // the MFMA kernels cover this shape: bf16, head_dim 128, group size <= 16,
                    // 16-byte aligned rows (decided once from the views by the C-ABI layer)
};

inline bool mfma_path(const Shape &s) { return s.fast; }

// ---- attention (attn.hip) ---------------------------------------------------------------
// Workspace: part_o fp32 [B][Hq][nsplit][d] followed by part_ml fp32 [B][Hq][nsplit][2].
int attn_tile_tokens(const Shape &s);
size_t attn_workspace_bytes(const Shape &s, int nsplit);
// merge_in_kernel: with 2 .. 4 ranges per stream on the MFMA path the stream's last range merges
// the others' partials inside the launch (through static device memory) when the shape fits
// (attn_merges_in_kernel); otherwise partials go to the workspace and a merge kernel follows.
bool attn_merges_in_kernel(const Shape &s, int nsplit);
hipError_t launch_attn(const Shape &s, const void *q, float scale, const int32_t *sel_idx,
                       const int32_t *sel_cnt, int64_t kmax, void *out, float *lse, void *ws,
                       int nsplit, bool merge_in_kernel, hipStream_t stream);
// merge of nsplit partials per (sequence, head) in the layout above into the final output.
// With seq_meta (device int32 [B][2]: first workgroup, workgroup count) the partials are instead
// those of the fused focal kernel, [workgroup][wpk][Hq][d] / [..][2], wpk per workgroup.
hipError_t launch_attn_combine(const Shape &s, const float *part_o, const float *part_ml, int nsplit,
                               void *out, float *lse, hipStream_t stream, const int32_t *seq_meta = nullptr,
                               int wpk = 1);

// ---- focal scoring (score.hip) ----------------------------------------------------------
// Workspace: logits fp32 [B][Hq][pitch], part_ml fp32 [B][Hq][nsplit][2], mass partials.
int score_tile_tokens(const Shape &s);
size_t score_workspace_bytes(const Shape &s, int nsplit);
hipError_t launch_score(const Shape &s, const void *q, float scale, float *scores, float *lse,
                        float *img_mass, void *ws, int nsplit, hipStream_t stream);

// ---- focal scoring with register-resident logits (score_resident.hip) ---------------------
// The plan gives the grid (nranges * batch workgroups, at most one per compute unit) and the
// range length used when all sequences are equally long; ragged batches are split on the device.
// Workspace, W = nranges * batch: image-mass partials fp32 [W], per sequence its first workgroup
// and range count int32 [B][2] (the ranges' softmax statistics travel through static device memory).
struct ResidentPlan { int nranges, range_tokens, wpk; };
bool resident_plan(const Shape &s, int num_cu, ResidentPlan *plan);
size_t resident_workspace_bytes(const Shape &s, const ResidentPlan &p);
hipError_t launch_score_resident(const Shape &s, const ResidentPlan &p, const void *q, float scale, float *scores,
                                 float *lse, float *img_mass, void *ws, hipStream_t stream);

// ---- focal layer in one pass: dense attention output + scores (focal_fused.hip) -----------
// Uses the same plan as the register-resident scoring kernel.
size_t focal_fused_workspace_bytes(const Shape &s, const ResidentPlan &p);
hipError_t launch_focal_fused(const Shape &s, const ResidentPlan &p, const void *q, float scale, void *out,
                              float *scores, float *lse, float *img_mass, void *ws, hipStream_t stream);

// ---- how often a workgroup gave up waiting for another one of its launch (each file's own count;
// the copies synchronise with the device) ----------------------------------------------------
hipError_t score_resident_timeouts(uint32_t *n);
hipError_t focal_fused_timeouts(uint32_t *n);
hipError_t attn_merge_timeouts(uint32_t *n);

// ---- top-k (topk.hip) -------------------------------------------------------------------
size_t topk_workspace_bytes(int batch, int max_vis_len);
hipError_t launch_topk(const float *scores, const BatchDev &bv, int batch, double tau,
                       const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                       int32_t *sel_cnt, int64_t kmax, void *ws, hipStream_t stream);

// ---- streaming probe (probe.hip) ----------------------------------------------------------
hipError_t launch_stream_probe(const void *src, void *dst, size_t bytes, void *sink, hipStream_t stream);

}  // namespace fastocr
