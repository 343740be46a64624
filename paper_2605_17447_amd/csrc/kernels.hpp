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
    bool fast;      // the MFMA kernels cover this shape: bf16, head_dim 128 or 64, group size <= 16,
                    // 16-byte aligned rows (decided once from the views by the C-ABI layer); the
                    // one-pass focal kernel and the in-launch merge need head_dim 128, register-resident
                    // scoring takes both
};

inline bool mfma_path(const Shape &s) { return s.fast; }

// ---- host-side state shared by the launchers (api.hip) --------------------------------------
// Launch-shape overrides (fastocr_set_tuning); atomics, so that callers on several threads may
// read them while another thread sets one.
int tune_attn_waves();                 // 4 or 8
long long tune_spin_ticks();           // bounded wait of the single-launch forms, in 100 MHz wall-clock ticks
// Compute units the launch shapes are planned for: the current device's, or 256 (MI355X) when no
// device can be asked.
int plan_cu_count();

// Exchange slots of the single-launch forms.  Workgroups of such a launch hand each other data
// through static device memory, one slot per call in flight.  Two calls may share a slot only if
// the second cannot start before the first has ended, i.e. if they are enqueued on the same
// stream; so a slot belongs to a stream: the first k*EagerSlots streams of a device that ask for
// one keep it for the life of the process.  A call that is being captured into a HIP graph gets a
// slot of a separate pool that belongs to (capture, stream) and is never handed out again -- the
// graph may be replayed on any stream next to eager calls.  Returns the slot, or -1 when none is
// left (or the stream's capture state cannot be read): the caller then takes the form built from
// separate kernels, which shares nothing.
enum ExchangeKind { EX_SCORE = 0, EX_FUSED = 1, EX_MERGE = 2, EX_KINDS = 3 };
constexpr int kResSlots = 64;          // slots of each register-resident kernel (scoring, fused focal layer), 128 KB of static memory each
constexpr int kResEagerSlots = 16;     //   of which for streams; the rest for graph captures
constexpr int kMergeSlots = 16;        // slots of pruned attention's in-launch merge, 3.2 MB of static memory each
constexpr int kMergeEagerSlots = 4;
// *gave_up_flag: a device-visible word in pinned host memory that a wave sets when it gives up
// waiting inside a single-launch form (null if it could not be allocated yet: the first call on a
// device happened inside a capture); once it is set the library's own choice (tuning mode 1) is
// the separate-kernel forms for the rest of the process ("exchange_fallback" 0 re-arms it).
int exchange_slot(int kind, hipStream_t stream, uint32_t **gave_up_flag);
bool exchange_trusted();               // false once a wave has given up (or "exchange_fallback" 1)

// ---- attention (attn.hip) ---------------------------------------------------------------
// Workspace: part_o fp32 [B][Hq][nsplit][d] followed by part_ml fp32 [B][Hq][nsplit][2].
int attn_tile_tokens(const Shape &s);
size_t attn_workspace_bytes(const Shape &s, int nsplit);
// With 2 .. 4 ranges per stream on the MFMA path the stream's last range can merge the others'
// partials inside the launch (through static device memory) when the shape fits
// (attn_merges_in_kernel) and an exchange slot is given; otherwise partials go to the workspace
// and a merge kernel follows.
bool attn_merges_in_kernel(const Shape &s, int nsplit);
// merge_slot: exchange slot for the in-launch merge (EX_MERGE), or -1 = partials + merge kernel.
hipError_t launch_attn(const Shape &s, const void *q, float scale, const int32_t *sel_idx,
                       const int32_t *sel_cnt, int64_t kmax, void *out, float *lse, void *ws,
                       int nsplit, int merge_slot, uint32_t *gave_up_flag, hipStream_t stream);
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
// The top-k fused into a register-resident launch (sel_idx == nullptr: none): the arguments of
// fastocr_topk_fixation.
struct SelectArgs {
    double tau;
    const int32_t *prev_idx, *prev_cnt;
    int32_t *sel_idx, *sel_cnt;
    int64_t kmax;
};
// whether the fused select covers the shape (image spans of up to 16384 tokens)
bool resident_select_fits(const Shape &s);
bool resident_plan(const Shape &s, int num_cu, ResidentPlan *plan);
size_t resident_workspace_bytes(const Shape &s, const ResidentPlan &p);
hipError_t launch_score_resident(const Shape &s, const ResidentPlan &p, int sync_slot, uint32_t *gave_up_flag, const void *q, float scale,
                                 float *scores, float *lse, float *img_mass, void *ws, hipStream_t stream,
                                 const SelectArgs *select = nullptr);

// ---- focal layer in one pass: dense attention output + scores (focal_fused.hip) -----------
// Uses the same plan as the register-resident scoring kernel.
size_t focal_fused_workspace_bytes(const Shape &s, const ResidentPlan &p);
// A merge of attention partials handed on to the launch that follows (see launch_topk).
struct CombineArgs {
    const float *part_o, *part_ml;
    int nsplit, d, n_q_heads, wpk;
    const int32_t *seq_meta;
    uint16_t *out;              // bf16 [B, Hq, d]
};
// defer != nullptr: the merge of the output's partials is not launched; *defer describes it and the
// caller passes it to launch_topk, whose launch then does both (the top-k and that merge depend on
// this kernel only, not on each other).
hipError_t launch_focal_fused(const Shape &s, const ResidentPlan &p, int sync_slot, uint32_t *gave_up_flag, const void *q, float scale,
                              void *out, float *scores, float *lse, float *img_mass, void *ws, hipStream_t stream,
                              const SelectArgs *select = nullptr, CombineArgs *defer = nullptr);

// ---- how often a workgroup gave up waiting for another one of its launch (each file's own count;
// the copies synchronise with the device) ----------------------------------------------------
hipError_t score_resident_timeouts(uint32_t *n);
hipError_t focal_fused_timeouts(uint32_t *n);
hipError_t attn_merge_timeouts(uint32_t *n);

// ---- top-k (topk.hip) -------------------------------------------------------------------
size_t topk_workspace_bytes(int batch, int max_vis_len);
// combine != nullptr (only when topk_takes_combine says so): the launch gets one more workgroup per
// (sequence, query head), which merges that head's attention partials.
hipError_t launch_topk(const float *scores, const BatchDev &bv, int batch, double tau,
                       const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                       int32_t *sel_cnt, int64_t kmax, void *ws, hipStream_t stream,
                       const CombineArgs *combine = nullptr);
bool topk_takes_combine(int max_vis_len, int head_dim);

// ---- streaming probe (probe.hip) ----------------------------------------------------------
hipError_t launch_stream_probe(const void *src, void *dst, size_t bytes, void *sink, hipStream_t stream);

}  // namespace fastocr
