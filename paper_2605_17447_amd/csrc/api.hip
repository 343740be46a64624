// C ABI of the FastOCR decode hot path: host-side validation, workspace sizing, launch-shape
// choice and per-kernel event timers.  Every check happens before the first HIP call, so the
// error paths can be exercised without a GPU.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "fastocr.h"
#include "kernels.hpp"

namespace fastocr {

// ---- launch-shape overrides (fastocr_set_tuning) --------------------------------------------
// Plain values read on every call and written rarely, possibly from another thread: atomics.
static std::atomic<int> g_tune_score_resident{1};
static std::atomic<int> g_tune_focal_fused{1};
static std::atomic<int> g_tune_attn_waves{4};
static std::atomic<int> g_tune_attn_merge{1};          // pruned attention: ranges of a stream merged inside the launch (0 never, 1 yes)
static std::atomic<int> g_tune_barrier_spin_us{250000};      // bounded wait of the single-launch forms
static std::atomic<int> g_tune_splits[4];              // indexed by fastocr_op; 0 = automatic
static std::atomic<int> g_tune_timer_every{1};         // per-kernel timers: which launches record events (every n-th)
static std::atomic<int> g_exchange_distrusted{0};      // "exchange_fallback" 1
static std::atomic<int> g_tune_graph_replay{0};        // 1: the caller replays its calls from a HIP graph, where a launch follows the one before within half a microsecond
static std::atomic<int> g_tune_select_fused{0};        // top-k inside the scoring / focal-layer launch (0 never, 1 when it fits): measured slower, off by default

int tune_attn_waves() { return g_tune_attn_waves.load(std::memory_order_relaxed); }
long long tune_spin_ticks() { return 100ll * g_tune_barrier_spin_us.load(std::memory_order_relaxed); }   // the wall clock runs at 100 MHz

// Everything below that is more than one word (timers, slot registry, per-device tables) is
// guarded by one mutex; it is held for a few table look-ups per call.
static std::mutex g_mu;

// ---- per-kernel timers ------------------------------------------------------------------
struct KernelTimer {
    int capacity = 0;
    int count = 0;
    unsigned seen = 0;      // launches of the kernel since the timer was enabled
    hipEvent_t *start = nullptr;
    hipEvent_t *stop = nullptr;
};
static KernelTimer g_timers[K_COUNT];

TimerEvents timer_events(int kernel)
{
    std::lock_guard<std::mutex> lock(g_mu);
    KernelTimer &t = g_timers[kernel];
    if (t.count >= t.capacity) return TimerEvents{nullptr, nullptr};
    // an event pair costs the stream a few microseconds: only every timer_every-th launch carries one
    if (t.seen++ % (unsigned)g_tune_timer_every.load(std::memory_order_relaxed) != 0u) return TimerEvents{nullptr, nullptr};
    const int i = t.count++;
    return TimerEvents{t.start[i], t.stop[i]};
}

// ---- the device the call runs on ----------------------------------------------------------------
constexpr int kMaxDevices = 64;

static int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return -1; }
    return dev >= 0 && dev < kMaxDevices ? dev : -1;
}

int plan_cu_count()
{
    static int cached[kMaxDevices] = {0};          // 0 = not asked yet; guarded by g_mu
    const int dev = current_device();
    if (dev < 0) return 256;
    std::lock_guard<std::mutex> lock(g_mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) { (void)hipGetLastError(); n = 0; }
        cached[dev] = n > 0 ? n : 256;
    }
    return cached[dev];
}

// ---- exchange slots (see kernels.hpp) --------------------------------------------------------------
struct SlotOwner { hipStream_t stream; unsigned long long capture; bool free; };
struct SlotTable { std::vector<SlotOwner> eager, graph; };
static SlotTable g_slots[EX_KINDS][kMaxDevices];

static uint32_t *g_gave_up[kMaxDevices];       // pinned host memory, one word per device, never freed

int exchange_slot(int kind, hipStream_t stream, uint32_t **gave_up_flag)
{
    *gave_up_flag = nullptr;
    const int total = kind == EX_MERGE ? kMergeSlots : kResSlots;
    const int n_eager = kind == EX_MERGE ? kMergeEagerSlots : kResEagerSlots;
    const int dev = current_device();
    if (dev < 0) return -1;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    unsigned long long cap = 0;
    if (hipStreamGetCaptureInfo(stream, &st, &cap) != hipSuccess) {
        // e.g. the legacy default stream while another stream of the device is capturing
        (void)hipGetLastError();
        return -1;
    }
    if (st == hipStreamCaptureStatusInvalidated) return -1;
    const bool capturing = st == hipStreamCaptureStatusActive;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_gave_up[dev] && !capturing) {
        // one word of pinned host memory per device, allocated on the first eager call that reaches
        // this point (an allocation is not a capturable call) and kept until the process ends
        void *p = nullptr;
        if (hipHostMalloc(&p, 64, hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess && p) {
            memset(p, 0, 64);
            g_gave_up[dev] = static_cast<uint32_t *>(p);
        } else {
            (void)hipGetLastError();
        }
    }
    *gave_up_flag = g_gave_up[dev];
    SlotTable &t = g_slots[kind][dev];
    std::vector<SlotOwner> &pool = capturing ? t.graph : t.eager;
    const int cap_n = capturing ? total - n_eager : n_eager;
    const int first = capturing ? n_eager : 0;
    for (size_t i = 0; i < pool.size(); ++i)
        if (!pool[i].free && pool[i].stream == stream && (!capturing || pool[i].capture == cap)) return first + (int)i;
    for (size_t i = 0; i < pool.size(); ++i)
        if (pool[i].free) {                      // released by fastocr_stream_release
            pool[i] = SlotOwner{stream, capturing ? cap : 0ull, false};
            return first + (int)i;
        }
    if ((int)pool.size() >= cap_n) return -1;
    pool.push_back(SlotOwner{stream, capturing ? cap : 0ull, false});
    return first + (int)pool.size() - 1;
}

bool exchange_trusted()
{
    if (g_exchange_distrusted.load(std::memory_order_relaxed)) return false;
    const int dev = current_device();
    if (dev < 0) return true;
    std::lock_guard<std::mutex> lock(g_mu);
    const uint32_t *f = g_gave_up[dev];
    return !f || __atomic_load_n(f, __ATOMIC_RELAXED) == 0u;
}

// ---- workspace in static device memory, for fastocr_dense_decode_attn_static -------------------------
// The array's name is a host-side handle, not a device address: what kernels and copies get is the
// address hipGetSymbolAddress returns for the device that is current, asked for once per device
// (every GPU holds its own copy of the array at its own address).
static __device__ __align__(256) unsigned char scratch[FASTOCR_STATIC_SCRATCH_BYTES];
static void *g_scratch_ptr[kMaxDevices];       // guarded by g_mu

static void *static_scratch_ptr()
{
    const int dev = current_device();
    if (dev < 0) return nullptr;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

// ---- shapes -----------------------------------------------------------------------------
static int check_views(const fastocr_kv_view *kv, const fastocr_batch_view *bv, int n_q_heads)
{
    if (!kv || !bv) return FASTOCR_EINVAL;
    if (!kv->k || !kv->v) return FASTOCR_EINVAL;
    if (kv->dtype != FASTOCR_F32 && kv->dtype != FASTOCR_BF16) return FASTOCR_EUNSUPPORTED;
    if (kv->n_kv_heads < 1 || kv->head_dim < 1) return FASTOCR_EINVAL;
    if (n_q_heads < 1 || n_q_heads % kv->n_kv_heads != 0) return FASTOCR_EINVAL;
    if (kv->head_dim > 256 || n_q_heads > 256) return FASTOCR_EUNSUPPORTED;
    if (kv->stride_token < kv->head_dim || kv->stride_head < 0 || kv->stride_seq < 0) return FASTOCR_EINVAL;
    if (bv->batch < 0 || bv->max_seq_len < 0 || bv->max_vis_len < 0) return FASTOCR_EINVAL;
    if (bv->max_vis_len > bv->max_seq_len) return FASTOCR_EINVAL;
    if (bv->batch > 65535) return FASTOCR_EUNSUPPORTED;
    if (bv->batch > 0 && (!bv->seq_len || !bv->vis_start || !bv->vis_len)) return FASTOCR_EINVAL;
    if (kv->page_tokens < 0) return FASTOCR_EINVAL;
    if (kv->page_tokens > 0) {
        if (!kv->block_table || kv->stride_page < 1) return FASTOCR_EINVAL;
        const int64_t need = ((int64_t)bv->max_seq_len + kv->page_tokens - 1) / kv->page_tokens;
        if (kv->max_pages_per_seq < need || kv->max_pages_per_seq < 1) return FASTOCR_EINVAL;
    }
    return FASTOCR_OK;
}

static Shape make_shape(const fastocr_kv_view *kv, const fastocr_batch_view *bv, int n_q_heads)
{
    Shape s;
    s.kv.k = kv->k;
    s.kv.v = kv->v;
    s.kv.stride_token = kv->stride_token;
    s.kv.stride_head = kv->stride_head;
    s.kv.stride_seq = kv->stride_seq;
    s.kv.stride_page = kv->stride_page;
    s.kv.block_table = kv->block_table;
    s.kv.max_pages = kv->max_pages_per_seq;
    s.kv.page_tokens = kv->page_tokens;
    s.kv.n_kv_heads = kv->n_kv_heads;
    s.kv.head_dim = kv->head_dim;
    s.bv.seq_len = bv->seq_len;
    s.bv.vis_start = bv->vis_start;
    s.bv.vis_len = bv->vis_len;
    s.bv.max_seq_len = bv->max_seq_len;
    s.bv.max_vis_len = bv->max_vis_len;
    s.batch = bv->batch;
    s.n_q_heads = n_q_heads;
    s.dtype = kv->dtype;
    s.paged = kv->page_tokens > 0;
    // The MFMA kernels read 16-byte vectors: every cache row must start 16-byte aligned.
    auto a16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    const bool aligned = a16(kv->k) && a16(kv->v) && kv->stride_token % 8 == 0 &&
                         kv->stride_head % 8 == 0 && kv->stride_seq % 8 == 0 && kv->stride_page % 8 == 0;
    s.fast = kv->dtype == FASTOCR_BF16 && (kv->head_dim == 128 || kv->head_dim == 64) && n_q_heads / kv->n_kv_heads <= 16 && aligned;
    const int64_t esz = kv->dtype == FASTOCR_BF16 ? 2 : 4;
    auto m16 = [&](int64_t elems) { return (elems * esz) % 16 == 0; };
    s.vec16 = a16(kv->k) && a16(kv->v) && m16(kv->stride_token) && m16(kv->stride_head) && m16(kv->stride_seq) &&
              m16(kv->stride_page) && m16(kv->head_dim);
    return s;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Number of position ranges per (sequence, kv head): enough workgroups to fill the chip a few
// times over, never less than one tile per wave.  A pure function of the host-side shape so
// that the workspace query and the launch agree.
// Pruned attention as partials over four-wave workgroups of one tile per wave: the finest cut
// choose_splits ever makes of a short list.  *fits: such a cut leaves at most one workgroup per compute
// unit (only then is it taken).  The value is capped at that and so monotone in the list's length:
// it is what the workspace is sized for, whatever length the calls then have.
static int finest_splits(const Shape &s, int max_positions, bool *fits = nullptr)
{
    const int streams = s.batch * s.kv.n_kv_heads;
    const int ntile = (max_positions + 31) / 32;
    const int by_work = (ntile + 3) / 4;
    const int most = streams > 0 ? plan_cu_count() / streams : 1;
    if (fits) *fits = by_work <= most;
    const int n = by_work < most ? by_work : most;
    return n < 1 ? 1 : n;
}

// replay: 0 / 1 = as if "graph_replay" were that, -1 = the tuning's value.  *partials (if given) is set
// when the choice only holds as partials in the workspace followed by the merge kernel.
static int choose_splits(int op, const Shape &s, int max_positions, bool *partials = nullptr, int replay = -1)
{
    if (partials) *partials = false;
    if (replay < 0) replay = g_tune_graph_replay.load(std::memory_order_relaxed);
    const bool fast = s.fast;
    const int kNumCU = plan_cu_count();
    const int forced = g_tune_splits[op].load(std::memory_order_relaxed);
    const int tile = fast ? 32 : 64;
    const int waves_per_wg = fast ? 4 : 1;
    const int ntile = (max_positions + tile - 1) / tile;
    const int by_work = (ntile + waves_per_wg - 1) / waves_per_wg;
    int nsplit;
    if (forced > 0) {
        nsplit = forced;
    } else {
        const int streams = s.batch * (fast ? s.kv.n_kv_heads : s.n_q_heads);
        // Measured on MI355X: the streaming kernels run best with about one workgroup per compute
        // unit (few, long, equally sized streams), the plain-FMA kernels with many small ones.
        const int target_wg = fast ? kNumCU : 8 * kNumCU;
        if (fast && op == FASTOCR_OP_SPARSE_DECODE_ATTN && g_tune_attn_merge.load(std::memory_order_relaxed)) {
            // pruned attention is short: one launch whose eight-wave workgroups fill the chip once,
            // the ranges of a stream merged inside the launch.  Up to 16 tiles one workgroup has the
            // whole list in flight at once (two tiles per wave) and a cut only adds the merge (15 tiles,
            // 32 streams: 10.7 / 10.8 / 10.7 / 11.5 us with 1 / 2 / 3 / 4 ranges); beyond that three
            // ranges measured best (17 tiles, 4 streams: 10.7 / 10.7 / 10.3 / 10.6 us; 21 tiles, 32
            // streams: 13.7 / 12.7 / 11.3 / 11.5 us; 25 tiles: 15.4 / 13.2 / 11.5 / 11.7 us; 40 tiles:
            // 18.6 / 16.0 / 13.7 / 13.9 us), four from 48 tiles on
            int n = kNumCU / (streams > 0 ? streams : 1);
            const int by_len = ntile <= 16 ? 1 : (ntile < 48 ? 3 : 4);
            n = n < by_len ? n : by_len;
            n = n < 1 ? 1 : n;
            if (n == 1 || attn_merges_in_kernel(s, n)) {
                // A compute unit gathers rows at a few tens of GB/s, so a short list of few streams is
                // done sooner the more compute units share it -- but every range a stream is cut into
                // makes the in-launch merge wait longer for words to cross the chip (3 - 4 us against a
                // plain store of the partial).  Replayed from a graph, where the merge kernel starts
                // 0.4 us after the launch before it (eager: 2 - 3 us), partials over four-wave workgroups
                // of one tile per wave plus that kernel win as long as those workgroups find a compute
                // unit each (28- and 36-layer stacks, batch 4 - 16, 8 - 64 streams of 15 - 47 tiles:
                // 356 -> 331, 391 -> 376, 495 -> 443, 364 -> 323, 548 -> 452, 403 -> 327 us per decode
                // step; with 96 and 128 streams of 15 tiles, where they would not: 418 -> 464 and
                // 449 -> 506 us, so those keep the single launch; eager the fine cut costs 2 us per call).
                bool fits = false;
                const int fine = finest_splits(s, max_positions, &fits);
                if (replay == 1 && fits && fine > n) {
                    if (partials) *partials = true;
                    return fine;
                }
                return n;
            }
        }
        nsplit = (target_wg + streams - 1) / (streams > 0 ? streams : 1);
        // pruned attention is short: when eight waves get at most eight tiles each, or at least half
        // a chip of streams exists, one eight-wave workgroup per stream writes the final output
        // itself (no partials, no merge kernel -- a second launch costs more than it saves here)
        if (fast && op == FASTOCR_OP_SPARSE_DECODE_ATTN && (2 * streams >= kNumCU || ntile <= 64)) nsplit = 1;
    }
    if (nsplit > by_work) nsplit = by_work;
    if (nsplit > 256) nsplit = 256;
    if (nsplit < 1) nsplit = 1;
    return nsplit;
}

// Upper bound of the positions a pruned-attention call attends: all text plus kmax image tokens
// (kmax <= 0: unknown, the whole sequence).
static int sparse_positions(const fastocr_batch_view *bv, int64_t kmax)
{
    if (kmax <= 0 || kmax >= bv->max_vis_len) return bv->max_seq_len;
    return bv->max_seq_len - bv->max_vis_len + (int)kmax;
}

static size_t round256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace fastocr

using namespace fastocr;

extern "C" {

int64_t fastocr_keep_count(int64_t n_visual, double tau)
{
    if (n_visual <= 0 || !(tau > 0.0)) return 0;
    double x = ceil(tau * (double)n_visual - 1e-9);
    if (x < 0.0) x = 0.0;
    if (x > (double)n_visual) x = (double)n_visual;
    return (int64_t)x;
}

size_t fastocr_workspace_bytes(int op, const fastocr_kv_view *kv, const fastocr_batch_view *bv,
                               int n_q_heads, int64_t kmax)
{
    if (op == FASTOCR_OP_TOPK_FIXATION) {
        if (!bv || bv->batch < 0 || bv->max_vis_len < 0) return 0;
        return round256(topk_workspace_bytes(bv->batch, bv->max_vis_len));
    }
    if (op == FASTOCR_OP_FOCAL_SCORE_TOPK || op == FASTOCR_OP_FOCAL_ATTN_SCORE_TOPK) {
        // the fused launch, or the two separate calls one after the other in the same buffer
        const size_t a = fastocr_workspace_bytes(op == FASTOCR_OP_FOCAL_SCORE_TOPK ? FASTOCR_OP_FOCAL_SCORE : FASTOCR_OP_FOCAL_ATTN_SCORE,
                                                 kv, bv, n_q_heads, 0);
        const size_t b = fastocr_workspace_bytes(FASTOCR_OP_TOPK_FIXATION, kv, bv, n_q_heads, kmax);
        return a == 0 ? 0 : (a > b ? a : b);
    }
    if (op < 0 || op > FASTOCR_OP_FOCAL_ATTN_SCORE) return 0;
    if (check_views(kv, bv, n_q_heads) != FASTOCR_OK) return 0;
    Shape s = make_shape(kv, bv, n_q_heads);
    if (op == FASTOCR_OP_FOCAL_ATTN_SCORE) {
        // the one-pass kernel, or the two separate calls one after the other in the same buffer
        size_t need = fastocr_workspace_bytes(FASTOCR_OP_FOCAL_SCORE, kv, bv, n_q_heads, 0);
        const size_t dense = fastocr_workspace_bytes(FASTOCR_OP_DENSE_DECODE_ATTN, kv, bv, n_q_heads, 0);
        need = need > dense ? need : dense;
        ResidentPlan rp;
        if (s.kv.head_dim == 128 && resident_plan(s, plan_cu_count(), &rp)) {
            const size_t fused = round256(focal_fused_workspace_bytes(s, rp) + 256);
            need = need > fused ? need : fused;
        }
        return need;
    }
    // fewer positions never need more ranges, so a bound taken with a larger kmax (or none) also covers;
    // pruned attention: sized for the finest cut as well, whether or not "graph_replay" asks for it
    const int positions = op == FASTOCR_OP_SPARSE_DECODE_ATTN ? sparse_positions(bv, kmax) : bv->max_seq_len;
    int nsplit = choose_splits(op, s, positions, nullptr, 0);
    if (op == FASTOCR_OP_SPARSE_DECODE_ATTN && s.fast && g_tune_splits[op].load(std::memory_order_relaxed) <= 0) {
        const int finest = finest_splits(s, positions);
        nsplit = nsplit > finest ? nsplit : finest;
    }
    if (op == FASTOCR_OP_FOCAL_SCORE) {
        // sized for either scoring path, so that the choice can be made at launch
        size_t need = score_workspace_bytes(s, nsplit);
        ResidentPlan rp;
        if (resident_plan(s, plan_cu_count(), &rp)) need = need > resident_workspace_bytes(s, rp) ? need : resident_workspace_bytes(s, rp);
        return round256(need + 256);
    }
    return round256(attn_workspace_bytes(s, nsplit) + 256);
}

static int check_ws(const void *ws, size_t ws_bytes, size_t need)
{
    if (need == 0) return FASTOCR_OK;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || ws_bytes < need) return FASTOCR_EWORKSPACE;
    return FASTOCR_OK;
}

static int check_qo(const fastocr_kv_view *kv, const void *q, const void *out, float scale)
{
    if (!q || !isfinite(scale)) return FASTOCR_EINVAL;
    if (!aligned16(q) || (out && !aligned16(out))) return FASTOCR_EINVAL;
    (void)kv;
    return FASTOCR_OK;
}

// The register-resident kernels (scoring alone, or fused with the dense output) pay a few
// microseconds for their grid-wide exchange (statistics through memory, polled); the paths built
// from separate kernels pay a second read of K or a round trip of the logits through memory, and
// one or two more launches.  Measured on MI355X down to one image tile per wave (batch 1, N = 4096)
// the single-kernel forms are never slower: scoring 13 us against 5 + 6 us in two launches, the
// focal layer 16 + 5 us against 6 + 4 + 11 us, at batch 8 25 + 4 against 16 + 4 + 18 us.  So the
// size rule (mode 1) takes them whenever the shape fits, like mode 2; mode 0 = never.  The
// thresholds stay as the place to change that.
constexpr int kResidentMinTiles = 1;
constexpr int kFusedMinTiles = 1;

// mode: the tuning value (0 never, 1 the library's choice, 2 whenever the shape fits).  The
// library's own choice also requires that no wave of a single-launch form has ever given up
// waiting in this process: a launch that cannot have the chip to itself is not tried twice.
// On success *slot is the call's exchange slot.
static bool use_resident(int kind, int mode, const Shape &s, ResidentPlan *rp, int min_tiles, hipStream_t stream, int *slot,
                         uint32_t **flag)
{
    const int cus = plan_cu_count();
    if (mode == 0 || !resident_plan(s, cus, rp)) return false;
    if (kind == EX_FUSED && s.kv.head_dim != 128) return false;      // the one-pass focal kernel: head_dim 128 only
    if (rp->nranges * s.batch > cus) return false;
    if (mode != 2 && (rp->range_tokens / (32 * rp->wpk) < min_tiles || !exchange_trusted())) return false;
    *slot = exchange_slot(kind, stream, flag);
    return *slot >= 0;
}

static int check_topk_args(const float *scores, const fastocr_batch_view *bv, double tau, const int32_t *prev_idx,
                           const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax)
{
    if (!bv || bv->batch < 0 || bv->max_vis_len < 0 || bv->max_seq_len < 0) return FASTOCR_EINVAL;
    if (bv->max_vis_len > bv->max_seq_len) return FASTOCR_EINVAL;
    if (bv->batch > 65535) return FASTOCR_EUNSUPPORTED;
    if (!(tau >= 0.0 && tau <= 1.0)) return FASTOCR_EINVAL;
    if (bv->batch > 0 && (!bv->seq_len || !bv->vis_start || !bv->vis_len)) return FASTOCR_EINVAL;
    if (!sel_idx || !sel_cnt) return FASTOCR_EINVAL;
    if (!scores && bv->max_vis_len > 0 && bv->batch > 0) return FASTOCR_EINVAL;
    if ((prev_idx == nullptr) != (prev_cnt == nullptr)) return FASTOCR_EINVAL;
    if (kmax < 1 || kmax < fastocr_keep_count(bv->max_vis_len, tau)) return FASTOCR_EINVAL;
    return FASTOCR_OK;
}

// Scoring, optionally with the top-k inside the same launch (select != nullptr).  *fused tells the
// caller whether the select ran inside the launch; if not, it still has to be called.
static int focal_score_impl(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                            int n_q_heads, float scale, float *scores, float *lse, float *img_mass,
                            void *ws, size_t ws_bytes, void *hip_stream, const SelectArgs *select, bool *fused)
{
    if (fused) *fused = false;
    int rc = check_views(kv, bv, n_q_heads);
    if (rc != FASTOCR_OK) return rc;
    rc = check_qo(kv, q, nullptr, scale);
    if (rc != FASTOCR_OK) return rc;
    if (!scores && bv->max_vis_len > 0 && bv->batch > 0) return FASTOCR_EINVAL;
    const size_t need = fastocr_workspace_bytes(FASTOCR_OP_FOCAL_SCORE, kv, bv, n_q_heads, 0);
    rc = check_ws(ws, ws_bytes, need);
    if (rc != FASTOCR_OK) return rc;
    if (bv->batch == 0) return FASTOCR_OK;
    Shape s = make_shape(kv, bv, n_q_heads);
    const int nsplit = choose_splits(FASTOCR_OP_FOCAL_SCORE, s, bv->max_seq_len);
    ResidentPlan rp;
    hipError_t e;
    int slot = -1;
    uint32_t *flag = nullptr;
    if (use_resident(EX_SCORE, g_tune_score_resident.load(std::memory_order_relaxed), s, &rp, kResidentMinTiles, (hipStream_t)hip_stream, &slot, &flag)) {
        const bool fuse = select && g_tune_select_fused.load(std::memory_order_relaxed) != 0 && resident_select_fits(s);
        e = launch_score_resident(s, rp, slot, flag, q, scale, scores, lse, img_mass, ws, (hipStream_t)hip_stream, fuse ? select : nullptr);
        if (fused) *fused = fuse;
    } else {
        e = launch_score(s, q, scale, scores, lse, img_mass, ws, nsplit, (hipStream_t)hip_stream);
    }
    return e == hipSuccess ? FASTOCR_OK : FASTOCR_EHIP;
}

int fastocr_focal_score(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                        int n_q_heads, float scale, float *scores, float *lse, float *img_mass,
                        void *ws, size_t ws_bytes, void *hip_stream)
{
    return focal_score_impl(kv, bv, q, n_q_heads, scale, scores, lse, img_mass, ws, ws_bytes, hip_stream, nullptr, nullptr);
}

int fastocr_focal_score_topk(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                             int n_q_heads, float scale, double tau, const int32_t *prev_idx,
                             const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
                             float *scores, float *lse, float *img_mass, void *ws, size_t ws_bytes,
                             void *hip_stream)
{
    int rc = check_topk_args(scores, bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax);
    if (rc != FASTOCR_OK) return rc;
    const size_t need = fastocr_workspace_bytes(FASTOCR_OP_FOCAL_SCORE_TOPK, kv, bv, n_q_heads, kmax);
    if (need == 0) return check_views(kv, bv, n_q_heads) != FASTOCR_OK ? check_views(kv, bv, n_q_heads) : FASTOCR_EINVAL;
    rc = check_ws(ws, ws_bytes, need);
    if (rc != FASTOCR_OK) return rc;
    const SelectArgs sa{tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax};
    bool fused = false;
    rc = focal_score_impl(kv, bv, q, n_q_heads, scale, scores, lse, img_mass, ws, ws_bytes, hip_stream, &sa, &fused);
    if (rc != FASTOCR_OK || fused) return rc;
    return fastocr_topk_fixation(scores, bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax, ws, ws_bytes, hip_stream);
}

int fastocr_topk_fixation(const float *scores, const fastocr_batch_view *bv, double tau,
                          const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                          int32_t *sel_cnt, int64_t kmax, void *ws, size_t ws_bytes, void *hip_stream)
{
    const int rc0 = check_topk_args(scores, bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax);
    if (rc0 != FASTOCR_OK) return rc0;
    const size_t need = fastocr_workspace_bytes(FASTOCR_OP_TOPK_FIXATION, nullptr, bv, 0, kmax);
    int rc = check_ws(ws, ws_bytes, need);
    if (rc != FASTOCR_OK) return rc;
    if (bv->batch == 0) return FASTOCR_OK;
    BatchDev bd{bv->seq_len, bv->vis_start, bv->vis_len, bv->max_seq_len, bv->max_vis_len};
    hipError_t e = launch_topk(scores, bd, bv->batch, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax,
                               ws, (hipStream_t)hip_stream);
    return e == hipSuccess ? FASTOCR_OK : FASTOCR_EHIP;
}

static int attn_common(int op, const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                       int n_q_heads, float scale, const int32_t *sel_idx, const int32_t *sel_cnt,
                       int64_t kmax, void *out, float *lse, void *ws, size_t ws_bytes, void *hip_stream,
                       bool static_ws = false)
{
    int rc = check_views(kv, bv, n_q_heads);
    if (rc != FASTOCR_OK) return rc;
    if (!out) return FASTOCR_EINVAL;
    rc = check_qo(kv, q, out, scale);
    if (rc != FASTOCR_OK) return rc;
    if (op == FASTOCR_OP_SPARSE_DECODE_ATTN && (!sel_idx || !sel_cnt || kmax < 1)) return FASTOCR_EINVAL;
    const size_t need = fastocr_workspace_bytes(op, kv, bv, n_q_heads, kmax);
    if (static_ws) {
        // the library's own buffer: a shape that needs more than it holds is refused before any GPU call
        if (need > (size_t)FASTOCR_STATIC_SCRATCH_BYTES) return FASTOCR_ETOOLARGE;
        if (bv->batch == 0) return FASTOCR_OK;
        ws = static_scratch_ptr();
        ws_bytes = FASTOCR_STATIC_SCRATCH_BYTES;
        if (!ws) return FASTOCR_EHIP;
    }
    rc = check_ws(ws, ws_bytes, need);
    if (rc != FASTOCR_OK) return rc;
    if (bv->batch == 0) return FASTOCR_OK;
    Shape s = make_shape(kv, bv, n_q_heads);
    bool partials = false;
    const int nsplit = choose_splits(op, s, op == FASTOCR_OP_SPARSE_DECODE_ATTN ? sparse_positions(bv, kmax) : bv->max_seq_len, &partials);
    // the ranges of a stream merged inside the launch: when asked for, the shape fits, the stream has
    // an exchange slot and no such wait has ever been given up in this process (the range count
    // does not depend on the last two, so the workspace the caller sized always covers the
    // separate merge kernel)
    const int mode = g_tune_attn_merge.load(std::memory_order_relaxed);
    int merge_slot = -1;
    uint32_t *flag = nullptr;
    // (never for the static-workspace entry point: the first in-launch merge on a device allocates
    // the pinned "gave up" word)
    if (!static_ws && !partials && ((op == FASTOCR_OP_SPARSE_DECODE_ATTN && mode != 0) || mode == 2) && attn_merges_in_kernel(s, nsplit) && exchange_trusted())
        merge_slot = exchange_slot(EX_MERGE, (hipStream_t)hip_stream, &flag);
    hipError_t e = launch_attn(s, q, scale, sel_idx, sel_cnt, kmax, out, lse, ws, nsplit, merge_slot, flag, (hipStream_t)hip_stream);
    return e == hipSuccess ? FASTOCR_OK : FASTOCR_EHIP;
}

int fastocr_sparse_decode_attn(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                               int n_q_heads, float scale, const int32_t *sel_idx, const int32_t *sel_cnt,
                               int64_t kmax, void *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    return attn_common(FASTOCR_OP_SPARSE_DECODE_ATTN, kv, bv, q, n_q_heads, scale, sel_idx, sel_cnt, kmax,
                       out, nullptr, ws, ws_bytes, hip_stream);
}

int fastocr_dense_decode_attn(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                              int n_q_heads, float scale, void *out, float *lse, void *ws, size_t ws_bytes,
                              void *hip_stream)
{
    return attn_common(FASTOCR_OP_DENSE_DECODE_ATTN, kv, bv, q, n_q_heads, scale, nullptr, nullptr, 0,
                       out, lse, ws, ws_bytes, hip_stream);
}

int fastocr_dense_decode_attn_static(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                                     int n_q_heads, float scale, void *out, float *lse, void *hip_stream)
{
    return attn_common(FASTOCR_OP_DENSE_DECODE_ATTN, kv, bv, q, n_q_heads, scale, nullptr, nullptr, 0,
                       out, lse, nullptr, 0, hip_stream, /*static_ws=*/true);
}

// defer (with *deferred): when the one-pass kernel runs and the top-k that follows can take the merge
// of the output's partials into its own launch, that merge is not launched here but described in *defer.
static int focal_attn_score_impl(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                                 int n_q_heads, float scale, void *out, float *scores, float *lse,
                                 float *img_mass, void *ws, size_t ws_bytes, void *hip_stream,
                                 const SelectArgs *select, bool *fused, CombineArgs *defer = nullptr, bool *deferred = nullptr)
{
    if (fused) *fused = false;
    if (deferred) *deferred = false;
    int rc = check_views(kv, bv, n_q_heads);
    if (rc != FASTOCR_OK) return rc;
    if (!out) return FASTOCR_EINVAL;
    rc = check_qo(kv, q, out, scale);
    if (rc != FASTOCR_OK) return rc;
    if (!scores && bv->max_vis_len > 0 && bv->batch > 0) return FASTOCR_EINVAL;
    const size_t need = fastocr_workspace_bytes(FASTOCR_OP_FOCAL_ATTN_SCORE, kv, bv, n_q_heads, 0);
    rc = check_ws(ws, ws_bytes, need);
    if (rc != FASTOCR_OK) return rc;
    if (bv->batch == 0) return FASTOCR_OK;
    Shape s = make_shape(kv, bv, n_q_heads);
    ResidentPlan rp;
    int slot = -1;
    uint32_t *flag = nullptr;
    if (use_resident(EX_FUSED, g_tune_focal_fused.load(std::memory_order_relaxed), s, &rp, kFusedMinTiles, (hipStream_t)hip_stream, &slot, &flag)) {
        const bool fuse = select && g_tune_select_fused.load(std::memory_order_relaxed) != 0 && resident_select_fits(s);
        const bool hand_on = defer && deferred && !fuse && topk_takes_combine(bv->max_vis_len, kv->head_dim);
        hipError_t e = launch_focal_fused(s, rp, slot, flag, q, scale, out, scores, lse, img_mass, ws, (hipStream_t)hip_stream,
                                          fuse ? select : nullptr, hand_on ? defer : nullptr);
        if (fused) *fused = fuse;
        if (hand_on) *deferred = true;
        return e == hipSuccess ? FASTOCR_OK : FASTOCR_EHIP;
    }
    rc = fastocr_dense_decode_attn(kv, bv, q, n_q_heads, scale, out, nullptr, ws, ws_bytes, hip_stream);
    if (rc != FASTOCR_OK) return rc;
    return focal_score_impl(kv, bv, q, n_q_heads, scale, scores, lse, img_mass, ws, ws_bytes, hip_stream, select, fused);
}

int fastocr_focal_attn_score(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                             int n_q_heads, float scale, void *out, float *scores, float *lse,
                             float *img_mass, void *ws, size_t ws_bytes, void *hip_stream)
{
    return focal_attn_score_impl(kv, bv, q, n_q_heads, scale, out, scores, lse, img_mass, ws, ws_bytes, hip_stream, nullptr, nullptr);
}

int fastocr_focal_attn_score_topk(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                                  int n_q_heads, float scale, double tau, const int32_t *prev_idx,
                                  const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
                                  void *out, float *scores, float *lse, float *img_mass, void *ws,
                                  size_t ws_bytes, void *hip_stream)
{
    int rc = check_topk_args(scores, bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax);
    if (rc != FASTOCR_OK) return rc;
    const size_t need = fastocr_workspace_bytes(FASTOCR_OP_FOCAL_ATTN_SCORE_TOPK, kv, bv, n_q_heads, kmax);
    if (need == 0) return check_views(kv, bv, n_q_heads) != FASTOCR_OK ? check_views(kv, bv, n_q_heads) : FASTOCR_EINVAL;
    rc = check_ws(ws, ws_bytes, need);
    if (rc != FASTOCR_OK) return rc;
    const SelectArgs sa{tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax};
    bool fused = false, deferred = false;
    CombineArgs merge;
    rc = focal_attn_score_impl(kv, bv, q, n_q_heads, scale, out, scores, lse, img_mass, ws, ws_bytes, hip_stream, &sa, &fused,
                               &merge, &deferred);
    if (rc != FASTOCR_OK || fused) return rc;
    if (deferred) {
        // the merge of the output's partials and the top-k both wait for the one-pass kernel only: one launch
        // (the select keeps its keys in registers at these sizes and uses no workspace, the partials stay where they are)
        BatchDev bd{bv->seq_len, bv->vis_start, bv->vis_len, bv->max_seq_len, bv->max_vis_len};
        hipError_t e = launch_topk(scores, bd, bv->batch, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax, ws,
                                   (hipStream_t)hip_stream, &merge);
        return e == hipSuccess ? FASTOCR_OK : FASTOCR_EHIP;
    }
    return fastocr_topk_fixation(scores, bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax, ws, ws_bytes, hip_stream);
}

int fastocr_select_focal_layers(const float *ratio, int steps, int layers, int batch, double rho,
                                int gap, int32_t *focal_out, int32_t *n_out)
{
    if (!ratio || !focal_out || !n_out || steps < 1 || layers < 1 || batch < 1 || gap < 0) return FASTOCR_EINVAL;
    if (!(rho >= 0.0 && rho <= 1.0)) return FASTOCR_EINVAL;
    std::vector<double> mean((size_t)layers, 0.0);
    for (int t = 0; t < steps; ++t)
        for (int i = 0; i < layers; ++i)
            for (int b = 0; b < batch; ++b) {
                const float r = ratio[((size_t)t * layers + i) * batch + b];
                if (!isfinite(r)) return FASTOCR_EINVAL;
                mean[i] += (double)r;
            }
    for (int i = 0; i < layers; ++i) mean[i] /= (double)steps * (double)batch;
    std::vector<int> order((size_t)layers);
    for (int i = 0; i < layers; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return mean[x] > mean[y]; });
    const int budget = (int)floor(rho * (double)layers + 1e-9);
    std::vector<int> taken;
    for (int i : order) {
        if ((int)taken.size() >= budget) break;
        bool far = true;
        for (int j : taken) far = far && abs(i - j) > gap;
        if (far) taken.push_back(i);
    }
    std::sort(taken.begin(), taken.end());
    for (size_t x = 0; x < taken.size(); ++x) focal_out[x] = taken[x];
    *n_out = (int32_t)taken.size();
    return FASTOCR_OK;
}

int fastocr_kernel_timer_enable(int kernel, int capacity)
{
    if (kernel < 0 || kernel >= K_COUNT || capacity < 0) return FASTOCR_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    KernelTimer &t = g_timers[kernel];
    for (int i = 0; i < t.capacity; ++i) {
        (void)hipEventDestroy(t.start[i]);
        (void)hipEventDestroy(t.stop[i]);
    }
    delete[] t.start;
    delete[] t.stop;
    t = KernelTimer();
    if (capacity == 0) return FASTOCR_OK;
    t.start = new hipEvent_t[capacity];
    t.stop = new hipEvent_t[capacity];
    for (int i = 0; i < capacity; ++i) {
        if (hipEventCreate(&t.start[i]) != hipSuccess || hipEventCreate(&t.stop[i]) != hipSuccess) {
            t.capacity = 0;
            return FASTOCR_EHIP;
        }
    }
    t.capacity = capacity;
    return FASTOCR_OK;
}

int fastocr_kernel_timer_read(int kernel, float *ms_out, int max_out)
{
    if (kernel < 0 || kernel >= K_COUNT || (max_out > 0 && !ms_out)) return FASTOCR_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    KernelTimer &t = g_timers[kernel];
    const int n = t.count;
    for (int i = 0; i < n && i < max_out; ++i) {
        if (hipEventSynchronize(t.stop[i]) != hipSuccess) return FASTOCR_EHIP;
        if (hipEventElapsedTime(&ms_out[i], t.start[i], t.stop[i]) != hipSuccess) return FASTOCR_EHIP;
    }
    t.count = 0;
    return n;
}

int fastocr_stream_probe(const void *src, void *dst, size_t bytes, void *sink, void *hip_stream)
{
    if (!src || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u))
        return FASTOCR_EINVAL;
    if (!dst && !sink) return FASTOCR_EINVAL;
    hipError_t e = launch_stream_probe(src, dst, bytes, sink, (hipStream_t)hip_stream);
    return e == hipSuccess ? FASTOCR_OK : FASTOCR_EHIP;
}

int fastocr_stream_release(void *hip_stream)
{
    // the slot numbers of the streams that stay must not move (their calls may be in flight), so a
    // released entry is only marked free and handed to the next stream that asks
    std::lock_guard<std::mutex> lock(g_mu);
    for (int kind = 0; kind < EX_KINDS; ++kind)
        for (int dev = 0; dev < kMaxDevices; ++dev)
            for (SlotOwner &o : g_slots[kind][dev].eager)
                if (!o.free && o.stream == (hipStream_t)hip_stream) o.free = true;
    return FASTOCR_OK;
}

int fastocr_exchange_timeouts(uint64_t *count)
{
    if (!count) return FASTOCR_EINVAL;
    uint32_t a = 0, b = 0, c = 0;
    if (score_resident_timeouts(&a) != hipSuccess || focal_fused_timeouts(&b) != hipSuccess ||
        attn_merge_timeouts(&c) != hipSuccess)
        return FASTOCR_EHIP;
    *count = (uint64_t)a + b + c;
    return FASTOCR_OK;
}

int fastocr_set_tuning(const char *key, int value)
{
    if (!key || value < 0) return FASTOCR_EINVAL;
    if (!strcmp(key, "splits_score")) g_tune_splits[FASTOCR_OP_FOCAL_SCORE] = value;
    else if (!strcmp(key, "splits_sparse")) g_tune_splits[FASTOCR_OP_SPARSE_DECODE_ATTN] = value;
    else if (!strcmp(key, "splits_dense")) g_tune_splits[FASTOCR_OP_DENSE_DECODE_ATTN] = value;
    else if (!strcmp(key, "attn_waves") && (value == 4 || value == 8)) g_tune_attn_waves = value;
    else if (!strcmp(key, "graph_replay") && (value == 0 || value == 1)) g_tune_graph_replay = value;
    else if (!strcmp(key, "timer_every") && value >= 1) g_tune_timer_every = value;
    else if (!strcmp(key, "attn_merge") && value <= 2) g_tune_attn_merge = value;
    else if (!strcmp(key, "barrier_spin_us")) g_tune_barrier_spin_us = value ? value : 250000;
    else if (!strcmp(key, "score_resident") && value <= 2) g_tune_score_resident = value;
    else if (!strcmp(key, "focal_fused") && value <= 2) g_tune_focal_fused = value;
    else if (!strcmp(key, "select_fused") && value <= 1) g_tune_select_fused = value;
    else if (!strcmp(key, "exchange_fallback") && value <= 1) {
        g_exchange_distrusted = value;
        if (value == 0) {
            // re-arm: forget that waves have given up (the caller has taken the other work off the GPU)
            std::lock_guard<std::mutex> lock(g_mu);
            for (int d = 0; d < kMaxDevices; ++d)
                if (g_gave_up[d]) __atomic_store_n(g_gave_up[d], 0u, __ATOMIC_RELAXED);
        }
    }
    else return FASTOCR_EINVAL;
    return FASTOCR_OK;
}

const char *fastocr_strerror(int status)
{
    switch (status) {
    case FASTOCR_OK: return "ok";
    case FASTOCR_EINVAL: return "invalid argument";
    case FASTOCR_EUNSUPPORTED: return "unsupported dtype, head_dim or head count";
    case FASTOCR_EWORKSPACE: return "workspace missing, misaligned or too small";
    case FASTOCR_EHIP: return "HIP runtime error";
    case FASTOCR_ETOOLARGE: return "shape needs more scratch than the library's static buffer holds (FASTOCR_STATIC_SCRATCH_BYTES)";
    default: return "unknown status";
    }
}

const char *fastocr_version(void) { return "fastocr-mi355x 0.1 (gfx950)"; }

}  // extern "C"
