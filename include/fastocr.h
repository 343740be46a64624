/*
 * fastocr.h -- C ABI of the FastOCR per-decode-step hot path for AMD MI355X (gfx950).
 *
 * The path has three steps, repeated at every decode step (Sec. 3, Alg. 1 of the
 * FastOCR paper):
 *   1. fastocr_focal_score        head-averaged attention of the current query over the
 *                                 whole cache, read at the image tokens (Eq. 1, Eq. 2);
 *   2. fastocr_topk_fixation      TopK_{ceil(tau N)} of those scores (Sec. 3.1.2), warm
 *                                 started from the previous step's focal token set
 *                                 (Cross-Step Fixation Reuse, Sec. 3.2);
 *   3. fastocr_sparse_decode_attn attention restricted to the kept set K = T u F
 *                                 (Eq. 2, non-focal branch);
 * plus fastocr_dense_decode_attn, attention over the full cache (Eq. 2, focal branch;
 * also the warm-up steps and the "vanilla" comparator of Table 2).
 *
 * General conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless marked HOST.
 *     The library never allocates, frees, writes or compacts the KV cache: the full cache
 *     stays in place (no eviction).
 *   - Calls validate their arguments on the host, enqueue kernels on `hip_stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and return without
 *     synchronising.  The return value is a fastocr_status; device-side faults are not
 *     reported here.
 *   - `ws` is caller-provided device scratch of at least fastocr_workspace_bytes(...)
 *     bytes, 256-byte aligned, private to the call until the stream reaches its end.
 *   - Single-launch forms.  fastocr_focal_score, fastocr_focal_attn_score and
 *     fastocr_sparse_decode_attn each have a form in which the workgroups of ONE launch hand each
 *     other data through static device memory (see the Concurrency notes at each call), one
 *     "exchange slot" per call in flight.  A slot belongs to a stream: the first 16 streams of a
 *     GPU that use scoring (16 for the focal layer, 4 for pruned attention) keep a slot until
 *     fastocr_stream_release (or the end of the process), and calls in order on one stream share
 *     it safely.  A call that is being
 *     captured into a HIP graph gets a slot of a separate pool (48 / 48 / 12) that belongs to that
 *     capture and stream, so a replay may run next to eager calls on any stream; instantiate a
 *     captured graph once (two instances replayed at the same time would share its slots).  A
 *     stream or capture beyond these counts gets the forms built from separate kernels, which
 *     share nothing.  The library is thread-safe in the sense that calls on different streams may
 *     come from different threads; fastocr_set_tuning and the timers may be called from any thread.
 *     fastocr_topk_fixation keeps no state between or across workgroups at all.
 *   - Sequences are independent.  Sequence b holds seq_len[b] tokens; its image tokens
 *     are the contiguous span [vis_start[b], vis_start[b] + vis_len[b]); every other
 *     position (text before, text after, generated tokens, the current token) is text.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Image-token indices (sel_idx, prev_idx) are relative to the start of the span.
 */
#ifndef FASTOCR_H
#define FASTOCR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FASTOCR_OK = 0,
    FASTOCR_EINVAL = -1,        /* null pointer, negative size, tau outside [0,1], ...   */
    FASTOCR_EUNSUPPORTED = -2,  /* dtype / head_dim / group size the kernels do not cover */
    FASTOCR_EWORKSPACE = -3,    /* ws NULL, misaligned or smaller than required           */
    FASTOCR_EHIP = -4,          /* a HIP runtime call (launch, event) failed              */
    FASTOCR_ETOOLARGE = -5      /* fastocr_dense_decode_attn_static: the shape needs more scratch
                                   than FASTOCR_STATIC_SCRATCH_BYTES                       */
} fastocr_status;

typedef enum { FASTOCR_F32 = 0, FASTOCR_BF16 = 1 } fastocr_dtype;

typedef enum {
    FASTOCR_OP_FOCAL_SCORE = 0,
    FASTOCR_OP_TOPK_FIXATION = 1,
    FASTOCR_OP_SPARSE_DECODE_ATTN = 2,
    FASTOCR_OP_DENSE_DECODE_ATTN = 3,
    FASTOCR_OP_FOCAL_ATTN_SCORE = 4,
    FASTOCR_OP_FOCAL_SCORE_TOPK = 5,
    FASTOCR_OP_FOCAL_ATTN_SCORE_TOPK = 6
} fastocr_op;

/*
 * One layer's KV cache (device memory, read-only for the library).
 * Element (sequence b, token j, kv head g, component c) of K lives at element offset
 *   contiguous (page_tokens == 0):  b*stride_seq + j*stride_token + g*stride_head + c
 *   paged      (page_tokens  > 0):  block_table[b*max_pages_per_seq + j/page_tokens]*stride_page
 *                                   + (j % page_tokens)*stride_token + g*stride_head + c
 * from `k` (same for `v`).  head_dim is contiguous.  Strides are in elements, must be
 * multiples of 8 elements (16-byte rows for bf16) and k, v 16-byte aligned.
 */
typedef struct {
    const void *k;
    const void *v;
    int32_t dtype;              /* fastocr_dtype; Q and the attention output use it too  */
    int32_t n_kv_heads;
    int32_t head_dim;
    int64_t stride_token;
    int64_t stride_head;
    int64_t stride_seq;
    int32_t page_tokens;
    int64_t stride_page;
    const int32_t *block_table; /* DEVICE int32 [batch, max_pages_per_seq]; NULL if contiguous */
    int32_t max_pages_per_seq;
} fastocr_kv_view;

/*
 * Per-sequence geometry: DEVICE int32[batch] arrays plus HOST upper bounds that size the
 * launch grids.  Required: 0 <= vis_start[b], 0 <= vis_len[b], vis_start[b]+vis_len[b] <=
 * seq_len[b] <= max_seq_len, vis_len[b] <= max_vis_len.  The arrays are read on the
 * device only; a sequence that violates the bounds is clamped to them, never read out of
 * range.
 */
typedef struct {
    int32_t batch;
    const int32_t *seq_len;
    const int32_t *vis_start;
    const int32_t *vis_len;
    int32_t max_seq_len;
    int32_t max_vis_len;
} fastocr_batch_view;

/* ceil(tau * n_visual), the size of the focal token set (Sec. 3.1.2), clamped to
 * [0, n_visual].  tau * n is formed in double and a product that exceeds an integer by
 * less than 1e-9 does not round up.  Host function, no GPU involved. */
int64_t fastocr_keep_count(int64_t n_visual, double tau);

/* Bytes of device scratch `op` needs for these shapes (host function; only the host
 * fields of the views are read).  kmax is the row pitch of the selected sets: it sizes the
 * top-k's workspace and bounds the positions pruned attention can attend (a size obtained with a
 * larger kmax, or with kmax = 0, also suffices).  Returns 0 on invalid arguments. */
size_t fastocr_workspace_bytes(int op, const fastocr_kv_view *kv, const fastocr_batch_view *bv,
                               int n_q_heads, int64_t kmax);

/*
 * Step 1 (Eq. 1; text under Eq. 2; softmax of App. B).  For every sequence b and image
 * token i:
 *     scores[b*max_vis_len + i] = (1/n_q_heads) * sum_h softmax_j(scale * <q[b,h], K[b,j,kv(h)]>)[vis_start[b]+i]
 * with the softmax over ALL seq_len[b] cached tokens.  Entries i >= vis_len[b] are not
 * written.
 *   q        [batch, n_q_heads, head_dim], kv->dtype, contiguous, 16-byte aligned
 *   scores   fp32 [batch, max_vis_len]
 *   lse      fp32 [batch, n_q_heads] natural-log sum-exp of each head's logits, or NULL
 *   img_mass fp32 [batch] sum_i scores[b,i] = the image-attention ratio of Eq. 1, or NULL
 * Kernels: bf16 caches with head_dim 128 or 64 and at most 16 query heads per kv head run on the
 * matrix-core kernels (all calls); every other shape (fp32 caches, other head dimensions up to 256,
 * larger groups) runs on plain-FMA kernels that accumulate in fp64, to the same error bars.
 * Concurrency: when the shape fits (bf16, head_dim 128 or 64, 1/2/4/8 kv heads with at most 8 query heads
 * each, batch <= 256 and <= the compute-unit count) this call (and, at head_dim 128, fastocr_focal_attn_score) runs as ONE kernel whose
 * workgroups -- at most one per compute unit -- wait for each other's softmax statistics, so
 * all of them must be on the chip together.  Launched alone on the GPU (any number of calls in
 * order on one stream, HIP graphs included) that always holds.  If other kernels occupy compute
 * units at the same time, a workgroup gives up after 0.25 s and the affected scores are NaN rather
 * than wrong; the give-up is recorded (fastocr_exchange_timeouts) and from then on the library
 * itself takes the forms built from separate kernels for the rest of the process
 * (fastocr_set_tuning("exchange_fallback", 0) re-arms the single-launch forms).  Callers that
 * overlap other GPU work by design should select the separate kernels up front with
 * fastocr_set_tuning("score_resident", 0) and ("focal_fused", 0).
 */
int fastocr_focal_score(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                        int n_q_heads, float scale, float *scores, float *lse, float *img_mass,
                        void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Step 2 (Sec. 3.1.2 TopK; Sec. 3.2 / Alg. 1 reuse of the previous focal token set).
 * For every sequence b: the k_b = fastocr_keep_count(vis_len[b], tau) image tokens with
 * the largest score, ties broken towards the lower index, written to
 * sel_idx[b*kmax + 0..k_b) in ASCENDING index order; sel_cnt[b] = k_b.  Entries beyond
 * k_b are left as they were.
 *   scores   fp32 [batch, max_vis_len] (row pitch max_vis_len)
 *   prev_idx int32 [batch, kmax] / prev_cnt int32 [batch]: last step's set, or both NULL.
 *            Used only to bound the search (the k_b-th best of the old set's current
 *            scores is a lower bound of the new threshold); the result never depends on
 *            it.  A set of the wrong size, out of range or not strictly ascending is
 *            ignored.  prev_idx may alias sel_idx and prev_cnt may alias sel_cnt.
 *   kmax     row pitch of sel_idx / prev_idx; must be >= keep_count(max_vis_len, tau)
 * NaN scores order above every number.
 */
int fastocr_topk_fixation(const float *scores, const fastocr_batch_view *bv, double tau,
                          const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                          int32_t *sel_cnt, int64_t kmax, void *ws, size_t ws_bytes,
                          void *hip_stream);

/*
 * Step 3 (Eq. 2, non-focal branch).  For every sequence b and query head h:
 *     out[b,h,:] = sum_{j in J_b} softmax_{J_b}(scale * <q[b,h], K[b,j,kv(h)]>)[j] * V[b,j,kv(h),:]
 *     J_b = {text positions of b} u {vis_start[b] + sel_idx[b*kmax + r] : 0 <= r < sel_cnt[b]}
 * sel_idx entries must be distinct and inside [0, vis_len[b]); their order is free.
 * An entry outside the span is clamped into it.  An empty J_b gives a zero row.
 *   out  [batch, n_q_heads, head_dim], kv->dtype (bf16 rounded to nearest even), 16-byte aligned;
 *        q as in fastocr_focal_score
 * Concurrency: when a (sequence, kv head) stream is cut into 2 .. 4 ranges (bf16, head_dim 128 or 64, at
 * most 8 query heads per kv head, at most 128 streams) and the call's stream owns an exchange slot,
 * the stream's last workgroup waits for the partial results of the others, which were dispatched
 * before it and wait for nobody.  That wait is microseconds; if it exceeds 0.25 s the affected
 * outputs are NaN rather than wrong, the give-up is recorded and the library takes the separate
 * merge kernel from then on (as for fastocr_focal_score).  A partial published late -- after its
 * call gave up -- carries that call's own number and is never accepted by a later call.
 * fastocr_set_tuning("attn_merge", 0) always selects partials in the workspace and a separate merge
 * kernel.
 */
int fastocr_sparse_decode_attn(const fastocr_kv_view *kv, const fastocr_batch_view *bv,
                               const void *q, int n_q_heads, float scale, const int32_t *sel_idx,
                               const int32_t *sel_cnt, int64_t kmax, void *out, void *ws,
                               size_t ws_bytes, void *hip_stream);

/*
 * Eq. 2, focal branch: the same with J_b = [0, seq_len[b]).
 *   lse  fp32 [batch, n_q_heads] natural-log sum-exp of the logits, or NULL
 */
int fastocr_dense_decode_attn(const fastocr_kv_view *kv, const fastocr_batch_view *bv,
                              const void *q, int n_q_heads, float scale, void *out, float *lse,
                              void *ws, size_t ws_bytes, void *hip_stream);

/*
 * fastocr_dense_decode_attn for callers that cannot provide (or allocate) a workspace: code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results, but the split partials live in a buffer of
 * FASTOCR_STATIC_SCRATCH_BYTES (8 MiB) of static device memory inside the library (each GPU the
 * library runs on holds one such buffer until the process ends).  The call allocates nothing: no
 * hipMalloc / hipFree, no allocating library routine, and the in-launch merge of
 * fastocr_set_tuning("attn_merge", 2) is never taken here.
 *   - Shapes whose partials need more than the buffer (fastocr_workspace_bytes(
 *     FASTOCR_OP_DENSE_DECODE_ATTN, ...) > FASTOCR_STATIC_SCRATCH_BYTES) are refused with
 *     FASTOCR_ETOOLARGE before anything is enqueued; every configuration of the paper's models
 *     needs about 1 MiB.
 *   - All calls on one GPU share that GPU's buffer: calls in order on one stream are safe (every
 *     partial a call reads it has written first, so nothing needs clearing), calls that overlap
 *     on one GPU (different streams, concurrent graph replays) race on it and give wrong outputs.
 */
#define FASTOCR_STATIC_SCRATCH_BYTES (8u << 20)
int fastocr_dense_decode_attn_static(const fastocr_kv_view *kv, const fastocr_batch_view *bv,
                                     const void *q, int n_q_heads, float scale, void *out, float *lse,
                                     void *hip_stream);

/*
 * A focal layer in one call (Alg. 1, focal branch; Eq. 1 and Eq. 2 with the full cache): the
 * dense attention output of fastocr_dense_decode_attn AND the scores, lse and img_mass of
 * fastocr_focal_score for the same q, computed from a single pass over K and V where the
 * shape allows it (bf16, head_dim 128, group size <= 8, 1/2/4/8 KV heads, batch <= compute
 * units, at most 32 tiles of 32 image tokens per wave); other shapes run the two separate
 * kernels one after the other on the same stream, with identical results up to rounding order.
 * Arguments as in those two calls; out and scores are both required, lse and img_mass optional.
 * Workspace: fastocr_workspace_bytes(FASTOCR_OP_FOCAL_ATTN_SCORE, ...).
 */
int fastocr_focal_attn_score(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                             int n_q_heads, float scale, void *out, float *scores, float *lse,
                             float *img_mass, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Steps 1 and 2 in one call (Sec. 3.1.2: TopK_{ceil(tau N)} applied directly to the focal layer's
 * head-averaged attention): fastocr_focal_score followed by fastocr_topk_fixation on its scores, and
 * the same for a whole focal layer (fastocr_focal_attn_score + fastocr_topk_fixation; Alg. 1,
 * focal branch).  Results are those of the separate calls bit for bit (same scores, same exact
 * select).  Arguments as in the separate calls; `scores` is required (it is also the hand-over
 * buffer); prev_idx / sel_idx may alias.
 * Workspace: fastocr_workspace_bytes(FASTOCR_OP_FOCAL_SCORE_TOPK | FASTOCR_OP_FOCAL_ATTN_SCORE_TOPK, ..., kmax).
 * By default the two steps run as two launches one after the other on the stream.  With
 * fastocr_set_tuning("select_fused", 1), when scoring runs as its single register-resident kernel
 * and no image span exceeds 16384 tokens, the select runs INSIDE that launch: every range stores
 * its scores at agent scope and counts itself out, and the sequence's last range to finish selects
 * over the whole sequence -- no second launch, nobody waits.  That form is measured slower on
 * MI355X (the select then runs on 8 waves instead of 16 and ends the launch alone), so it is not
 * the default.
 * fastocr_focal_attn_score_topk by default: when the layer runs as its one-pass kernel and no image span
 * exceeds 16384 tokens, the merge of the dense output's partials is done by extra workgroups of the
 * select's launch (both depend on the one-pass kernel only): two launches instead of three, same bits.
 */
int fastocr_focal_score_topk(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                             int n_q_heads, float scale, double tau, const int32_t *prev_idx,
                             const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
                             float *scores, float *lse, float *img_mass, void *ws, size_t ws_bytes,
                             void *hip_stream);
int fastocr_focal_attn_score_topk(const fastocr_kv_view *kv, const fastocr_batch_view *bv, const void *q,
                                  int n_q_heads, float scale, double tau, const int32_t *prev_idx,
                                  const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
                                  void *out, float *scores, float *lse, float *img_mass, void *ws,
                                  size_t ws_bytes, void *hip_stream);

/*
 * Focal Layer Selection (Sec. 3.1.1; first block of Alg. 1).  HOST function, no GPU involved.
 *   ratio  HOST fp32 [steps][layers][batch]: the image-attention ratio r_i^(t) of Eq. 1 of layer i
 *          at warm-up step t for sequence b -- what fastocr_focal_score returns in img_mass
 *          (the softmax runs over image and text positions together, so the ratio's
 *          denominator is 1).
 * Layers are ranked by the mean of their ratio over steps and batch (one focal set serves the
 * whole batch), descending, equal means in layer order; they are taken greedily while fewer
 * than floor(rho * layers) are taken and the layer is more than `gap` layers away from every
 * layer already taken.  The chosen layers are written ascending to focal_out[0 .. *n_out)
 * (HOST int32, room for `layers` entries).  The mean is formed in double; rho * layers within
 * 1e-9 below an integer counts as that integer.
 * Returns FASTOCR_EINVAL for null pointers, steps/layers/batch < 1, rho outside [0,1], gap < 0
 * or a non-finite ratio.
 */
int fastocr_select_focal_layers(const float *ratio, int steps, int layers, int batch, double rho,
                                int gap, int32_t *focal_out, int32_t *n_out);

/*
 * Per-kernel timing with HIP events recorded on the stream the kernel is launched on.
 * fastocr_kernel_timer_enable(kernel, capacity) makes every later launch of that kernel
 * record a start/stop event pair (up to `capacity` launches; capacity 0 disables and
 * frees the events).  fastocr_kernel_timer_read synchronises the recorded events and
 * writes up to `max_out` durations in milliseconds to the HOST array `ms_out`; returns
 * the number of launches recorded so far (or a negative status) and resets the count.
 * An event pair costs the stream a few microseconds per launch (measured: 4.5 us per step with
 * one timed kernel); fastocr_set_tuning("timer_every", n) makes only every n-th launch of a
 * timed kernel, counted from fastocr_kernel_timer_enable, carry one.
 */
typedef enum {
    FASTOCR_KERNEL_SCORE_LOGITS = 0,   /* streams K: logits + per-split softmax statistics */
    FASTOCR_KERNEL_SCORE_FINALIZE = 1,
    FASTOCR_KERNEL_TOPK = 2,
    FASTOCR_KERNEL_SPARSE_ATTN = 3,
    FASTOCR_KERNEL_DENSE_ATTN = 4,
    FASTOCR_KERNEL_ATTN_COMBINE = 5,
    FASTOCR_KERNEL_FOCAL_FUSED = 6,    /* one pass over K and V: attention partials + scores */
    FASTOCR_KERNEL_COUNT = 7
} fastocr_kernel;

int fastocr_kernel_timer_enable(int kernel, int capacity);
int fastocr_kernel_timer_read(int kernel, float *ms_out, int max_out);

/*
 * Measurement helper, not part of the method: a plain streaming kernel of known size.
 * dst != NULL copies `bytes` (rounded down to 16) from src to dst; dst == NULL only reads
 * src (`sink`, 4 device bytes, is then required and practically never written).  Used for the
 * measured HBM ceiling and to calibrate the profiler's fetch/write byte counters.
 * src, dst 16-byte aligned device pointers.
 */
int fastocr_stream_probe(const void *src, void *dst, size_t bytes, void *sink, void *hip_stream);

/* Launch-shape overrides for measurement sweeps and deployment choices (value >= 0):
 *   "splits_score" | "splits_dense" | "splits_sparse"   ranges per stream; 0 = automatic
 *   "score_resident" | "focal_fused"   0 = always the separate kernels; 1 = chosen by the library
 *       (default: the single-kernel form whenever the shape fits, the stream has an exchange slot
 *       and no wave of such a form has ever given up waiting in this process); 2 = the
 *       single-kernel form whenever the shape fits and the stream has a slot
 *   "attn_waves"      4 | 8: waves per workgroup of attention launches that leave partials
 *   "attn_merge"      pruned attention with several ranges per stream: 1 = merged inside the launch
 *       (default, under the same conditions as above), 0 = by a second kernel, 2 = dense attention
 *       merges inside the launch too (measured slower, kept for comparison)
 *   "graph_replay"    1 = the caller replays its calls from a HIP graph, where a launch starts well under a
 *       microsecond after the one before: pruned attention over short lists of few streams (as long as
 *       every workgroup of the cut finds a compute unit) is then cut into one tile per wave and merged by
 *       a second kernel; 0 (default) = calls are launched one by one, such lists stay one launch.  The
 *       workspace size covers both, results agree to rounding.
 *   "select_fused"    fastocr_focal_score_topk / fastocr_focal_attn_score_topk: 0 = the select is a launch of
 *       its own (default), 1 = it runs inside the scoring launch when it can
 *   "timer_every"     n >= 1: see the kernel timers above
 *   "barrier_spin_us" how long a workgroup of a single-launch form waits for the others; 0 restores
 *       the default of 250000; 1 makes waiting workgroups give up at once (tests use it to exercise
 *       the NaN path; every kernel still ends normally)
 *   "exchange_fallback"  1 = treat the single-launch forms as distrusted (as after a give-up);
 *       0 = forget every recorded give-up and trust them again
 * Returns FASTOCR_EINVAL for an unknown key or a value outside the key's range.  Values are read
 * by later calls; workspace sizes must be asked for after the split and merge keys are set. */
int fastocr_set_tuning(const char *key, int value);

/*
 * Gives back the exchange slots a stream holds on every GPU (see "Single-launch forms" above), e.g.
 * before the stream is destroyed, so that other streams can have them.  No call of this library
 * may be in flight on the stream, and HIP graphs captured on it keep their own slots.  A stream
 * that calls the library again afterwards simply gets slots anew.  Host function; always
 * FASTOCR_OK (a stream that holds nothing is not an error).
 */
int fastocr_stream_release(void *hip_stream);

/*
 * For the callers of the single-launch forms (see the Concurrency notes above): how many waves
 * have given up waiting for another workgroup of their own launch since the library was loaded
 * (each such wave left NaN in what it could not finish).  0 in any run where those launches had
 * the GPU to themselves.  Copies three counters from the device: synchronises with it, so not
 * for use under stream capture.  count: host pointer.
 */
int fastocr_exchange_timeouts(uint64_t *count);

const char *fastocr_strerror(int status);
const char *fastocr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTOCR_H */
