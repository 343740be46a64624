// TopK_{ceil(tau N)} over one sequence's image scores (Sec. 3.1.2), exact and deterministic,
// warm-started from the previous step's focal token set (Cross-Step Fixation Reuse, Sec. 3.2).
//
// The scores become order-preserving 32-bit keys; the k-th largest key (the threshold) is found
// exactly; everything above it, plus the lowest-index keys equal to it until k, is written in
// ascending index order.  The previous step's set -- the warm start -- gives a lower bound of the
// threshold (its k tokens' smallest current key can only be at or below it) that shortens the
// search; the result never depends on it.
//   Image spans up to 16384 tokens (topk_reg_kernel): one workgroup per sequence with all keys in
//   registers; the threshold comes from histogram passes over a window of key values that starts at
//   the bound (topk_dev.hpp).
//   Longer spans (topk_general_kernel): keys in LDS or in the workspace, an MSB-first 8-bit radix
//   select over a candidate list, the writing spread over several workgroups per sequence.

#include "topk_dev.hpp"
#include "combine.hpp"

namespace fastocr {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kCandCap = 4096;
constexpr int kLdsKeyCap = 24576;

// General form, for image spans beyond the register-resident kernel below.
// Grid (parts, batch).  The workgroups of a sequence do not talk to each other: each one loads ALL
// of the sequence's keys into LDS (64 KB at N = 16384, read from cache), finds the exact threshold
// for itself and writes only its own contiguous segment of the ascending result, at the position
// that the count of selected tokens before the segment gives.  Redundant arithmetic is cheap here;
// a candidate list handed from workgroup to workgroup through memory costs several dependent
// round trips.  The threshold search is shortened by a lower bound theta0 of the threshold:
//   theta0 = max(bound from the previous set, bound from a sample)
//   previous set (warm start): the smallest current key among its k tokens -- a certain bound
//     (k tokens reach it), tight when the fixation moved little;
//   sample: the r-th largest of 1024 evenly spaced scores, r chosen so that about 1.5 k tokens
//     reach it -- a likely bound only.
// Keys at or above theta0 are compacted into a candidate list; if at least k and at most kCandCap
// came in, the k largest overall are among them and the radix select runs over the candidates,
// otherwise over all N keys: the result is the same in every case.
// Image spans whose keys do not fit LDS run as one workgroup per sequence with the keys in the
// workspace.
__global__ __launch_bounds__(kTopkThreads) void topk_general_kernel(
    const float *__restrict__ scores, BatchDev bv, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
    uint32_t *__restrict__ gkeys, int lds_keys)
{
    extern __shared__ uint32_t dyn_keys[];
    __shared__ uint32_t hist[2][256];
    __shared__ uint32_t cand[kCandCap];
    __shared__ uint32_t cand_i[kCandCap];
    __shared__ int s_pick[2];
    __shared__ uint32_t s_theta_prev;
    __shared__ int s_bad, s_ncand;
    __shared__ int w_gt[kTopkWaves], w_eq[kTopkWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int part = blockIdx.x, nparts = gridDim.x, b = blockIdx.y;
    const SeqGeom geo = seq_geom(bv, b);
    const int N = geo.N;
    const int k = (int)min((int64_t)keep_count_dev(N, tau), kmax);
    const int pcnt = prev_cnt ? prev_cnt[b] : -1;
    int32_t *out = sel_idx + (int64_t)b * kmax;
    const float *srow = scores + (int64_t)b * bv.max_vis_len;

    if (k <= 0 || k >= N) {
        // nothing to select: the first workgroup writes the trivial set
        if (part == 0) {
            if (k >= N && k > 0)
                for (int i = tid; i < N; i += kTopkThreads) out[i] = i;
            if (tid == 0) sel_cnt[b] = k <= 0 ? 0 : N;
        }
        return;
    }

    if (tid == 0) { s_theta_prev = 0xffffffffu; s_bad = 0; s_ncand = 0; }
    const bool in_lds = N <= lds_keys;
    uint32_t *keys = in_lds ? dyn_keys : (gkeys + (int64_t)b * bv.max_vis_len);
    for (int i = tid; i < N; i += kTopkThreads) keys[i] = order_key(srow[i]);
    // ---- bound from the previous set: k distinct valid tokens (strictly ascending) or ignored ----
    const bool have_prev = in_lds && prev_idx && pcnt == k;
    uint32_t lo = 0xffffffffu;
    int bad = 0;
    if (have_prev) {
        const int32_t *prev = prev_idx + (int64_t)b * kmax;
        for (int r = tid; r < k; r += kTopkThreads) {
            const int i = prev[r];
            const int nx = (r + 1 < k) ? prev[r + 1] : 0x7fffffff;
            if (i < 0 || i >= N || i >= nx) bad = 1;
            else lo = min(lo, order_key(srow[i]));
        }
    }
    __syncthreads();

    uint32_t theta;
    int ties;
    bool from_cand = false;
    int nc = 0;
    if (in_lds) {
        uint32_t theta0 = 0u;
        if (have_prev) {
            if (bad) s_bad = 1;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, o));
            if (lane == 0) atomicMin(&s_theta_prev, lo);
            __syncthreads();
            if (!s_bad) theta0 = s_theta_prev;
        }
        // ---- bound from a sample of kTopkThreads evenly spaced scores -----------------------------
        {
            const int ns = min(N, kTopkThreads);
            if (tid < ns) cand[tid] = keys[(int)(((int64_t)tid * N) / ns)];
            __syncthreads();
            // about 1.5 k of the N tokens should reach the bound: rank 1.5 k ns / N in the sample, plus slack
            const int r = (int)(((int64_t)3 * k * ns) / ((int64_t)2 * N)) + 24;
            if (r < ns) {
                int unused;
                // the upper 16 bits are enough for a bound (fp32: sign, exponent, 7 mantissa bits)
                const uint32_t ths = radix_select<kTopkThreads>(cand, ns, r, hist, s_pick, &unused, 16);
                theta0 = max(theta0, ths);
            }
            __syncthreads();
        }
        // ---- candidates: every key of the sequence at or above the bound ---------------------------
        for (int i0 = 0; i0 < N; i0 += kTopkThreads) {
            const int ii = i0 + tid;
            const uint32_t key = ii < N ? keys[ii] : 0u;
            const bool c = ii < N && key >= theta0;
            const uint64_t mk = __ballot(c);
            int base = 0;
            if (lane == 0 && mk) base = atomicAdd(&s_ncand, __popcll(mk));
            base = __shfl(base, 0);
            if (c) {
                const int pos = base + __popcll(mk & ((1ull << lane) - 1ull));
                if (pos < kCandCap) { cand[pos] = key; cand_i[pos] = (uint32_t)ii; }
            }
        }
        __syncthreads();
        nc = s_ncand;
        from_cand = nc >= k && nc <= kCandCap;
    }
    if (from_cand) theta = radix_select<kTopkThreads>(cand, nc, k, hist, s_pick, &ties);
    else theta = radix_select<kTopkThreads>(keys, N, k, hist, s_pick, &ties);

    // ---- this workgroup's segment of the token range, and how much of the result precedes it ------
    const int seg = ((N + nparts - 1) / nparts + 63) / 64 * 64;
    const int p0 = min(N, part * seg), p1 = min(N, p0 + seg);
    int ngt = 0, neq = 0;
    if (from_cand) {
        for (int c = tid; c < nc; c += kTopkThreads) {
            const bool before = (int)cand_i[c] < p0;
            ngt += before && cand[c] > theta;
            neq += before && cand[c] == theta;
        }
    } else {
        for (int i = tid; i < p0; i += kTopkThreads) {
            const uint32_t key = keys[i];
            ngt += key > theta;
            neq += key == theta;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { ngt += __shfl_xor(ngt, o); neq += __shfl_xor(neq, o); }
    if (lane == 0) { w_gt[wave] = ngt; w_eq[wave] = neq; }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int w = 0; w < kTopkWaves; ++w) { gt_before += w_gt[w]; eq_before += w_eq[w]; }
    __syncthreads();

    // ---- ordered compaction of the segment: each wave owns a contiguous piece of it ---------------
    const int wseg = ((p1 - p0 + kTopkWaves - 1) / kTopkWaves + 63) / 64 * 64;
    const int s0 = min(p1, p0 + wave * wseg), s1 = min(p1, s0 + wseg);
    ngt = 0;
    neq = 0;
    for (int i = s0 + lane; i < s1; i += 64) {
        const uint32_t key = keys[i];
        ngt += key > theta;
        neq += key == theta;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { ngt += __shfl_xor(ngt, o); neq += __shfl_xor(neq, o); }
    if (lane == 0) { w_gt[wave] = ngt; w_eq[wave] = neq; }
    __syncthreads();
    // ties go to the lowest indices: the first `ties` keys equal to the threshold are taken
    int eq_seen = eq_before, out_pos = gt_before + min(ties, eq_before);
    for (int w = 0; w < wave; ++w) {
        out_pos += w_gt[w] + min(max(ties - eq_seen, 0), w_eq[w]);
        eq_seen += w_eq[w];
    }
    for (int i0 = s0; i0 < s1; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = (i < s1) ? keys[i] : 0u;
        const bool is_eq = (i < s1) && key == theta;
        const bool is_gt = (i < s1) && key > theta;
        const uint64_t below = (1ull << lane) - 1ull;
        const uint64_t eq_mask = __ballot(is_eq);
        const bool take = is_gt || (is_eq && eq_seen + __popcll(eq_mask & below) < ties);
        const uint64_t tk_mask = __ballot(take);
        if (take) out[out_pos + __popcll(tk_mask & below)] = i;
        eq_seen += __popcll(eq_mask);
        out_pos += __popcll(tk_mask);
    }
    if (part == 0 && tid == 0) sel_cnt[b] = k;
}

constexpr int kTopkPer = 16;
constexpr int kTopkRegKeys = kTopkThreads * kTopkPer;

// VEC: every row of scores starts 16-byte aligned and holds whole 16-byte pieces.  PER: keys per
// thread, the fewest that hold the longest image span (every per-key instruction is executed by all
// sixteen waves whether their keys are real or padding: at 4096 tokens, 16 keys per thread would be
// four times the work).
template <bool VEC, int PER>
__global__ __launch_bounds__(kTopkThreads) void topk_reg_kernel(
    const float *__restrict__ scores, BatchDev bv, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax)
{
    __shared__ uint32_t hist[kWinBins];
    __shared__ __align__(16) uint32_t list[kWinListWords];
    __shared__ int s_pick[4];
    __shared__ __align__(16) int w_ac[4 * kTopkWaves];

    TopkRegShared sh;
    sh.hist = hist; sh.list = list; sh.pick = s_pick; sh.w_ac = w_ac;
    topk_reg_body<kTopkThreads, PER, false, VEC>(scores, bv, blockIdx.x, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax, sh,
                                          [](int, int) {});
}

// The same, with batch * Hq more workgroups behind the selecting ones: each merges the attention
// partials of one (sequence, query head) of the focal layer whose scores are being selected from.
// The two kinds of workgroup share nothing but the launch.
template <bool VEC, int PER>
__global__ __launch_bounds__(kTopkThreads) void focal_tail_kernel(
    const float *__restrict__ scores, BatchDev bv, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax, int batch, CombineArgs c)
{
    __shared__ uint32_t hist[kWinBins];
    __shared__ __align__(16) uint32_t list[kWinListWords];
    __shared__ int s_pick[4];
    __shared__ __align__(16) int w_ac[4 * kTopkWaves];
    __shared__ float sm_max[4];
    __shared__ float sm_z[256];
    __shared__ __align__(16) float sm_o[1024];

    if ((int)blockIdx.x < batch) {
        TopkRegShared sh;
        sh.hist = hist; sh.list = list; sh.pick = s_pick; sh.w_ac = w_ac;
        topk_reg_body<kTopkThreads, PER, false, VEC>(scores, bv, blockIdx.x, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax, sh,
                                              [](int, int) {});
    } else {
        const int x = (int)blockIdx.x - batch;
        const int b = x / c.n_q_heads, h = x - b * c.n_q_heads;
        combine_wide_body<uint16_t>(c.part_o, c.part_ml, c.nsplit, c.d, c.out, nullptr, c.seq_meta, c.wpk, h, b, c.n_q_heads,
                                    CombineShared{sm_max, sm_z, sm_o});
    }
}

bool topk_takes_combine(int max_vis_len, int head_dim) { return max_vis_len > 0 && max_vis_len <= kTopkRegKeys && head_dim % 4 == 0 && head_dim <= 256; }

// Workgroups per sequence: one per 1024 image tokens, as long as the grid still fits the chip in
// one round (each workgroup occupies a compute unit with its keys in LDS).
static int topk_parts(int batch, int max_vis_len)
{
    if (max_vis_len > kLdsKeyCap) return 1;
    const int by_size = (max_vis_len + kTopkThreads - 1) / kTopkThreads;
    const int by_chip = 256 / max(1, batch);
    return max(1, min(by_size, by_chip));
}

// Workspace: the keys of image spans that do not fit LDS, uint32 [batch][max_vis_len].
size_t topk_workspace_bytes(int batch, int max_vis_len)
{
    size_t bytes = 0;
    if (max_vis_len > kLdsKeyCap) bytes += (size_t)batch * (size_t)max_vis_len * sizeof(uint32_t);
    return (bytes + 255) / 256 * 256;
}

hipError_t launch_topk(const float *scores, const BatchDev &bv, int batch, double tau,
                       const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                       int32_t *sel_cnt, int64_t kmax, void *ws, hipStream_t stream, const CombineArgs *combine)
{
    if (combine && !topk_takes_combine(bv.max_vis_len, combine->d)) return hipErrorInvalidValue;
    const int lds_keys = bv.max_vis_len <= kLdsKeyCap ? bv.max_vis_len : 0;
    const size_t dyn = (size_t)lds_keys * sizeof(uint32_t);
    // once per device: the opt-in belongs to the device's copy of the code
    static bool attr_set_on[64] = {false};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    bool &attr_set = attr_set_on[dev];
    if (!attr_set) {
        // gfx950 has 160 KB of LDS per workgroup; the keys of up to 24576 tokens take 96 KB next to
        // the static candidate arrays.  If the runtime refuses the opt-in, a launch that needs it
        // reports the error itself.
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(topk_general_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsKeyCap * (int)sizeof(uint32_t)) != hipSuccess)
            (void)hipGetLastError();
        attr_set = true;
    }
    if (bv.max_vis_len <= kTopkRegKeys) {
        const bool vec = (reinterpret_cast<uintptr_t>(scores) & 15u) == 0 && (bv.max_vis_len & 3) == 0;
#define FASTOCR_TOPK_REG(V, P) FASTOCR_LAUNCH(K_TOPK, (topk_reg_kernel<V, P>), dim3(batch), dim3(kTopkThreads), 0, stream, scores, \
                                              bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax)
        if (combine) {
            const dim3 grid(batch + batch * combine->n_q_heads);
#define FASTOCR_TAIL(V, P) FASTOCR_LAUNCH(K_TOPK, (focal_tail_kernel<V, P>), grid, dim3(kTopkThreads), 0, stream, scores, \
                                          bv, tau, prev_idx, prev_cnt, sel_idx, sel_cnt, kmax, batch, *combine)
            if (bv.max_vis_len <= kTopkThreads * 4) { if (vec) FASTOCR_TAIL(true, 4); else FASTOCR_TAIL(false, 4); }
            else if (bv.max_vis_len <= kTopkThreads * 8) { if (vec) FASTOCR_TAIL(true, 8); else FASTOCR_TAIL(false, 8); }
            else { if (vec) FASTOCR_TAIL(true, kTopkPer); else FASTOCR_TAIL(false, kTopkPer); }
#undef FASTOCR_TAIL
            return hipGetLastError();
        }
        if (bv.max_vis_len <= kTopkThreads * 4) { if (vec) FASTOCR_TOPK_REG(true, 4); else FASTOCR_TOPK_REG(false, 4); }
        else if (bv.max_vis_len <= kTopkThreads * 8) { if (vec) FASTOCR_TOPK_REG(true, 8); else FASTOCR_TOPK_REG(false, 8); }
        else { if (vec) FASTOCR_TOPK_REG(true, kTopkPer); else FASTOCR_TOPK_REG(false, kTopkPer); }
#undef FASTOCR_TOPK_REG
        return hipGetLastError();
    }
    uint32_t *gkeys = reinterpret_cast<uint32_t *>(ws);
    // Several workgroups per sequence write their segments while others may still be reading the
    // previous set: not when that set lives in the buffer being written.
    const size_t span = (size_t)batch * (size_t)kmax;
    const bool aliased = prev_idx && prev_idx < sel_idx + span && sel_idx < prev_idx + span;
    const int parts = aliased ? 1 : topk_parts(batch, bv.max_vis_len);
    FASTOCR_LAUNCH(K_TOPK, topk_general_kernel, dim3(parts, batch), dim3(kTopkThreads), dyn, stream, scores, bv, tau, prev_idx,
                   prev_cnt, sel_idx, sel_cnt, kmax, gkeys, lds_keys);
    return hipGetLastError();
}

}  // namespace fastocr
