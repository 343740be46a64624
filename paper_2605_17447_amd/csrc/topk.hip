// TopK_{ceil(tau N)} over one sequence's image scores (Sec. 3.1.2), exact and deterministic,
// warm-started from the previous step's focal token set (Cross-Step Fixation Reuse, Sec. 3.2).
//
// One 1024-thread workgroup per sequence; the scores become order-preserving 32-bit keys held
// in LDS.  The k-th largest key (the threshold) is found by an MSB-first 8-bit radix select.
// Warm start: the smallest current key among the previous set's k tokens is a lower bound of
// the new threshold (k tokens reach it), so only the candidates at or above it -- usually
// little more than k of them, because the fixation moves slowly -- enter the radix select.
// The threshold, and therefore the result, is the same as without the previous set; a stale
// set only makes the candidate list long, and past a cap the select runs over all N keys.
// The final pass writes every key above the threshold, and the lowest-index keys equal to it
// until k are written, in ascending index order (ballot/popcount compaction per wave).
#include "kernels.hpp"

namespace fastocr {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kCandCap = 4096;
constexpr int kLdsKeyCap = 32768;

__device__ __forceinline__ uint32_t order_key(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u << 1) == 0u) u = 0u;                 // -0.0 compares equal to +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int keep_count_dev(int n, double tau)
{
#pragma clang fp contract(off)
    if (n <= 0 || !(tau > 0.0)) return 0;
    double x = ceil(tau * (double)n - 1e-9);
    if (x < 0.0) x = 0.0;
    if (x > (double)n) x = (double)n;
    return (int)x;
}

// k-th largest (1-based rank `k`) of keys[0..n): returns the threshold key and, through
// *ties_needed, how many keys equal to it belong to the top k.  All threads must call.
__device__ uint32_t radix_select(const uint32_t *keys, int n, int k, uint32_t *hist, int *s_pick,
                                 int *ties_needed)
{
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t prefix = 0u, mask = 0u;
    int kk = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0u;
        __syncthreads();
        for (int i0 = 0; i0 < n; i0 += kTopkThreads) {
            const int i = i0 + tid;
            const bool in = i < n;
            const uint32_t key = in ? keys[i] : 0u;
            const bool live = in && ((key & mask) == prefix);
            const uint32_t dgt = (key >> shift) & 255u;
            // a whole wave on one digit (the usual case for the exponent byte) adds once
            const uint64_t live_mask = __ballot(live);
            if (live_mask) {
                const int first = __ffsll((long long)live_mask) - 1;
                const uint32_t d0 = __shfl(dgt, first);
                const uint64_t same = __ballot(live && dgt == d0);
                if (same == live_mask) {
                    if (lane == first) atomicAdd(&hist[d0], (uint32_t)__popcll(live_mask));
                } else if (live) {
                    atomicAdd(&hist[dgt], 1u);
                }
            }
        }
        __syncthreads();
        if (tid < 64) {
            // lane owns digits 255-4*lane .. 252-4*lane (descending)
            uint32_t c[4], tot = 0u;
#pragma unroll
            for (int x = 0; x < 4; ++x) { c[x] = hist[255 - (4 * lane + x)]; tot += c[x]; }
            uint32_t incl = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            const uint32_t above = incl - tot;           // keys in strictly larger digits
            if (above < (uint32_t)kk && incl >= (uint32_t)kk) {
                // the k-th key falls into one of this lane's four digits
                uint32_t run = above;
                for (int x = 0; x < 4; ++x) {
                    if (run + c[x] >= (uint32_t)kk) {
                        s_pick[0] = 255 - (4 * lane + x);
                        s_pick[1] = kk - (int)run;
                        break;
                    }
                    run += c[x];
                }
            }
        }
        __syncthreads();
        prefix |= ((uint32_t)s_pick[0]) << shift;
        mask |= 255u << shift;
        kk = s_pick[1];
        __syncthreads();
    }
    *ties_needed = kk;
    return prefix;
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(
    const float *__restrict__ scores, BatchDev bv, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
    uint32_t *__restrict__ gkeys, int lds_keys)
{
    extern __shared__ uint32_t dyn_keys[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t cand[kCandCap];
    __shared__ int s_pick[2];
    __shared__ uint32_t s_theta0;
    __shared__ int s_bad, s_ncand;
    __shared__ int w_gt[kTopkWaves], w_eq[kTopkWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const SeqGeom geo = seq_geom(bv, b);
    const int N = geo.N;
    const int k = (int)min((int64_t)keep_count_dev(N, tau), kmax);
    const int pcnt = prev_cnt ? prev_cnt[b] : -1;
    int32_t *out = sel_idx + (int64_t)b * kmax;

    if (k <= 0) {
        if (tid == 0) sel_cnt[b] = 0;
        return;
    }
    if (k >= N) {
        for (int i = tid; i < N; i += kTopkThreads) out[i] = i;
        if (tid == 0) sel_cnt[b] = N;
        return;
    }

    uint32_t *keys = (N <= lds_keys) ? dyn_keys : (gkeys + (int64_t)b * bv.max_vis_len);
    const float *srow = scores + (int64_t)b * bv.max_vis_len;
    for (int i = tid; i < N; i += kTopkThreads) keys[i] = order_key(srow[i]);
    if (tid == 0) { s_theta0 = 0xffffffffu; s_bad = 0; s_ncand = 0; }
    __syncthreads();

    uint32_t theta;
    int ties;
    bool have = false;
    if (prev_idx && pcnt == k) {
        // lower bound of the threshold from the previous set (must be k distinct valid tokens)
        const int32_t *prev = prev_idx + (int64_t)b * kmax;
        uint32_t lo = 0xffffffffu;
        int bad = 0;
        for (int r = tid; r < k; r += kTopkThreads) {
            const int i = prev[r];
            const int nx = (r + 1 < k) ? prev[r + 1] : 0x7fffffff;
            if (i < 0 || i >= N || i >= nx) bad = 1;
            else lo = min(lo, keys[i]);
        }
        if (bad) s_bad = 1;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, o));
        if (lane == 0) atomicMin(&s_theta0, lo);
        __syncthreads();
        if (!s_bad) {
            const uint32_t th0 = s_theta0;
            for (int i0 = 0; i0 < N; i0 += kTopkThreads) {
                const int i = i0 + tid;
                const bool c = (i < N) && keys[i] >= th0;
                const uint64_t mk = __ballot(c);
                int base = 0;
                if (lane == 0 && mk) base = atomicAdd(&s_ncand, __popcll(mk));
                base = __shfl(base, 0);
                if (c) {
                    const int pos = base + __popcll(mk & ((1ull << lane) - 1ull));
                    if (pos < kCandCap) cand[pos] = keys[i];
                }
            }
            __syncthreads();
            const int nc = s_ncand;
            if (nc <= kCandCap) {                          // nc >= k by construction
                theta = radix_select(cand, nc, k, hist, s_pick, &ties);
                have = true;
            }
        }
    }
    if (!have) theta = radix_select(keys, N, k, hist, s_pick, &ties);

    // ---- ordered compaction: each wave owns a contiguous index segment ----------------------
    const int seg = ((N + kTopkWaves - 1) / kTopkWaves + 63) / 64 * 64;
    const int s0 = wave * seg, s1 = min(N, s0 + seg);
    int ngt = 0, neq = 0;
    for (int i = s0 + lane; i < s1; i += 64) {
        const uint32_t key = keys[i];
        ngt += key > theta;
        neq += key == theta;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { ngt += __shfl_xor(ngt, o); neq += __shfl_xor(neq, o); }
    if (lane == 0) { w_gt[wave] = ngt; w_eq[wave] = neq; }
    __syncthreads();
    int eq_seen = 0, out_pos = 0;
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
    if (tid == 0) sel_cnt[b] = k;
}

size_t topk_workspace_bytes(int batch, int max_vis_len)
{
    if (max_vis_len <= kLdsKeyCap) return 0;
    return (size_t)batch * (size_t)max_vis_len * sizeof(uint32_t);
}

hipError_t launch_topk(const float *scores, const BatchDev &bv, int batch, double tau,
                       const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                       int32_t *sel_cnt, int64_t kmax, void *ws, hipStream_t stream)
{
    const int lds_keys = bv.max_vis_len <= kLdsKeyCap ? bv.max_vis_len : 0;
    const size_t dyn = (size_t)lds_keys * sizeof(uint32_t);
    static bool attr_set = false;
    if (!attr_set) {
        // gfx950 has 160 KB of LDS per workgroup; the keys of up to 32768 tokens take 128 KB.
        // If the runtime refuses the opt-in, a launch that needs it reports the error itself.
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(topk_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsKeyCap * (int)sizeof(uint32_t)) != hipSuccess)
            (void)hipGetLastError();
        attr_set = true;
    }
    FASTOCR_LAUNCH(K_TOPK, topk_kernel, dim3(batch), dim3(kTopkThreads), dyn, stream, scores, bv, tau, prev_idx,
                   prev_cnt, sel_idx, sel_cnt, kmax, reinterpret_cast<uint32_t *>(ws), lds_keys);
    return hipGetLastError();
}

}  // namespace fastocr
