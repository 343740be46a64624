// Device code of the exact top-k select as templates (workgroup size and keys per thread are
// parameters, a hook is called for every selected entry); topk.hip instantiates it.
#pragma once
#include "kernels.hpp"

namespace fastocr {

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
// With stop_shift > 0 only the bits at and above it are resolved: the result is the k-th largest
// key with its low bits cleared, a lower bound of it (and *ties_needed is meaningless).
// Two histograms alternate between the passes (the idle one is cleared while the other is being
// filled), which leaves two workgroup barriers per 8-bit pass.
template <int THREADS>
__device__ uint32_t radix_select(const uint32_t *keys, int n, int k, uint32_t (*hist)[256], int *s_pick,
                                 int *ties_needed, int stop_shift = 0)
{
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t prefix = 0u, mask = 0u;
    int kk = k, cur = 0;
    if (tid < 256) hist[0][tid] = 0u;
    __syncthreads();
    for (int shift = 24; shift >= stop_shift; shift -= 8) {
        uint32_t *h = hist[cur];
        if (tid < 256) hist[cur ^ 1][tid] = 0u;
        for (int i0 = 0; i0 < n; i0 += THREADS) {
            const int i = i0 + tid;
            const bool in = i < n;
            const uint32_t key = in ? keys[i] : 0u;
            const bool live = in && ((key & mask) == prefix);
            const uint32_t dgt = (key >> shift) & 255u;
            // a whole wave on one digit (the usual case for the exponent byte) adds once
            const uint64_t live_mask = __ballot(live);
            if (live_mask) {
                const int first = __builtin_amdgcn_readfirstlane(__ffsll((long long)live_mask) - 1);
                const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)dgt, first);
                const uint64_t same = __ballot(live && dgt == d0);
                if (same == live_mask) {
                    if (lane == first) atomicAdd(&h[d0], (uint32_t)__popcll(live_mask));
                } else if (live) {
                    atomicAdd(&h[dgt], 1u);
                }
            }
        }
        __syncthreads();
        if (tid < 64) {
            // lane owns digits 255-4*lane .. 252-4*lane (descending)
            uint32_t c[4], tot = 0u;
#pragma unroll
            for (int x = 0; x < 4; ++x) { c[x] = h[255 - (4 * lane + x)]; tot += c[x]; }
            const uint32_t incl = (uint32_t)wave_scan_incl((int)tot);
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
        // the next pass writes s_pick only after its own first barrier, which every thread
        // reaches after this read
        prefix |= ((uint32_t)s_pick[0]) << shift;
        mask |= 255u << shift;
        kk = s_pick[1];
        cur ^= 1;
    }
    __syncthreads();          // callers may reuse keys, hist and s_pick right away
    *ties_needed = kk;
    return prefix;
}

// Image spans of up to kTopkRegKeys tokens: one workgroup per sequence, thread t keeps the keys of
// tokens 16t .. 16t+15 in registers.  The candidate list (keys at or above the bound theta0, see
// above) and the result are both written in index order through block-wide prefix sums, so no
// atomics or index arrays are needed, and the scores are read exactly once.
constexpr int kRegCandCap = 8192;          // candidates this kernel selects among (keep ratios up to 1/3 at 16384 tokens)

// exclusive prefix sums of (a, c) over the workgroup's THREADS threads; totals through *ta, *tc.  All threads call.
// w_ac: 2 x THREADS/64 wave totals, 16-byte aligned.
typedef int i32x4 __attribute__((ext_vector_type(4)));
template <int THREADS>
__device__ __forceinline__ void block_scan2(int a, int c, int *w_ac, int &a_excl, int &c_excl, int *ta, int *tc)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ai = wave_scan_incl(a), ci = wave_scan_incl(c);
    if (lane == 63) { w_ac[wave] = ai; w_ac[(THREADS / 64) + wave] = ci; }
    __syncthreads();
    int ab = 0, cb = 0, at = 0, ct = 0;
#pragma unroll
    for (int v = 0; v < (THREADS / 64) / 4; ++v) {
        const i32x4 x = reinterpret_cast<const i32x4 *>(w_ac)[v], y = reinterpret_cast<const i32x4 *>(w_ac)[(THREADS / 64) / 4 + v];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (4 * v + e < wave) { ab += x[e]; cb += y[e]; }
            at += x[e];
            ct += y[e];
        }
    }
    a_excl = ab + ai - a;
    c_excl = cb + ci - c;
    *ta = at;
    *tc = ct;
    __syncthreads();
}

// Shared memory of topk_reg_body, provided by the calling kernel.
struct TopkRegShared {
    uint32_t (*hist)[256];      // [2][256]
    uint32_t *cand;             // [kRegCandCap]
    uint32_t *all_keys;         // [max_vis_len]: all keys, only touched when the candidate list fails
    int *pick;                  // [2]
    uint32_t *theta_prev;       // [1]
    int *bad;                   // [1]
    int *w_ac;                  // [2 * THREADS / 64], 16-byte aligned
};

// One workgroup of THREADS threads selects sequence b's set; thread t keeps the keys of tokens
// PER t .. PER t + PER - 1 in registers (THREADS * PER >= max_vis_len).  publish(position, index) is
// called by the thread that writes sel_idx[position] = index, for every entry of the result.
// COHERENT: the scores were written earlier in the SAME launch by other workgroups (agent-scope
// stores, completed before this workgroup was told so): they are read with agent-scope loads, which
// never hit a line this compute unit's caches may still hold from before.
template <bool COHERENT>
__device__ __forceinline__ float score_at(const float *p)
{
    if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

template <int THREADS, int PER, bool COHERENT = false, typename Publish>
__device__ __forceinline__ void topk_reg_body(
    const float *__restrict__ scores, const BatchDev &bv, int b, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax, const TopkRegShared &sh,
    Publish publish)
{
    const int tid = threadIdx.x, lane = tid & 63;
    int32_t *out = sel_idx + (int64_t)b * kmax;
    const float *srow = scores + (int64_t)b * bv.max_vis_len;

    // The thread's 16 scores and its first two entries of the previous set are requested before
    // the sequence's geometry is known (the rows are max_vis_len and kmax entries long whatever the
    // sequence's own counts are): one memory round trip instead of two before the keys exist.
    const int base = tid * PER;
    const bool whole = base + PER <= bv.max_vis_len && (reinterpret_cast<uintptr_t>(srow + base) & 15u) == 0;
    f32x4 raw[PER / 4];
#pragma unroll
    for (int v = 0; v < PER / 4; ++v) raw[v] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (whole) {
#pragma unroll
        for (int v = 0; v < PER / 4; ++v) {
            if (COHERENT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) raw[v][e] = score_at<true>(srow + base + 4 * v + e);
            } else {
                raw[v] = *reinterpret_cast<const f32x4 *>(srow + base + 4 * v);
            }
        }
    }
    const int32_t *prev = prev_idx ? prev_idx + (int64_t)b * kmax : nullptr;
    int prev0 = 0, prev1 = 0;
    if (prev && tid < kmax) prev0 = prev[tid];
    if (prev && tid + 1 < kmax) prev1 = prev[tid + 1];

    const SeqGeom geo = seq_geom(bv, b);
    const int N = geo.N;
    const int k = (int)min((int64_t)keep_count_dev(N, tau), kmax);
    const int pcnt = prev_cnt ? prev_cnt[b] : -1;

    if (k <= 0 || k >= N) {
        if (k >= N && k > 0)
            for (int i = tid; i < N; i += THREADS) { out[i] = i; publish(i, i); }
        if (tid == 0) sel_cnt[b] = k <= 0 ? 0 : N;
        return;
    }
    if (tid == 0) { (*sh.theta_prev) = 0xffffffffu; (*sh.bad) = 0; }

    // ---- the thread's 16 keys; tokens past N get key 0 and are never counted ----------------------
    const int nvalid = min(max(N - base, 0), PER);
    // which of the thread's keys are real, as a bit mask in a vector register (PER lane masks kept in
    // scalar registers, as `j < nvalid` would have it, take most of the scalar file)
    const uint32_t vmask = nvalid >= 32 ? 0xffffffffu : ((1u << nvalid) - 1u);
    auto real = [&](int j) { return ((vmask >> j) & 1u) != 0u; };
    uint32_t key[PER];
    if (whole) {
#pragma unroll
        for (int v = 0; v < PER / 4; ++v)
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * v + e] = real(4 * v + e) ? order_key(raw[v][e]) : 0u;
    } else {
#pragma unroll
        for (int j = 0; j < PER; ++j) key[j] = j < nvalid ? order_key(score_at<COHERENT>(srow + base + j)) : 0u;
    }
    // ---- bound from the previous set: k distinct valid tokens (strictly ascending) or ignored ----
    const bool have_prev = prev_idx && pcnt == k;
    uint32_t lo = 0xffffffffu;
    int bad = 0;
    if (have_prev) {
        for (int r = tid; r < k; r += THREADS) {
            const int i = r == tid ? prev0 : prev[r];
            const int nx = (r + 1 < k) ? (r == tid ? prev1 : prev[r + 1]) : 0x7fffffff;
            if (i < 0 || i >= N || i >= nx) bad = 1;
            else lo = min(lo, order_key(score_at<COHERENT>(srow + i)));
        }
    }
    // ---- bound from a sample: the first key of every thread (every PER-th token) ---------------------
    // (run before the previous set's bound is reduced: the gather of the previous set's current scores
    // above is a dependent memory round trip, and the sample select needs nothing from memory)
    const int ns = (N + PER - 1) / PER;
    if (tid < ns) sh.cand[tid] = key[0];
    __syncthreads();
    uint32_t theta0 = 0u;
    {
        // about 1.5 k of the N tokens should reach the bound: rank 1.5 k ns / N in the sample, plus slack
        const int r = (int)(((int64_t)3 * k * ns) / ((int64_t)2 * N)) + 24;
        if (r < ns) {
            int unused;
            // the upper 16 bits are enough for a bound (fp32: sign, exponent, 7 mantissa bits)
            const uint32_t ths = radix_select<THREADS>(sh.cand, ns, r, sh.hist, sh.pick, &unused, 16);
            theta0 = max(theta0, ths);
        }
    }
    if (have_prev) {
        if (bad) (*sh.bad) = 1;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, o));
        if (lane == 0) atomicMin(&(*sh.theta_prev), lo);
        __syncthreads();
        if (!(*sh.bad)) theta0 = max(theta0, *sh.theta_prev);
    }
    __syncthreads();
    // ---- candidates, compacted in index order --------------------------------------------------------
    int mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine += (real(j) && key[j] >= theta0) ? 1 : 0;
    int pos, unused_excl, nc, unused_tot;
    block_scan2<THREADS>(mine, 0, sh.w_ac, pos, unused_excl, &nc, &unused_tot);
    const bool from_cand = nc >= k && nc <= kRegCandCap;
    uint32_t theta;
    int ties;
    if (from_cand) {
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (real(j) && key[j] >= theta0) sh.cand[pos++] = key[j];
        __syncthreads();
        theta = radix_select<THREADS>(sh.cand, nc, k, sh.hist, sh.pick, &ties);
    } else {
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (real(j)) sh.all_keys[base + j] = key[j];
        __syncthreads();
        theta = radix_select<THREADS>(sh.all_keys, N, k, sh.hist, sh.pick, &ties);
    }
    // ---- the result in ascending index order; ties go to the lowest indices ------------------------
    // bit j of the masks: key j of this thread lies above / on the threshold
    uint32_t m_gt = 0u, m_eq = 0u;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        m_gt |= (real(j) && key[j] > theta) ? (1u << j) : 0u;
        m_eq |= (real(j) && key[j] == theta) ? (1u << j) : 0u;
    }
    int gt_excl, eq_excl, gt_tot, eq_tot;
    block_scan2<THREADS>(__popc(m_gt), __popc(m_eq), sh.w_ac, gt_excl, eq_excl, &gt_tot, &eq_tot);
    // of this thread's keys on the threshold, the first (ties - eq_excl) are still wanted
    uint32_t take = m_gt;
    {
        int want = min(max(ties - eq_excl, 0), __popc(m_eq));
        uint32_t rest = m_eq;
        while (want > 0) { const uint32_t low = rest & (0u - rest); take |= low; rest ^= low; --want; }
    }
    int opos = gt_excl + min(ties, eq_excl);
    while (take) {
        const int sel = base + __ffs((int)take) - 1;
        out[opos] = sel;
        publish(opos, sel);
        ++opos;
        take &= take - 1u;
    }
    if (tid == 0) sel_cnt[b] = k;
}


}  // namespace fastocr
