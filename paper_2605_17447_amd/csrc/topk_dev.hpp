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

// ---- the register-resident select ----------------------------------------------------------------------
// Image spans of up to THREADS * PER tokens: one workgroup per sequence, thread t keeps the keys of
// tokens PER t .. PER t + PER - 1 in registers, so the scores are read exactly once.  The threshold
// (the k-th largest key) is found by histogram passes straight from the registers (window_select
// below), the result is written in index order through a block-wide prefix sum: no candidate list,
// no atomics on memory, no index arrays.

// max / min over the 64 lanes of a wave with data-parallel-primitive moves (see wave_scan_incl);
// the result is the same in every lane
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
#define FASTOCR_DPP_STEP(CTRL, ROWS) x = max(x, (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, ROWS, 0xf, false))
    FASTOCR_DPP_STEP(0x111, 0xf); FASTOCR_DPP_STEP(0x112, 0xf); FASTOCR_DPP_STEP(0x114, 0xf); FASTOCR_DPP_STEP(0x118, 0xf);
    FASTOCR_DPP_STEP(0x142, 0xa); FASTOCR_DPP_STEP(0x143, 0xc);
#undef FASTOCR_DPP_STEP
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) { return ~wave_max_u32(~x); }

// exclusive prefix sums of (a, c) over the workgroup's THREADS threads; totals through *ta, *tc.  All threads call.
// w_ac: at least 2 x THREADS/64 wave totals, 16-byte aligned.
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
constexpr int kWinBins = 512;               // bins of a histogram pass
constexpr int kWinRank = 64;                // a bin of at most this many keys is ranked key by key
constexpr int kWinListWords = 3 * kWinRank; // the bin's keys, then how many keys lie above / equal each of them
struct TopkRegShared {
    uint32_t *hist;             // [kWinBins]
    uint32_t *list;             // [kWinListWords], 16-byte aligned
    int *pick;                  // [4]: bin, rank within it, keys copied so far
    int *w_ac;                  // [4 * THREADS / 64], 16-byte aligned
};

// The k-th largest of the workgroup's keys, all of them in the threads' registers, given a window lo <= key <= key_max that holds at least the k
// largest.  A histogram pass counts the window's keys in 512 bins of 2^shift key values; the first
// window's bins are as fine as the spread of the keys allows (flat scores: a small fraction of an
// octave of an fp32 score per bin; heavy tails: most keys still sit in the low bins, next to the
// k-th).  The bin that holds the k-th largest key becomes the next window, 512 times finer, until it
// holds at most kWinRank keys; those are copied to LDS and ranked: every pair is compared once, spread
// over all threads, and the key with above < rank <= above + equal is the threshold.  A window of
// single key values (shift 0) names the threshold by its bin.  One pass and the ranking is the usual
// case.  hist and the list's counters must be zero and pick[2] = 0 on entry (the caller clears them
// before a barrier of its own).  *ties = how many keys equal to the threshold belong to the k largest.
template <int THREADS, int PER>
__device__ __forceinline__ uint32_t window_select(const uint32_t (&key)[PER], uint32_t lo, uint32_t key_max,
                                                  int k, const TopkRegShared &sh, int *ties)
{
    static_assert(THREADS >= kWinBins && THREADS % 256 == 0, "one thread clears one bin; whole vectors of wave totals");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t *h = sh.hist;
    uint32_t span = key_max - lo;                    // the window: lo <= key <= lo + span
    int shift = max(0, 23 - (int)__builtin_clz(span | 1u));                     // span >> shift < 512
    int rank = k, nb = 0;
    if (span == 0u) {                                // every key of the window is the same
        *ties = k;
        return lo;
    }
    // key - lo <= span in unsigned arithmetic is the whole test (a key below lo wraps around to more
    // than any span).  Padding keys (0, past the sequence's end) are not masked out: they can only
    // fall into the lowest bin of a window that starts at key 0, below every real key or equal to the
    // smallest ones, and ranks are counted from the top -- neither the threshold nor the tie count
    // sees them; the caller drops them from the output by its own mask.
    while (true) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t d = key[j] - lo;
            if (d <= span) atomicAdd(&h[d >> shift], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            // lane owns bins 511-8*lane .. 504-8*lane (descending)
            uint32_t c[8], tot = 0u;
#pragma unroll
            for (int x = 0; x < 8; ++x) { c[x] = h[kWinBins - 1 - (8 * lane + x)]; tot += c[x]; }
            const uint32_t incl = (uint32_t)wave_scan_incl((int)tot);
            const uint32_t above = incl - tot;
            if (above < (uint32_t)rank && incl >= (uint32_t)rank) {
                uint32_t run = above;
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    if (run < (uint32_t)rank && run + c[x] >= (uint32_t)rank) {
                        sh.pick[0] = kWinBins - 1 - (8 * lane + x);
                        sh.pick[1] = rank - (int)run;
                    }
                    run += c[x];
                }
            }
        }
        __syncthreads();
        const int bin = sh.pick[0];
        rank = sh.pick[1];
        nb = (int)h[bin];
        lo += (uint32_t)bin << shift;
        if (shift == 0) {                            // the window's bins were single key values
            *ties = rank;
            return lo;
        }
        span = (1u << shift) - 1u;                   // the bin is the next window
        if (nb <= kWinRank) break;
        shift = max(0, shift - 9);                   // ... cut into 512 bins again
        __syncthreads();                             // everybody has read pick and the histogram
        if (tid < kWinBins) h[tid] = 0u;
        __syncthreads();
    }
    // ---- the bin's keys into LDS --------------------------------------------------------------------------
    // At most kWinRank of the workgroup's keys are in the bin, so nearly all of a wave's PER lane masks
    // (one per key position, in scalar registers) are empty and are skipped by a scalar branch; a wave
    // that holds any reserves its places with one counter update.
    if constexpr (PER <= 16) {
        uint64_t hit[PER];
        int mine = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            hit[j] = __builtin_amdgcn_ballot_w64(key[j] - lo <= span);
            mine += __popcll(hit[j]);
        }
        if (mine) {
            int pos = 0;
            if (lane == 0) pos = atomicAdd(&sh.pick[2], mine);
            pos = __builtin_amdgcn_readfirstlane(pos);
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                if (hit[j]) {
                    const int before = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(hit[j] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hit[j], 0u));
                    if (key[j] - lo <= span && pos + before < kWinRank) sh.list[pos + before] = key[j];
                    pos += __popcll(hit[j]);
                }
            }
        }
    } else {
        // (many keys per thread: that many lane masks would crowd the scalar registers of the kernel
        // around this code; the places are dealt lane by lane instead)
        uint32_t hit = 0u;                           // bit j: key j lies in the bin (shifted in from the top key down)
#pragma unroll
        for (int j = PER - 1; j >= 0; --j) hit = hit + hit + ((key[j] - lo <= span) ? 1u : 0u);
        const int mine = __popc(hit);
        const int upto = wave_scan_incl(mine);
        const int total = __builtin_amdgcn_readlane(upto, 63);
        if (total) {
            int pos = 0;
            if (lane == 0) pos = atomicAdd(&sh.pick[2], total);
            pos = __builtin_amdgcn_readfirstlane(pos) + upto - mine;
            if (hit) {
#pragma unroll
                for (int j = 0; j < PER; ++j)
                    if (((hit >> j) & 1u) && pos < kWinRank) sh.list[pos++] = key[j];
            }
        }
    }
    __syncthreads();
    // ---- every pair once: thread (wave w, lane i) compares key i with keys w*E .. w*E+E-1 --------------
    {
        constexpr int E = kWinRank / (THREADS / 64);
        static_assert(E % 4 == 0, "whole 16-byte reads");
        if (lane < nb && wave * E < nb) {
            const uint32_t e = sh.list[lane];
            int gt = 0, eq = 0;
#pragma unroll
            for (int v = 0; v < E / 4; ++v) {
                const u32x4 x = reinterpret_cast<const u32x4 *>(sh.list)[wave * (E / 4) + v];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const bool there = wave * E + 4 * v + c < nb;
                    gt += (there && x[c] > e) ? 1 : 0;
                    eq += (there && x[c] == e) ? 1 : 0;
                }
            }
            if (gt) atomicAdd(&sh.list[kWinRank + lane], (uint32_t)gt);
            if (eq) atomicAdd(&sh.list[2 * kWinRank + lane], (uint32_t)eq);
        }
    }
    __syncthreads();
    if (tid < nb) {
        const int gt = (int)sh.list[kWinRank + tid], eq = (int)sh.list[2 * kWinRank + tid];
        if (gt < rank && rank <= gt + eq) { sh.pick[0] = (int)sh.list[tid]; sh.pick[1] = rank - gt; }     // equal keys write the same
    }
    __syncthreads();
    *ties = sh.pick[1];
    return (uint32_t)sh.pick[0];
}

// One workgroup of THREADS threads selects sequence b's set.  publish(position, index) is called by
// the thread that writes sel_idx[position] = index, for every entry of the result.
// The first window runs from a lower bound of the threshold to the largest key.  The bound is the
// smallest key of all, or -- the warm start -- the smallest CURRENT key among the previous set's k
// tokens when that set is k distinct valid tokens: k keys reach it, so the threshold cannot lie
// below, and when the fixation moved little it cuts the window to the top few per cent of the keys.
// The result never depends on the bound.
// COHERENT: the scores were written earlier in the SAME launch by other workgroups (agent-scope
// stores, completed before this workgroup was told so): they are read with agent-scope loads, which
// never hit a line this compute unit's caches may still hold from before.
template <bool COHERENT>
__device__ __forceinline__ float score_at(const float *p)
{
    if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

template <int THREADS, int PER, bool COHERENT, bool VEC, typename Publish>
__device__ __forceinline__ void topk_reg_body(
    const float *__restrict__ scores, const BatchDev &bv, int b, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax, const TopkRegShared &sh,
    Publish publish)
{
    static_assert(PER <= 32 && PER % 4 == 0, "a thread's keys are tracked in 32-bit masks and loaded 16 bytes at a time");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int W = THREADS / 64;
    int32_t *out = sel_idx + (int64_t)b * kmax;
    const float *srow = scores + (int64_t)b * bv.max_vis_len;

    // the select's LDS starts out clear (the barrier further down stands between this and its first use)
    if (tid < kWinBins) sh.hist[tid] = 0u;
    if (tid < 2 * kWinRank) sh.list[kWinRank + tid] = 0u;
    if (tid == 0) sh.pick[2] = 0;
    if (bv.max_vis_len <= 0 || kmax <= 0) {                       // no row to read from, nothing to keep
        if (tid == 0) sel_cnt[b] = 0;
        return;
    }

    // The thread's first two entries of the previous set and its scores are requested before the
    // sequence's geometry is known (the rows are kmax and max_vis_len entries long whatever the
    // sequence's own counts are): one memory round trip instead of two before the keys exist.  The
    // previous set's entries go first: loads come back in the order they were sent, so the score
    // that the first entry points at can be requested while the thread's own scores are still on
    // their way.  Everything up to the keys is straight-line code with clamped addresses instead of
    // branches: across a branch the compiler waits for every outstanding load.
    const int32_t *pv = prev_idx ? prev_idx + (int64_t)b * kmax : reinterpret_cast<const int32_t *>(srow);
    const int pv_last = prev_idx ? (int)min(kmax, (int64_t)0x7fffffff) - 1 : 0;
    const int prev0 = pv[min(tid, pv_last)], prev1 = pv[min(tid + 1, pv_last)];
    const int base = tid * PER;
    // VEC (rows start 16-byte aligned and hold whole 16-byte pieces; the host knows): a piece lies inside
    // the row or past it -- then it is read from the row's start and masked out, like single scores
    // past the row's end otherwise
    float raw[PER];
    if constexpr (VEC && !COHERENT) {
#pragma unroll
        for (int v = 0; v < PER / 4; ++v) {
            const int at = base + 4 * v + 4 <= bv.max_vis_len ? base + 4 * v : 0;
            const f32x4 x = *reinterpret_cast<const f32x4 *>(srow + at);
#pragma unroll
            for (int e = 0; e < 4; ++e) raw[4 * v + e] = x[e];
        }
    } else {
#pragma unroll
        for (int j = 0; j < PER; ++j) raw[j] = score_at<COHERENT>(srow + (base + j < bv.max_vis_len ? base + j : 0));
    }

    const int e_seq = bv.seq_len[b], e_start = bv.vis_start[b], e_vis = bv.vis_len[b];
    const int e_prev = (prev_cnt ? prev_cnt : bv.vis_len)[b];
    const SeqGeom geo = seq_geom_of(bv, e_seq, e_start, e_vis);
    const int N = geo.N;
    const int k = (int)min((int64_t)keep_count_dev(N, tau), kmax);
    const int pcnt = prev_cnt ? e_prev : -1;

    // ---- bound from the previous set: k distinct valid tokens (strictly ascending) or none ----------
    // entry r = tid: its current score is requested here (from a clamped address when there is no
    // such entry), used further down
    const bool have_prev = prev_idx && pcnt == k && k > 0 && k < N;
    uint32_t lo_prev = have_prev ? 0xffffffffu : 0u;
    const bool first_mine = have_prev && tid < k;
    const bool first_ok = prev0 >= 0 && prev0 < N && prev0 < ((tid + 1 < k) ? prev1 : 0x7fffffff);
    const float first_score = score_at<COHERENT>(srow + ((first_mine && first_ok) ? prev0 : 0));
    if (first_mine && !first_ok) lo_prev = 0u;                    // not a set of k tokens: no bound

    if (k <= 0 || k >= N) {
        if (k >= N && k > 0)
            for (int i = tid; i < N; i += THREADS) { out[i] = i; publish(i, i); }
        if (tid == 0) sel_cnt[b] = k <= 0 ? 0 : N;
        return;
    }

    // ---- the thread's keys; tokens past N get key 0 and are never counted ---------------------------
    const int nvalid = min(max(N - base, 0), PER);
    // which of the thread's keys are real, as a bit mask in a vector register (PER lane masks kept in
    // scalar registers, as `j < nvalid` would have it, take most of the scalar file)
    const uint32_t vmask = nvalid >= 32 ? 0xffffffffu : ((1u << nvalid) - 1u);
    auto real = [&](int j) { return ((vmask >> j) & 1u) != 0u; };
    uint32_t key[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) key[j] = real(j) ? order_key(raw[j]) : 0u;
    // the previous set's entries beyond the first THREADS (keep ratios above 1/PER)
    if (have_prev) {
        for (int r = tid + THREADS; r < k; r += THREADS) {
            const int i = pv[r];
            const int nx = (r + 1 < k) ? pv[r + 1] : 0x7fffffff;
            if (i < 0 || i >= N || i >= nx) lo_prev = 0u;
            else lo_prev = min(lo_prev, order_key(score_at<COHERENT>(srow + i)));
        }
        if (first_mine && first_ok) lo_prev = min(lo_prev, order_key(first_score));
    }
    // ---- the largest and the smallest key and the previous set's bound: one exchange through LDS --------
    uint32_t kmx = 0u, kmn = 0xffffffffu;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        kmx = max(kmx, key[j]);                                   // (padding keys are 0)
        kmn = min(kmn, key[j]);
    }
    if (nvalid < PER) {                                           // the thread at the sequence's end and those past it
        kmn = 0xffffffffu;
#pragma unroll
        for (int j = 0; j < PER; ++j) kmn = min(kmn, real(j) ? key[j] : 0xffffffffu);
    }
    // A third bound costs nothing more: every thread that holds a real key holds one at or above the
    // smallest of the threads' own maxima, so when k does not exceed the number of such threads, k keys
    // reach that value (scores without structure: about a third of the keys, which spares the
    // histogram pass the other two thirds of its LDS atomics).
    uint32_t lo_own = (nvalid > 0 && k <= (N + PER - 1) / PER) ? kmx : (nvalid > 0 ? 0u : 0xffffffffu);
    kmx = wave_max_u32(kmx);
    kmn = wave_min_u32(kmn);
    lo_prev = wave_min_u32(lo_prev);
    lo_own = wave_min_u32(lo_own);
    if (lane == 0) {
        sh.w_ac[wave] = (int)kmx;
        sh.w_ac[W + wave] = (int)~kmn;
        sh.w_ac[2 * W + wave] = (int)~lo_prev;
        sh.w_ac[3 * W + wave] = (int)~lo_own;
    }
    __syncthreads();
    uint32_t nmn = 0u, nlo = 0u, now = 0u;                        // complements: everything is a maximum
#pragma unroll
    for (int v = 0; v < W / 4; ++v) {
        const i32x4 *wv = reinterpret_cast<const i32x4 *>(sh.w_ac);
        const i32x4 x = wv[v], y = wv[W / 4 + v], z = wv[2 * (W / 4) + v], u = wv[3 * (W / 4) + v];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            kmx = max(kmx, (uint32_t)x[e]);
            nmn = max(nmn, (uint32_t)y[e]);
            nlo = max(nlo, (uint32_t)z[e]);
            now = max(now, (uint32_t)u[e]);
        }
    }
    // (a sequence whose threads past its end vote 0xffffffff alone cannot happen: N >= 1 here)
    const uint32_t lo = max(max(~nmn, ~nlo), ~now);               // (w_ac is next written two barriers further on)

    // ---- the threshold ---------------------------------------------------------------------------------
    int ties;
    const uint32_t theta = window_select<THREADS, PER>(key, lo, kmx, k, sh, &ties);

    // ---- the result in ascending index order; ties go to the lowest indices ------------------------
    // bit j of the masks: key j of this thread lies above / on the threshold
    // (shifted in from the top key down: a compare and an add-with-carry per key and mask; a padding key,
    // 0, is never above a threshold and is taken off the ties by the validity mask)
    uint32_t m_gt = 0u, m_eq = 0u;
#pragma unroll
    for (int j = PER - 1; j >= 0; --j) {
        m_gt = m_gt + m_gt + ((key[j] > theta) ? 1u : 0u);
        m_eq = m_eq + m_eq + ((key[j] == theta) ? 1u : 0u);
    }
    m_eq &= vmask;
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
