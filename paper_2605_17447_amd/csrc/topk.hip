// TopK_{ceil(tau N)} over one sequence's image scores (Sec. 3.1.2), exact and deterministic,
// warm-started from the previous step's focal token set (Cross-Step Fixation Reuse, Sec. 3.2).
//
// The scores become order-preserving 32-bit keys.  The k-th largest key (the threshold) is found
// by an MSB-first 8-bit radix select in LDS; everything above it, plus the lowest-index keys equal
// to it until k, is written in ascending index order.  To keep the select short and the whole
// chip busy, a sequence is spread over several 1024-thread workgroups that first reduce the N
// keys to a short candidate list bounded below by (a) the previous step's set -- the warm start:
// its k tokens' smallest current key can only be at or below the new threshold -- and (b) a
// sample of the scores; see topk_kernel.  The result never depends on either bound.
#include <atomic>

#include "kernels.hpp"

namespace fastocr {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kCandCap = 4096;
constexpr int kLdsKeyCap = 24576;
constexpr int kBitmapWords = 1024;        // candidates path: image spans of up to 32768 tokens

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
__device__ uint32_t radix_select(const uint32_t *keys, int n, int k, uint32_t *hist, int *s_pick,
                                 int *ties_needed, int stop_shift = 0)
{
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t prefix = 0u, mask = 0u;
    int kk = k;
    for (int shift = 24; shift >= stop_shift; shift -= 8) {
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

// Per-sequence counters of the multi-workgroup path: candidates appended so far, workgroups
// arrived.  They live in static device memory (zero when the module is loaded) rather than in the
// caller's workspace, which would have to be cleared by an extra launch before every call; the
// workgroup that arrives last is the only one still running for its sequence and clears them, so
// a slot is clean again when its call ends.  Calls take slots round-robin: up to kTopkSlots calls
// may overlap on one GPU.  Batches beyond kTopkMaxBatch use one workgroup per sequence.
struct TopkCounters { uint32_t ncand, arrived; };
constexpr int kTopkSlots = 32;
constexpr int kTopkMaxBatch = 1024;
__device__ TopkCounters g_topk_ctr[kTopkSlots][kTopkMaxBatch];

// Grid (parts, batch).  Every workgroup of a sequence derives the same lower bound theta0 of the
// threshold for itself, filters its own slice of the scores against it and appends the survivors
// to the sequence's candidate list; the workgroup that arrives last selects among the candidates.
//   theta0 = max(bound from the previous set, bound from a sample)
//   previous set (warm start): the smallest current key among its k tokens -- a certain bound
//     (k tokens reach it), tight when the fixation moved little;
//   sample: the r-th largest of 1024 evenly spaced scores, r chosen so that about 1.5 k tokens
//     reach it -- a likely bound only, so the last workgroup checks that at least k candidates came
//     in.  If they did, the k largest overall are among them and the result is exact.
// If fewer than k or more than kCandCap candidates came in, the last workgroup selects over all N
// keys on its own: the result is the same in every case.
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(
    const float *__restrict__ scores, BatchDev bv, double tau, const int32_t *prev_idx,
    const int32_t *prev_cnt, int32_t *sel_idx, int32_t *sel_cnt, int64_t kmax,
    uint32_t *__restrict__ gkeys, int lds_keys, int sync_slot, unsigned long long *cand_list)
{
    TopkCounters *ctr = g_topk_ctr[sync_slot];
    extern __shared__ uint32_t dyn_keys[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t cand[kCandCap];
    __shared__ uint32_t cand_i[kCandCap];
    __shared__ uint32_t bitmap[kBitmapWords], bitmap_eq[kBitmapWords];
    __shared__ int s_pick[2];
    __shared__ uint32_t s_theta_prev;
    __shared__ int s_bad, s_ncand, s_base, s_last;
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

    if (tid == 0) { s_theta_prev = 0xffffffffu; s_bad = 0; s_ncand = 0; s_last = 0; }
    __syncthreads();

    uint32_t theta;
    int ties;
    const bool filtered = nparts > 1 && N <= kBitmapWords * 32;
    if (filtered) {
        // the three independent gathers (sample, own slice, previous set) are issued together
        const int ns = min(N, kTopkThreads);
        const float sample_v = tid < ns ? srow[(int)(((int64_t)tid * N) / ns)] : 0.f;
        const int own_i = part * kTopkThreads + tid;
        const float own_v = own_i < N ? srow[own_i] : 0.f;
        // ---- bound from the previous set: k distinct valid tokens (strictly ascending) or ignored ----
        uint32_t theta0 = 0u;
        if (prev_idx && pcnt == k) {
            const int32_t *prev = prev_idx + (int64_t)b * kmax;
            uint32_t lo = 0xffffffffu;
            int bad = 0;
            for (int r = tid; r < k; r += kTopkThreads) {
                const int i = prev[r];
                const int nx = (r + 1 < k) ? prev[r + 1] : 0x7fffffff;
                if (i < 0 || i >= N || i >= nx) bad = 1;
                else lo = min(lo, order_key(srow[i]));
            }
            if (bad) s_bad = 1;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) lo = min(lo, (uint32_t)__shfl_xor((int)lo, o));
            if (lane == 0) atomicMin(&s_theta_prev, lo);
            __syncthreads();
            if (!s_bad) theta0 = s_theta_prev;
        }
        // ---- bound from a sample of kTopkThreads evenly spaced scores -----------------------------
        {
            if (tid < ns) cand[tid] = order_key(sample_v);
            __syncthreads();
            // about 1.5 k of the N tokens should reach the bound: rank 1.5 k ns / N in the sample, plus slack
            const int r = (int)(((int64_t)3 * k * ns) / ((int64_t)2 * N)) + 24;
            if (r < ns) {
                int unused;
                // the upper 16 bits are enough for a bound (fp32: sign, exponent, 7 mantissa bits)
                const uint32_t ths = radix_select(cand, ns, r, hist, s_pick, &unused, 16);
                theta0 = max(theta0, ths);
            }
            __syncthreads();
        }
        // ---- filter the own slice, append the survivors to the sequence's list --------------------
        for (int ii = own_i; ii < N; ii += nparts * kTopkThreads) {
            const uint32_t key = order_key(ii == own_i ? own_v : srow[ii]);
            const bool c = key >= theta0;
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
        const int mine = s_ncand;
        if (tid == 0)
            s_base = mine > 0 ? (int)__hip_atomic_fetch_add(&ctr[b].ncand, (uint32_t)mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
        __syncthreads();
        // The list crosses compute units through agent-scope atomic stores (written through to
        // memory); each thread waits for its stores to be acknowledged before the workgroup is
        // counted in.
        unsigned long long *list = cand_list + (int64_t)b * kCandCap;
        for (int c = tid; c < min(mine, kCandCap); c += kTopkThreads) {
            const int pos = s_base + c;
            if (pos < kCandCap)
                __hip_atomic_store(&list[pos], ((unsigned long long)cand[c] << 32) | cand_i[c], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const uint32_t old = __hip_atomic_fetch_add(&ctr[b].arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == (uint32_t)nparts - 1u;
        }
        __syncthreads();
        if (!s_last) return;

        // ---- the last workgroup of the sequence selects among the candidates ----------------------
        const int nc = (int)__hip_atomic_load(&ctr[b].ncand, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (tid == 0) {                                    // clean for the next call on this slot
            __hip_atomic_store(&ctr[b].ncand, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&ctr[b].arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (nc >= k && nc <= kCandCap) {
            for (int c = tid; c < nc; c += kTopkThreads) {
                const unsigned long long e = __hip_atomic_load(&list[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                cand[c] = (uint32_t)(e >> 32);
                cand_i[c] = (uint32_t)e;
            }
            for (int w = tid; w < kBitmapWords; w += kTopkThreads) { bitmap[w] = 0u; bitmap_eq[w] = 0u; }
            __syncthreads();
            theta = radix_select(cand, nc, k, hist, s_pick, &ties);
            // mark the keys above the threshold, and separately those equal to it
            for (int c = tid; c < nc; c += kTopkThreads) {
                const uint32_t key = cand[c], i = cand_i[c];
                if (key > theta) atomicOr(&bitmap[i >> 5], 1u << (i & 31));
                else if (key == theta) atomicOr(&bitmap_eq[i >> 5], 1u << (i & 31));
            }
            __syncthreads();
            // ordered emission: word w of the bitmaps belongs to thread w; ties go to the lowest indices
            const int nwords = (N + 31) / 32;
            int eq_before = 0, out_before = 0;
            for (int w0 = 0; w0 < nwords; w0 += kTopkThreads) {
                const int w = w0 + tid;
                const uint32_t g = w < nwords ? bitmap[w] : 0u, e = w < nwords ? bitmap_eq[w] : 0u;
                const int ne = __popc(e);
                int ne_incl = ne;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(ne_incl, o); if (lane >= o) ne_incl += t; }
                if (lane == 63) w_eq[wave] = ne_incl;
                __syncthreads();
                int eq_off = eq_before;
                for (int x = 0; x < wave; ++x) eq_off += w_eq[x];
                int eq_tot = 0;
                for (int x = 0; x < kTopkWaves; ++x) eq_tot += w_eq[x];
                const int eq_excl = eq_off + ne_incl - ne;
                // ties of this word that are still wanted: its first (ties - eq_excl) set bits
                uint32_t take_eq = 0u;
                int want = min(max(ties - eq_excl, 0), ne);
                uint32_t rest = e;
                while (want > 0) { const uint32_t low = rest & (0u - rest); take_eq |= low; rest ^= low; --want; }
                const uint32_t sel = g | take_eq;
                const int nsel = __popc(sel);
                int ns_incl = nsel;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) { const int t = __shfl_up(ns_incl, o); if (lane >= o) ns_incl += t; }
                if (lane == 63) w_gt[wave] = ns_incl;
                __syncthreads();
                int pos = out_before;
                for (int x = 0; x < wave; ++x) pos += w_gt[x];
                int out_tot = 0;
                for (int x = 0; x < kTopkWaves; ++x) out_tot += w_gt[x];
                pos += ns_incl - nsel;
                uint32_t bits = sel;
                while (bits) { const int bit = __ffs((int)bits) - 1; out[pos++] = w * 32 + bit; bits &= bits - 1u; }
                eq_before += eq_tot;
                out_before += out_tot;
                __syncthreads();
            }
            if (tid == 0) sel_cnt[b] = k;
            return;
        }
    } else if (nparts > 1) {
        // image span too long for the bitmaps: only the last workgroup works
        if (tid == 0) {
            const uint32_t old = __hip_atomic_fetch_add(&ctr[b].arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == (uint32_t)nparts - 1u;
        }
        __syncthreads();
        if (!s_last) return;
        if (tid == 0) __hip_atomic_store(&ctr[b].arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- select over all N keys ---------------------------------------------------------------------
    uint32_t *keys = (N <= lds_keys) ? dyn_keys : (gkeys + (int64_t)b * bv.max_vis_len);
    for (int i = tid; i < N; i += kTopkThreads) keys[i] = order_key(srow[i]);
    __syncthreads();
    theta = radix_select(keys, N, k, hist, s_pick, &ties);

    // ordered compaction: each wave owns a contiguous index segment
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

// parts per sequence: one 1024-token slice each, at most 64
static int topk_parts(int max_vis_len) { return max(1, min(64, (max_vis_len + kTopkThreads - 1) / kTopkThreads)); }

size_t topk_workspace_bytes(int batch, int max_vis_len)
{
    size_t bytes = 0;
    if (max_vis_len > kLdsKeyCap) bytes += (size_t)batch * (size_t)max_vis_len * sizeof(uint32_t);
    bytes = (bytes + 255) / 256 * 256;
    bytes += (size_t)batch * kCandCap * sizeof(unsigned long long);
    return bytes;
}

hipError_t launch_topk(const float *scores, const BatchDev &bv, int batch, double tau,
                       const int32_t *prev_idx, const int32_t *prev_cnt, int32_t *sel_idx,
                       int32_t *sel_cnt, int64_t kmax, void *ws, hipStream_t stream)
{
    const int lds_keys = bv.max_vis_len <= kLdsKeyCap ? bv.max_vis_len : 0;
    const size_t dyn = (size_t)lds_keys * sizeof(uint32_t);
    static bool attr_set = false;
    if (!attr_set) {
        // gfx950 has 160 KB of LDS per workgroup; the keys of up to 24576 tokens take 96 KB next to
        // the static candidate and bitmap arrays.  If the runtime refuses the opt-in, a launch
        // that needs it reports the error itself.
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(topk_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsKeyCap * (int)sizeof(uint32_t)) != hipSuccess)
            (void)hipGetLastError();
        attr_set = true;
    }
    unsigned char *p = reinterpret_cast<unsigned char *>(ws);
    uint32_t *gkeys = reinterpret_cast<uint32_t *>(p);
    size_t off = 0;
    if (bv.max_vis_len > kLdsKeyCap) off += (size_t)batch * (size_t)bv.max_vis_len * sizeof(uint32_t);
    off = (off + 255) / 256 * 256;
    unsigned long long *cand_list = reinterpret_cast<unsigned long long *>(p + off);
    const int parts = batch <= kTopkMaxBatch ? topk_parts(bv.max_vis_len) : 1;
    static std::atomic<unsigned> call_no{0};
    const int sync_slot = (int)(call_no.fetch_add(1u) % (unsigned)kTopkSlots);
    FASTOCR_LAUNCH(K_TOPK, topk_kernel, dim3(parts, batch), dim3(kTopkThreads), dyn, stream, scores, bv, tau, prev_idx,
                   prev_cnt, sel_idx, sel_cnt, kmax, gkeys, lds_keys, sync_slot, cand_list);
    return hipGetLastError();
}

}  // namespace fastocr
