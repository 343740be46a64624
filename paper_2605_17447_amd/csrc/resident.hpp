// Pieces shared by the two kernels that keep a focal layer's logits in registers
// (score_resident.hip, focal_fused.hip): geometry constants, the tile-list macro, the
// global -> LDS copy and the cross-lane moves.
#pragma once
#include "kernels.hpp"
#include "topk_dev.hpp"

namespace fastocr {

constexpr int kResWaves = 8;
constexpr int kResThreads = 64 * kResWaves;
constexpr int kResTmax = 32;          // image tiles per wave held in registers
constexpr int kResTile = 32;
constexpr int kResMaxHq = 64;
constexpr int kResMaxBatch = 256;

#define RES_EACH_TILE(M)                                                                            \
    M(0) M(1) M(2) M(3) M(4) M(5) M(6) M(7) M(8) M(9) M(10) M(11) M(12) M(13) M(14) M(15)               \
    M(16) M(17) M(18) M(19) M(20) M(21) M(22) M(23) M(24) M(25) M(26) M(27) M(28) M(29) M(30) M(31)
static_assert(kResTmax == 32, "RES_EACH_TILE lists kResTmax tiles");

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds_base + 16 l
// (lds_base is wave-uniform).  Completion is tracked by vmcnt like any other vector load, but the
// compiler does not order later LDS reads after it: the reader waits for vmcnt itself.
__device__ __forceinline__ void lds_dma16(const uint16_t *src, unsigned char *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, /*nt*/ 2);
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}

// Data-parallel-primitive moves within a row of 16 lanes (full-rate VALU, no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i within each 8 lanes
constexpr int kDppRowMirror = 0x140;    // lane i <-> 15 - i within each 16 lanes
constexpr int kDppRor8 = 0x128;         // lane i <- lane i ^ 8

// ---- which (sequence, image-token range) a workgroup of a register-resident kernel works on ------
// The grid has W workgroups (at most one per compute unit).  With sequences of equal length every
// sequence gets W / batch ranges.  In a ragged batch an equal split would leave the chip waiting
// for the longest sequence's few workgroups, so the ranges are dealt in proportion to the sequences'
// token counts: the smallest T with  sum_b max(base_b, ceil(S_b / T)) <= W  (found by bisection) gives sequence b
// nr_b = max(base_b, ceil(S_b / T)) workgroups (base_b = what its image span needs at the most
// tiles a wave can park).  Every wave computes the same table from the device-side lengths (the
// host only knows their maxima): lane l looks after sequences 4l .. 4l+3, so batch <= 256.
struct RangeAlloc {
    int b, rng, nr, wg0;       // sequence, range within it, its range count, its first workgroup
    int R;                     // image tokens per range (a multiple of `unit`)
    int S, v0, N;              // the sequence's geometry
    bool active;               // false: this workgroup has nothing to do
};

__device__ __forceinline__ int wave_total(int x) { return __builtin_amdgcn_readlane(wave_scan_incl(x), 63); }

__device__ __forceinline__ RangeAlloc resident_alloc(const BatchDev &bv, int batch, int W, int nr_uniform, int R_uniform,
                                                     int unit, int w)
{
    const int lane = threadIdx.x & 63;
    const int cap_tokens = kResTmax * unit;
    int S[4], V0[4], N[4];
    bool same = true;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int bb = 4 * lane + j;
        S[j] = 0; V0[j] = 0; N[j] = 0;
        if (bb < batch) {
            const SeqGeom g = seq_geom(bv, bb);
            S[j] = g.S; V0[j] = g.v0; N[j] = g.N;
        }
    }
    const int S0 = __builtin_amdgcn_readlane(S[0], 0), N0 = __builtin_amdgcn_readlane(N[0], 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) same = same && (4 * lane + j >= batch || (S[j] == S0 && N[j] == N0));
    const bool uniform = __builtin_amdgcn_ballot_w64(!same) == 0ull;

    RangeAlloc ra;
    int start[4], cnt[4];
    if (uniform) {
        ra.b = w / nr_uniform;
        ra.rng = w - ra.b * nr_uniform;
        ra.nr = nr_uniform;
        ra.wg0 = ra.b * nr_uniform;
        ra.R = R_uniform;
        ra.active = ra.b < batch;
    } else {
        int wt[4], base[4], part = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool live = 4 * lane + j < batch;
            wt[j] = live ? max(S[j], 1) : 0;
            base[j] = live ? max(1, (N[j] + cap_tokens - 1) / cap_tokens) : 0;
            part += wt[j];
        }
        const int total = wave_total(part);
        auto need = [&](int T) {
            int f = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) f += wt[j] > 0 ? max(base[j], (wt[j] + T - 1) / T) : 0;
            return wave_total(f);
        };
        // T = max_seq_len always fits (every sequence then takes base_b workgroups, and the host has
        // checked that batch * max base <= W); bisect down from there to the smallest T that fits
        int lo = max(1, (total + W - 1) / W) - 1, hi = max(bv.max_seq_len, 1);
        if (lo + 1 <= hi && need(lo + 1) <= W) hi = lo + 1;
        while (hi - lo > 1) {
            const int mid = lo + (hi - lo) / 2;
            if (need(mid) <= W) hi = mid; else lo = mid;
        }
        const int T = hi;
        const bool fits = true;
        int mine = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            cnt[j] = wt[j] > 0 ? (fits ? max(base[j], (wt[j] + T - 1) / T) : base[j]) : 0;
            start[j] = mine;
            mine += cnt[j];
        }
        const int before = wave_scan_incl(mine) - mine;
        int fb = 0, fr = 0, fn = 0, f0 = 0;
        bool found = false;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s0 = before + start[j];
            if (cnt[j] > 0 && w >= s0 && w < s0 + cnt[j]) { found = true; fb = 4 * lane + j; fr = w - s0; fn = cnt[j]; f0 = s0; }
        }
        const unsigned long long who = __builtin_amdgcn_ballot_w64(found);
        ra.active = who != 0ull;
        const int owner = ra.active ? __builtin_amdgcn_readfirstlane(__ffsll((long long)who) - 1) : 0;
        ra.b = __builtin_amdgcn_readlane(fb, owner);
        ra.rng = __builtin_amdgcn_readlane(fr, owner);
        ra.nr = __builtin_amdgcn_readlane(fn, owner);
        ra.wg0 = __builtin_amdgcn_readlane(f0, owner);
        ra.R = 0;
    }
    // the sequence's geometry from the lane that loaded it
    const int ol = __builtin_amdgcn_readfirstlane(min(ra.b, 255) >> 2), oj = ra.b & 3;
    const int ps = oj == 0 ? S[0] : (oj == 1 ? S[1] : (oj == 2 ? S[2] : S[3]));
    const int pv = oj == 0 ? V0[0] : (oj == 1 ? V0[1] : (oj == 2 ? V0[2] : V0[3]));
    const int pn = oj == 0 ? N[0] : (oj == 1 ? N[1] : (oj == 2 ? N[2] : N[3]));
    ra.S = __builtin_amdgcn_readlane(ps, ol);
    ra.v0 = __builtin_amdgcn_readlane(pv, ol);
    ra.N = __builtin_amdgcn_readlane(pn, ol);
    if (!uniform) ra.R = max(unit, ((ra.N + ra.nr - 1) / max(ra.nr, 1) + unit - 1) / unit * unit);
    return ra;
}

// ---- exchange of the ranges' softmax statistics ----------------------------------------------------
// One 64-bit word {max, sum-exp} per (workgroup, head) in static device memory; zero means "not
// published yet" (a published word is never zero: the sum is positive, or the maximum is the finite
// stand-in for "no logit").  The words cross compute units (and XCDs, each with its own L2) through
// agent-scope atomic stores and loads, which go through to memory, instead of plain stores bracketed
// by release/acquire fences: a fence writes back or invalidates the XCD's whole L2 and costs
// microseconds.  Every word is its own "ready" flag, so nothing has to be ordered: a reader polls
// until the words it needs are non-zero.  The last range of a sequence to finish reading zeroes the
// sequence's words again (resident_retire), so a slot is clean when its call ends.
constexpr int kResMaxWg = 256;

// (max, sum-exp) of head h over this workgroup's waves, from the per-wave values in LDS
__device__ __forceinline__ void resident_own_stats(const float (*sm_m)[8], const float (*sm_z)[8], int h, int G, int Hkv,
                                                   int wpk, float &M, float &Z)
{
    const int g = h / G, x = h - g * G;
    M = kMinusHuge;
    Z = 0.f;
    for (int sb = 0; sb < wpk; ++sb) softmax_merge(M, Z, sm_m[g + sb * Hkv][x], sm_z[g + sb * Hkv][x]);
}

// threads 0 .. Hq-1 publish this range's row; no wait, no ordering
__device__ __forceinline__ void resident_publish(unsigned long long *row, const float (*sm_m)[8], const float (*sm_z)[8],
                                                 int Hq, int G, int Hkv, int wpk)
{
    if ((int)threadIdx.x < Hq) {
        float M, Z;
        resident_own_stats(sm_m, sm_z, threadIdx.x, G, Hkv, wpk, M, Z);
        const unsigned long long mz = (unsigned long long)__float_as_uint(M) | ((unsigned long long)__float_as_uint(Z) << 32);
        __hip_atomic_store(&row[threadIdx.x], mz, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Gathering the statistics: a wave needs the sequence-wide (reference, sum) of ITS OWN group of heads
// only (kv head kvh: heads kvh*G .. kvh*G+G-1), which is all it takes to finish its own weights: no
// exchange between the workgroup's waves, no barrier.  Lane 8s + x looks after head x of the group
// in the ranges s, s + 8, s + 16, ..; the eight partial results per head are then combined with lane
// moves, and every lane with the same x ends up with the same pair.  GROUP words per lane are
// requested together and polled until every one is there (one memory round trip per attempt; only
// what is still missing is asked for again: a few hundred bytes per attempt, served by the
// memory-side cache, next to nothing against the ranges still streaming).  resident_heads_request
// sends the first attempt for the first group without waiting, so that its round trip can pass
// behind other work; resident_heads_gather takes its answer as the first attempt.  The workgroup's
// own statistics never leave the chip.  Returns false when a word did not appear within spin_ticks
// of the 100 MHz wall clock.
template <int GROUP>
struct StatRows { unsigned long long mz[GROUP]; };

template <int GROUP>
__device__ __forceinline__ StatRows<GROUP> resident_heads_request(const unsigned long long *stats, int rng, int nranges, int Hq,
                                                                  int G, int kvh, int i0 = 0)
{
    const int lane = threadIdx.x & 63, x = lane & 7, s = lane >> 3;
    StatRows<GROUP> rows;
#pragma unroll
    for (int j = 0; j < GROUP; ++j) {
        const int rr = s + 8 * (i0 + j);
        rows.mz[j] = 1ull;                                       // nothing to read: counts as there
        if (rr < nranges && rr != rng && x < G)
            rows.mz[j] = __hip_atomic_load(stats + (int64_t)rr * Hq + kvh * G + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return rows;
}

template <int GROUP>
__device__ __forceinline__ bool resident_heads_gather(const unsigned long long *stats, int rng, int nranges, int Hq, int G,
                                                      int Hkv, int wpk, int kvh, const float (*sm_m)[8], const float (*sm_z)[8],
                                                      long long spin_ticks, float &M, float &Z, const StatRows<GROUP> *first = nullptr)
{
    const int lane = threadIdx.x & 63, x = lane & 7, s = lane >> 3;
    M = kMinusHuge;
    Z = 0.f;
    const long long t_start = wall_clock64();
    const int rounds = (nranges + 7) / 8;
    for (int i0 = 0; i0 < rounds; i0 += GROUP) {
        StatRows<GROUP> rows = (first != nullptr && i0 == 0) ? *first : resident_heads_request<GROUP>(stats, rng, nranges, Hq, G, kvh, i0);
        while (true) {
            bool missing = false;
#pragma unroll
            for (int j = 0; j < GROUP; ++j) missing = missing || rows.mz[j] == 0ull;
            if (__builtin_amdgcn_ballot_w64(missing) == 0ull) break;
            __builtin_amdgcn_s_sleep(1);
            if (wall_clock64() - t_start > spin_ticks) return false;
#pragma unroll
            for (int j = 0; j < GROUP; ++j) {
                const int rr = s + 8 * (i0 + j);
                if (rows.mz[j] == 0ull)                          // (zero only where this lane has something to read)
                    rows.mz[j] = __hip_atomic_load(stats + (int64_t)rr * Hq + kvh * G + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
#pragma unroll
        for (int j = 0; j < GROUP; ++j) {
            const int rr = s + 8 * (i0 + j);
            if (rr >= nranges || x >= G) continue;
            if (rr == rng) {
                float Mo, Zo;
                resident_own_stats(sm_m, sm_z, kvh * G + x, G, Hkv, wpk, Mo, Zo);
                softmax_merge(M, Z, Mo, Zo);
            } else {
                softmax_merge(M, Z, __uint_as_float((uint32_t)rows.mz[j]), __uint_as_float((uint32_t)(rows.mz[j] >> 32)));
            }
        }
    }
    // the eight lanes of a head (8 apart): the other half of the row, the next row, the other half of the wave
    softmax_merge(M, Z, dpp_move<kDppRor8>(M), dpp_move<kDppRor8>(Z));
    {
        const uint32_t mu = __builtin_bit_cast(uint32_t, M), zu = __builtin_bit_cast(uint32_t, Z);
        const auto ms = __builtin_amdgcn_permlane16_swap(mu, mu, false, false);
        const auto zs = __builtin_amdgcn_permlane16_swap(zu, zu, false, false);
        M = __builtin_bit_cast(float, (uint32_t)ms[0]);
        Z = __builtin_bit_cast(float, (uint32_t)zs[0]);
        softmax_merge(M, Z, __builtin_bit_cast(float, (uint32_t)ms[1]), __builtin_bit_cast(float, (uint32_t)zs[1]));
    }
    {
        const uint32_t mu = __builtin_bit_cast(uint32_t, M), zu = __builtin_bit_cast(uint32_t, Z);
        const auto ms = __builtin_amdgcn_permlane32_swap(mu, mu, false, false);
        const auto zs = __builtin_amdgcn_permlane32_swap(zu, zu, false, false);
        M = __builtin_bit_cast(float, (uint32_t)ms[0]);
        Z = __builtin_bit_cast(float, (uint32_t)zs[0]);
        softmax_merge(M, Z, __builtin_bit_cast(float, (uint32_t)ms[1]), __builtin_bit_cast(float, (uint32_t)zs[1]));
    }
    return true;
}

// Called by every thread when the workgroup is done reading (after a __syncthreads): `last` says
// whether this range was the sequence's last to finish reading; it then clears the sequence's words
// and the count.
__device__ __forceinline__ void resident_retire(bool last, unsigned long long *stats, int nranges, int Hq, uint32_t *left)
{
    if (last) {
        for (int i = threadIdx.x; i < nranges * Hq; i += kResThreads)
            __hip_atomic_store(&stats[i], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (threadIdx.x == 0) __hip_atomic_store(left, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---- top-k of the finished scores inside the same launch --------------------------------------------
// (Sec. 3.1.2: TopK is applied directly to the focal layer's head-averaged attention.)  Every range
// stores its scores with agent-scope stores, waits until they have been performed, and counts
// itself out on a per-sequence counter; the range that counts last -- every score of its sequence
// is then visible at agent scope -- runs the exact register select of topk_dev.hpp over the whole
// sequence (512 threads x 32 keys) and writes the set.  Nobody waits for anybody: no polling, no
// fence.  The selecting workgroup leaves the counter at zero for the next call on the slot.
constexpr int kSelPer = 32;
constexpr int kSelMaxKeys = kResThreads * kSelPer;               // 16384 image tokens per sequence
constexpr int kSelLdsBytes = 4 * kWinBins + 4 * kWinListWords + 256;

template <bool SELECT>
__device__ __forceinline__ void store_score(float *p, float x)
{
    if (SELECT) __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = x;
}

// Called by every thread of a range's workgroup after its scores have been stored with
// store_score<true>.  lds: at least kSelLdsBytes of the workgroup's LDS that nobody uses any more.
// The select's arguments are the kernel's FIRST argument and are read from the kernel-argument
// segment here, when they are needed: as ordinary arguments they would sit in scalar registers
// through the whole tile loop, which has none to spare.
// (The batch description is read there too, rather than kept across the tile loop.)
struct ResidentArgsHead {       // how both kernels' argument lists begin
    SelectArgs sel;
    KvDev kv;
    BatchDev bv;
};

__device__ __forceinline__ void resident_select_tail(const float *scores, int b, int nranges, uint32_t *done, unsigned char *lds)
{
    __shared__ int sm_selects;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // this thread's score stores have been performed
    __syncthreads();                                         // ... and every other thread's of the workgroup
    if (threadIdx.x == 0) {
        const uint32_t before = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm_selects = before == (uint32_t)nranges - 1u;
    }
    __syncthreads();
    if (!sm_selects) return;
    const ResidentArgsHead *ka = (const ResidentArgsHead *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ka)::"memory");
    const SelectArgs sa = ka->sel;
    const BatchDev bv = ka->bv;
    TopkRegShared sh;
    sh.hist = reinterpret_cast<uint32_t *>(lds);
    sh.list = reinterpret_cast<uint32_t *>(lds + 4 * kWinBins);
    int *misc = reinterpret_cast<int *>(lds + 4 * kWinBins + 4 * kWinListWords);
    sh.w_ac = misc;                                          // 4 * 8 wave values, 16-byte aligned
    sh.pick = misc + 32;
    topk_reg_body<kResThreads, kSelPer, true, false>(scores, bv, b, sa.tau, sa.prev_idx, sa.prev_cnt, sa.sel_idx, sa.sel_cnt,
                                              sa.kmax, sh, [](int, int) {});
    if (threadIdx.x == 0) __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace fastocr
