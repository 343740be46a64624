// Focal layer in one pass (Sec. 3.1.1, Eq. 1; Alg. 1, focal branch): the layer's dense decode
// attention output AND the head-averaged focal scores of the image tokens from a single read
// of K and V.  A focal layer needs both -- its own attention output over the full cache and the
// scores that the following layers' fixation sets are cut from -- and K is the larger part of
// either computation's traffic, so reading it twice (dense attention, then scoring) wastes a
// third of the bytes.
//
// Structure (shared with the scoring-only kernel in score_resident.hip):
//   - one 512-thread workgroup per (image-token range, sequence), at most one per compute unit,
//     so the whole grid is resident; wave w streams KV head w % Hkv in 32-token tiles;
//   - K and V tiles travel HBM -> LDS directly (one 8 KB slot each per wave); the next K tile is
//     requested as soon as the current one has been read into registers, likewise for V, so one
//     tile of each is always in flight while the other is being consumed;
//   - logits are produced transposed, C[token][column]: columns 0..7 are the group's heads for
//     the tile's first 16 tokens, columns 8..15 the same heads for its last 16 (two accumulators,
//     one select), so every lane holds 4 logits of ONE head; they stay in 4 VGPRs named for the
//     tile until the normalisers are known;
//   - the same layout serves P*V: with P masked to "first-half tokens in columns 0..7, second-half
//     tokens in columns 8..15" one v_mfma_f32_16x16x32_bf16 per 16 output dims accumulates
//     O^T[dim][column]; columns n and n+8 are the two halves' partial sums of head n and are added
//     at the end.  The running maximum of a head is uniform over the wave (it scales whole
//     accumulator columns); rescaling happens only in tiles where some head's maximum grew;
//   - each wave leaves an attention partial (accumulator, max, sum) in the workspace for the
//     split-merge kernel of attn.hip; the ranges then exchange their softmax statistics, meet at
//     the per-sequence barrier and turn the parked logits into scores exactly as the
//     scoring-only kernel does.
#include "kernels.hpp"
#include "resident.hpp"

namespace fastocr {

// statistics words per (workgroup, head), per sequence the count of ranges done reading, and a
// count of the waves that gave up waiting: same protocol as score_resident.hip, own arrays
__device__ unsigned long long g_fus_stats[kResSlots][kResMaxWg * kResMaxHq];
__device__ uint32_t g_fus_left[kResSlots][kResMaxBatch];
__device__ uint32_t g_fus_timeouts;
__device__ uint32_t g_fus_done[kResSlots][kResMaxBatch];     // fused top-k: ranges of a sequence whose scores are out

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// One logit per image tile of the wave, indexed by the (wave-uniform) tile number: the compiler
// keeps such a vector in 32 consecutive VGPRs and addresses it through the register-index mode,
// so the tile loop stays a loop instead of 32 unrolled copies that overflow the instruction cache.
typedef float f32x32 __attribute__((ext_vector_type(32)));
static_assert(kResTmax == 32, "one f32x32 per logit row holds kResTmax tiles");

template <bool PAGED, bool SELECT>
__global__ __launch_bounds__(kResThreads) void focal_fused_kernel(
    SelectArgs sel_args /* first: read straight from the kernel-argument segment when the select starts */,
    KvDev kv, BatchDev bv, const uint16_t *__restrict__ q, int Hq, int G, float scale_log2,
    int batch, int nranges_uniform, int R_uniform, int sync_slot, long long spin_ticks,
    float *__restrict__ scores, float *__restrict__ lse_out, float *__restrict__ mass_part,
    float *__restrict__ att_o, float *__restrict__ att_ml, int32_t *__restrict__ seq_meta,
    uint32_t *__restrict__ gave_up_flag)
{
    static_assert(sizeof(unsigned char[kResWaves][2][8192]) >= (size_t)kSelLdsBytes, "the select reuses the tile buffers");
    __shared__ __align__(16) unsigned char smem[kResWaves][2][8192];      // [wave][K, V]
    __shared__ float sm_m[kResWaves][8], sm_z[kResWaves][8];
    __shared__ float sm_red[kResWaves];
    __shared__ int sm_met, sm_last;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int Hkv = kv.n_kv_heads;
    const int wpk = kResWaves / Hkv;
    const int kvh = wave % Hkv, sub = wave / Hkv;

    // which sequence and which of its ranges (all wave-uniform); ragged batches get ranges in
    // proportion to their lengths
    const RangeAlloc ra = resident_alloc(bv, batch, gridDim.x, nranges_uniform, R_uniform, kResTile * wpk, blockIdx.x);
    if (!ra.active) return;
    const int rng = ra.rng, b = ra.b, nranges = ra.nr, R = ra.R, wg0 = ra.wg0;
    const int S = ra.S, v0 = ra.v0, N = ra.N;
    // where the sequence's partials are, for the merge and image-mass kernels that follow
    if (rng == 0 && threadIdx.x == 0) { seq_meta[2 * b] = wg0; seq_meta[2 * b + 1] = nranges; }
    const int Tn = S - N;

    // image tiles of this wave: tile ti = sub + j*wpk of the range, j = 0 .. nimg-1
    const int r0 = rng * R, r1 = min(N, r0 + R);
    const int nt_range = r1 > r0 ? (r1 - r0 + kResTile - 1) / kResTile : 0;
    const int nimg = min(nt_range > sub ? (nt_range - sub + wpk - 1) / wpk : 0, kResTmax);
    // text tiles of this wave: u = slot + i*nslots
    const int ntt = (Tn + kResTile - 1) / kResTile;
    const int slot = rng * wpk + sub, nslots = nranges * wpk;
    const int ntext = ntt > slot ? (ntt - slot + nslots - 1) / nslots : 0;

    // Q as the B operand of the logits: column n = li holds head n & 7 of the group
    const int hcol = li & 7;
    const bool hi = li >= 8;                     // this lane's logits belong to the tile's last 16 tokens
    u32x4 qq[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        qq[kk] = u32x4{0u, 0u, 0u, 0u};
        if (hcol < G)
            qq[kk] = *reinterpret_cast<const u32x4 *>(q + ((int64_t)b * Hq + (int64_t)kvh * G + hcol) * 128 + 8 * (4 * kk + lg));
    }
    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(kv.k);
    const uint16_t *vbase = reinterpret_cast<const uint16_t *>(kv.v);

    const int rot = nimg > 0 ? (wave * 5 + rng * 3 + b * 7) % nimg : 0;
    auto img_first = [&](int x) {                                                  // span-relative
        int j = x + rot;
        j = j >= nimg ? j - nimg : j;
        return r0 + (sub + j * wpk) * kResTile;
    };
    auto text_first = [&](int x) { return (slot + x * nslots) * kResTile; };       // text-relative

    // A tile goes into the wave's K or V slot: load e brings rows 4e .. 4e+3, lane (lg, li) one
    // 16-byte chunk of row 4e + lg, which lands at slot + 1024 e + 16 lane.  For K the chunk is
    // li ^ (row & 15) (the swizzle that makes the MFMA operand reads conflict-free); V stays
    // row-major (chunk li).  Rows past the end of a ragged tile are clamped to its last row.
    const int64_t seq_base = row_offset<false>(kv, b, 0, kvh);
    const uint32_t stride_b = (uint32_t)kv.stride_token * 2u;            // bytes; 32 rows fit 32 bits (host-checked)
    const uint32_t rowoff_lg = (uint32_t)lg * stride_b;
    uint32_t chunk_k[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) chunk_k[k] = 16u * (uint32_t)((li ^ lg) ^ (4 * k));
    const uint32_t chunk_v = 16u * (uint32_t)li;
    const unsigned char *kbytes = reinterpret_cast<const unsigned char *>(kv.k);
    const unsigned char *vbytes = reinterpret_cast<const unsigned char *>(kv.v);

    auto issue_run = [&](int first_tok, int rv, bool isv) {
        unsigned char *dst = smem[wave][isv ? 1 : 0];
        const unsigned char *bytes = isv ? vbytes : kbytes;
        const uint32_t limit = (uint32_t)(rv - 1) * stride_b;
        if (PAGED) {
            const int pt = kv.page_tokens;
            const int pg0 = first_tok / pt, in0 = first_tok - pg0 * pt;
            const int32_t *bt = kv.block_table + (int64_t)b * kv.max_pages;
            const int64_t pa = bt[min(pg0, kv.max_pages - 1)], pb = bt[min(pg0 + 1, kv.max_pages - 1)];
            const unsigned char *base_a = bytes + 2 * (pa * kv.stride_page + (int64_t)kvh * kv.stride_head + (int64_t)in0 * kv.stride_token);
            const unsigned char *base_b = bytes + 2 * (pb * kv.stride_page + (int64_t)kvh * kv.stride_head + (int64_t)(in0 - pt) * kv.stride_token);
            const uint32_t split = (uint32_t)(pt - in0) * stride_b;      // first byte offset of the second page
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t ro = min(rowoff_lg + (uint32_t)(4 * e) * stride_b, limit);
                const unsigned char *base = ro >= split ? base_b : base_a;
                lds_dma16(reinterpret_cast<const uint16_t *>(base + (ro + (isv ? chunk_v : chunk_k[e & 3]))), dst + 1024 * e);
            }
        } else {
            const unsigned char *base = bytes + 2 * (seq_base + (int64_t)first_tok * kv.stride_token);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t ro = min(rowoff_lg + (uint32_t)(4 * e) * stride_b, limit);
                lds_dma16(reinterpret_cast<const uint16_t *>(base + (ro + (isv ? chunk_v : chunk_k[e & 3]))), dst + 1024 * e);
            }
        }
    };
    // Past the wave's last tile the refill stays unconditional (the readers' "at most 8 loads
    // outstanding" waits count on it) but fetches 256 bytes of the query, which are in cache.
    const uint16_t *qrow = q + ((int64_t)b * Hq + (int64_t)kvh * G) * 128;
    auto issue_dummy = [&](bool isv) {
        unsigned char *dst = smem[wave][isv ? 1 : 0];
#pragma unroll
        for (int e = 0; e < 8; ++e) lds_dma16(qrow + chunk_v / 2, dst + 1024 * e);
    };
    auto issue_img = [&](int x, bool isv) {
        if (x >= nimg) { issue_dummy(isv); return; }
        const int jf = img_first(x);
        issue_run(v0 + jf, min(kResTile, r1 - jf), isv);
    };
    // text positions map to tokens with a gap at the image span, so the rows are addressed one by one
    auto issue_text = [&](int x, bool isv) {
        const int tf = text_first(x);
        unsigned char *dst = smem[wave][isv ? 1 : 0];
        const uint16_t *base = isv ? vbase : kbase;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int tc = min(tf + 4 * e + lg, Tn - 1);
            const int tok = tc < v0 ? tc : tc + N;
            lds_dma16(base + row_offset<PAGED>(kv, b, tok, kvh) + (isv ? chunk_v : chunk_k[e & 3]) / 2, dst + 1024 * e);
        }
    };
    // tile number n of the wave (text tiles first, then image tiles), or the dummy past the end
    auto issue_any = [&](int n, bool isv) {
        if (n < ntext) issue_text(n, isv);
        else issue_img(n - ntext, isv);
    };

    const int tt0 = 16 * (li >> 3) + 4 * lg;        // tile-relative token of this lane's first logit
    float m = kMinusHuge, z = 0.f;                  // running max (uniform over the head's lanes), this lane's sum
    f32x4 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // LDS byte addresses: K rows li and 16 + li as the A operand, V rows 4lg.. and 16 + 4lg..
    uint32_t rd_addr[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        rd_addr[kk] = lds_address(&smem[wave][0][0]) + li * 256 + ((((4 * kk + lg) ^ li) & 15) << 4);
    const uint32_t rd_v = lds_address(&smem[wave][1][0]) + (4 * lg) * 256 + li * 16;

    // The newest outstanding loads are always the 8 of the other slot's refill, so "at most 8
    // outstanding" means the tile wanted here has landed.  Reads and waits are written in assembly:
    // the compiler neither orders LDS reads after loads that land in LDS by themselves without
    // draining ALL of them, nor may it move the products above the wait.
    // rows li (first call) and 16 + li (second call) of the K tile, in two halves so that only
    // four operand registers are live at a time
    auto read_k_lo = [&](u32x4(&kb)[4]) {
        asm volatile(
            "s_waitcnt vmcnt(8)\n\t"
            "ds_read_b128 %0, %4\n\t"
            "ds_read_b128 %1, %5\n\t"
            "ds_read_b128 %2, %6\n\t"
            "ds_read_b128 %3, %7\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(kb[0]), "=&v"(kb[1]), "=&v"(kb[2]), "=&v"(kb[3])
            : "v"(rd_addr[0]), "v"(rd_addr[1]), "v"(rd_addr[2]), "v"(rd_addr[3])
            : "memory");
    };
    auto read_k_hi = [&](u32x4(&kb)[4]) {
        asm volatile(
            "ds_read_b128 %0, %4 offset:4096\n\t"
            "ds_read_b128 %1, %5 offset:4096\n\t"
            "ds_read_b128 %2, %6 offset:4096\n\t"
            "ds_read_b128 %3, %7 offset:4096\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(kb[0]), "=&v"(kb[1]), "=&v"(kb[2]), "=&v"(kb[3])
            : "v"(rd_addr[0]), "v"(rd_addr[1]), "v"(rd_addr[2]), "v"(rd_addr[3])
            : "memory");
    };
    // vv[e]: dims 8li .. 8li+7 of token 4lg + e (e < 4) or 16 + 4lg + e - 4 of the tile
    auto read_v = [&](u32x4(&vv)[8]) {
        asm volatile(
            "s_waitcnt vmcnt(8)\n\t"
            "ds_read_b128 %0, %8\n\t"
            "ds_read_b128 %1, %8 offset:256\n\t"
            "ds_read_b128 %2, %8 offset:512\n\t"
            "ds_read_b128 %3, %8 offset:768\n\t"
            "ds_read_b128 %4, %8 offset:4096\n\t"
            "ds_read_b128 %5, %8 offset:4352\n\t"
            "ds_read_b128 %6, %8 offset:4608\n\t"
            "ds_read_b128 %7, %8 offset:4864\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(vv[0]), "=&v"(vv[1]), "=&v"(vv[2]), "=&v"(vv[3]), "=&v"(vv[4]), "=&v"(vv[5]), "=&v"(vv[6]), "=&v"(vv[7])
            : "v"(rd_v)
            : "memory");
    };

    // One tile: logits, online softmax, P*V.  nlive = tokens of the tile that exist (may exceed 32).
    // Returns this lane's 4 logits (log2 domain; -inf for tokens past the end).
    auto tile_step = [&](int nlive, auto &&next_k, auto &&next_v) -> f32x4 {
        u32x4 kb[4];
        f32x4 c0 = f32x4{0.f, 0.f, 0.f, 0.f}, c1 = c0;
        read_k_lo(kb);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[kk]),
                                                         __builtin_bit_cast(bf16x8, qq[kk]), c0, 0, 0, 0);
        read_k_hi(kb);
        next_k();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[kk]),
                                                         __builtin_bit_cast(bf16x8, qq[kk]), c1, 0, 0, 0);
        f32x4 s;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float x = hi ? c1[r] : c0[r];
            s[r] = (tt0 + r < nlive) ? x * scale_log2 : -INFINITY;
        }
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        mx = fmaxf(mx, dpp_move<kDppRor8>(mx));
        mx = rows_max(mx);
        const float m_new = fmaxf(m, mx);
        if (__builtin_amdgcn_ballot_w64(m_new != m) != 0ull) {
            const float alpha = fast_exp2(m - m_new);
            z *= alpha;
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[t] *= alpha;
            m = m_new;
        }
        float p[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) p[r] = fast_exp2(s[r] - m);
        z += (p[0] + p[1]) + (p[2] + p[3]);
        const uint32_t w0 = __builtin_bit_cast(uint32_t, bf16x2{(__bf16)p[0], (__bf16)p[1]});
        const uint32_t w1 = __builtin_bit_cast(uint32_t, bf16x2{(__bf16)p[2], (__bf16)p[3]});
        // contraction slots of lane group lg: tokens 4lg..4lg+3, then 16+4lg..16+4lg+3
        const u32x4 pb = u32x4{hi ? 0u : w0, hi ? 0u : w1, hi ? w0 : 0u, hi ? w1 : 0u};

        u32x4 vv[8];
        read_v(vv);
        next_v();
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int w = t >> 1;
            const uint32_t selb = (t & 1) ? 0x07060302u : 0x05040100u;
            u32x4 a;
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) a[pp] = __builtin_amdgcn_perm(vv[2 * pp + 1][w], vv[2 * pp][w], selb);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                             __builtin_bit_cast(bf16x8, pb), acc[t], 0, 0, 0);
        }
        return s;
    };

    // ---- stream: text tiles, then image tiles (logits parked in registers) ----------------------
    f32x32 park0, park1, park2, park3;          // logit r of image tile J in park<r>[J]
    if (ntext + nimg > 0) {
        issue_any(0, false);
        issue_any(0, true);
        for (int x = 0; x < ntext; ++x)
            (void)tile_step(Tn - text_first(x), [&]() { issue_any(x + 1, false); }, [&]() { issue_any(x + 1, true); });
        for (int J = 0; J < nimg; ++J) {
            const f32x4 s = tile_step(r1 - img_first(J), [&]() { issue_img(J + 1, false); }, [&]() { issue_img(J + 1, true); });
            park0[J] = s[0];
            park1[J] = s[1];
            park2[J] = s[2];
            park3[J] = s[3];
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the trailing refills must not land later

    // Lane coordinates are derived afresh for the rest of the kernel: carried across the tile loop
    // they would occupy registers it has no room for.
    int tx_p = threadIdx.x;
    asm volatile("" : "+v"(tx_p));
    const int lane_p = tx_p & 63, li_p = lane_p & 15, lg_p = lane_p >> 4, hcol_p = li_p & 7;
    const int tt0_p = 16 * (li_p >> 3) + 4 * lg_p;

    // ---- attention partial of this wave: O^T columns n and n + 8 are the same head's halves -----
    z += dpp_move<kDppRor8>(z);
    z = rows_sum(z);
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] += dpp_move<kDppRor8>(acc[t][r]);
    if (li_p < 8 && li_p < G) {
        // lane_p (head li_p, group lg_p) holds dims 32lg + 8r + t in acc[t][r]
        const int64_t row = ((int64_t)(wg0 + rng) * wpk + sub) * Hq + kvh * G + li_p;      // [workgroup][sub][head]
        float *po = att_o + row * 128 + 32 * lg_p;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            *reinterpret_cast<f32x4 *>(po + 8 * r) = f32x4{acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
            *reinterpret_cast<f32x4 *>(po + 8 * r + 4) = f32x4{acc[4][r], acc[5][r], acc[6][r], acc[7][r]};
        }
        if (lg_p == 0) {
            att_ml[2 * row] = m;
            att_ml[2 * row + 1] = z;
            sm_m[wave][li_p] = m;
            sm_z[wave][li_p] = z;
        }
    }
    if (threadIdx.x == 0) sm_met = 1;
    __syncthreads();

    // ---- range statistics: published as self-validating words, gathered by polling (resident.hpp) ----
    // (Asking for the other ranges' words before the partial is written, as the scoring kernel does at the
    // end of its stream, gains 0.4 us at the largest shapes and loses 2 us at the small ones, where the
    // ranges end together, the first answer comes back incomplete and a second round trip follows.)
    unsigned long long *stats = g_fus_stats[sync_slot] + (int64_t)wg0 * Hq;
    resident_publish(stats + (int64_t)rng * Hq, sm_m, sm_z, Hq, G, Hkv, wpk);
    // the log-sum-exp of this wave's heads over the whole sequence (lane 8s + x: head x of the group)
    float lh;
    {
        float M, Z;
        const bool ok = resident_heads_gather<4>(stats, rng, nranges, Hq, G, Hkv, wpk, kvh, sm_m, sm_z, spin_ticks, M, Z);
        if (!ok && lane_p == 0) {
            sm_met = 0;
            __hip_atomic_fetch_add(&g_fus_timeouts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (gave_up_flag) __hip_atomic_store(gave_up_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        lh = (hcol_p < G && Z > 0.f) ? M + log2f(Z) : (hcol_p < G ? -INFINITY : INFINITY);
    }
    __syncthreads();      // whether every wave has met its ranges
    // This range is done reading: count it out.  The last one of the sequence clears the
    // sequence's words and the count when the kernel ends.
    uint32_t *left = &g_fus_left[sync_slot][b];
    // (the count's old value is only looked at when the kernel ends: nobody waits for the atomic)
    uint32_t left_before = 0u;
    if (threadIdx.x == 0) left_before = __hip_atomic_fetch_add(left, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    auto leave = [&]() {
        if (threadIdx.x == 0) sm_last = left_before == (uint32_t)nranges - 1u;
        __syncthreads();
        resident_retire(sm_last != 0, stats, nranges, Hq, left);
    };
    if (!sm_met) {
        // a range of the sequence never published: poison this range's scores
        for (int i = threadIdx.x; i < r1 - r0; i += kResThreads)
            store_score<SELECT>(&scores[(int64_t)b * bv.max_vis_len + r0 + i], __builtin_nanf(""));
        if (SELECT) resident_select_tail(scores, b, nranges, &g_fus_done[sync_slot][b], &smem[0][0][0]);
        leave();
        return;
    }
    if (lse_out && rng == 0 && sub == 0 && lane_p < G) lse_out[(int64_t)b * Hq + kvh * G + lane_p] = lh * kLn2;

    // ---- probabilities of the parked logits, summed over the heads of each token ---------------
    float *red = reinterpret_cast<float *>(&smem[0][0][0]);          // [Hkv][R], at most 32 KB
    for (int J = 0; J < nimg; ++J) {
        // this lane_p's 4 tokens of tile J, one head each on 8 neighbouring lanes
        f32x4 v = f32x4{park0[J], park1[J], park2[J], park3[J]};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float x = fast_exp2(v[r] - lh);
            x += dpp_move<kDppXor1>(x);
            x += dpp_move<kDppXor2>(x);
            x += dpp_move<kDppHalfMirror>(x);
            v[r] = x;
        }
        if ((li_p & 7) == 0) *reinterpret_cast<f32x4 *>(&red[kvh * R + img_first(J) - r0 + tt0_p]) = v;
    }
    __syncthreads();
    float local = 0.f;
    const float inv = 1.0f / (float)Hq;
    for (int i = threadIdx.x; i < r1 - r0; i += kResThreads) {
        float a = 0.f;
        for (int g = 0; g < Hkv; ++g) a += red[g * R + i];
        a *= inv;
        store_score<SELECT>(&scores[(int64_t)b * bv.max_vis_len + r0 + i], a);
        local += a;
    }
    if (mass_part) {
        local = wave_sum(local);
        if (lane_p == 0) sm_red[wave] = local;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            for (int w = 0; w < kResWaves; ++w) t += sm_red[w];
            mass_part[wg0 + rng] = t;
        }
    }
    if (SELECT) resident_select_tail(scores, b, nranges, &g_fus_done[sync_slot][b], &smem[0][0][0]);
    leave();
}

__global__ void fused_mass_kernel(const float *__restrict__ mass_part, const int32_t *__restrict__ seq_meta,
                                  float *__restrict__ img_mass)
{
    const int b = blockIdx.x;
    const int first = seq_meta[2 * b], n = seq_meta[2 * b + 1];
    float t = 0.f;
    for (int x = threadIdx.x; x < n; x += 64) t += mass_part[first + x];
    t = wave_sum(t);
    if (threadIdx.x == 0) img_mass[b] = t;
}

// Workspace, with W = nranges * batch workgroups: attention partials fp32 [W][wpk][Hq][128] and
// [W][wpk][Hq][2], image-mass partials [W], and per sequence
// its first workgroup and range count int32 [B][2].
size_t focal_fused_workspace_bytes(const Shape &s, const ResidentPlan &p)
{
    const size_t W = (size_t)p.nranges * s.batch;
    size_t bytes = W * p.wpk * s.n_q_heads * (128 + 2) * sizeof(float);
    bytes += W * sizeof(float);
    bytes += (size_t)s.batch * 2 * sizeof(int32_t);
    return bytes;
}

hipError_t focal_fused_timeouts(uint32_t *n) { return hipMemcpyFromSymbol(n, HIP_SYMBOL(g_fus_timeouts), sizeof(uint32_t)); }

hipError_t launch_focal_fused(const Shape &s, const ResidentPlan &p, int sync_slot, uint32_t *flag, const void *q, float scale,
                              void *out, float *scores, float *lse, float *img_mass, void *ws, hipStream_t stream,
                              const SelectArgs *select, CombineArgs *defer)
{
    if (sync_slot < 0 || sync_slot >= kResSlots) return hipErrorInvalidValue;
    const int W = p.nranges * s.batch;
    float *att_o = reinterpret_cast<float *>(ws);
    float *att_ml = att_o + (size_t)W * p.wpk * s.n_q_heads * 128;
    float *mass_part = att_ml + (size_t)W * p.wpk * s.n_q_heads * 2;
    int32_t *seq_meta = reinterpret_cast<int32_t *>(mass_part + W);
    const float scale_log2 = scale * kLog2e;
    const int G = s.n_q_heads / s.kv.n_kv_heads;
    const long long spin_ticks = tune_spin_ticks();                  // 0.25 s unless overridden

    dim3 grid(W), block(kResThreads);
    const bool fuse = select && select->sel_idx;
    if (fuse && !resident_select_fits(s)) return hipErrorInvalidValue;
    const SelectArgs sa = fuse ? *select : SelectArgs{0.0, nullptr, nullptr, nullptr, nullptr, 0};
#define FASTOCR_FUS(P, S) FASTOCR_LAUNCH(K_FOCAL_FUSED, (focal_fused_kernel<P, S>), grid, block, 0, stream, sa, s.kv, s.bv, \
                       (const uint16_t *)q, s.n_q_heads, G, scale_log2, s.batch, p.nranges, p.range_tokens, \
                       sync_slot, spin_ticks, scores, lse, img_mass ? mass_part : nullptr, att_o, att_ml, seq_meta, flag)
    if (s.paged) { if (fuse) FASTOCR_FUS(true, true); else FASTOCR_FUS(true, false); }
    else         { if (fuse) FASTOCR_FUS(false, true); else FASTOCR_FUS(false, false); }
#undef FASTOCR_FUS
    if (img_mass) fused_mass_kernel<<<s.batch, 64, 0, stream>>>(mass_part, seq_meta, img_mass);
    // every sequence's partials: workgroups seq_meta[b][0] .. + seq_meta[b][1], wpk of them each
    if (defer) {
        *defer = CombineArgs{att_o, att_ml, p.nranges * p.wpk, s.kv.head_dim, s.n_q_heads, p.wpk, seq_meta, (uint16_t *)out};
        return hipGetLastError();
    }
    return launch_attn_combine(s, att_o, att_ml, p.nranges * p.wpk, out, nullptr, stream, seq_meta, p.wpk);
}

}  // namespace fastocr
