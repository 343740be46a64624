// Focal-layer scoring with the softmax weights kept on chip (Eq. 1; text under Eq. 2).
//
// The head average is taken after each head's softmax, so a score needs every head's
// normaliser over the whole cache.  The two-kernel path parks all fp32 logits in HBM; mixing
// those writes into the K stream costs far more than their bytes on this chip.  This kernel
// keeps what it needs of them in registers instead:
//   - one 512-thread workgroup per (image-token range, sequence), at most one per compute unit,
//     so the whole grid is resident at once; a ragged batch's sequences get ranges in proportion
//     to their lengths (resident_alloc in resident.hpp);
//   - wave w streams KV head w % Hkv (8/Hkv waves share a head and interleave its tiles), a
//     32-token tile (8 KB at head_dim 128, 4 KB at 64) at a time.  Tiles travel HBM -> LDS directly
//     (global_load_lds, 16 bytes per lane, two slots per wave, no staging registers); the XOR swizzle
//     that makes the MFMA operand reads conflict-free is applied by permuting which 16-byte chunk of a
//     row each lane fetches;
//   - C[head][token] = Q * K^T with v_mfma_f32_16x16x32_bf16 leaves 4 heads x 1 token per lane; each
//     logit becomes its softmax weight 2^(logit - ref) at once, relative to a reference that the lane
//     fixed with its first live logit (as accurate as relative to the true maximum for any exponent
//     in range), and the 4 weights stay in 4 VGPRs named for the tile -- the image-tile loop is fully
//     unrolled for that (up to 32 tiles = 128 VGPRs per lane); text tokens only feed the sums;
//   - the ranges of one sequence exchange their per-head (reference, sum) through static device
//     memory: each range publishes one self-validating 64-bit word per head (agent-scope atomic
//     store; zero = not there yet) and every wave polls for the other ranges' words of its own heads
//     (bounded spin, no counter, no fence), asking for them the moment its stream ends;
//   - every wave then scales its parked weights to the sequence's normalisers, the heads of a token
//     are summed through LDS and the finished scores are written -- the only HBM writes.
// head_dim 128 or 64 (a template parameter: rows of 256 or 128 bytes, 4 or 2 k-steps per logit).
// Shapes that do not fit (group size > 8, Hkv not dividing 8, more sequences than compute
// units, more than 32 tiles per wave, pages shorter than a tile) take the two-kernel path.
#include "kernels.hpp"
#include "resident.hpp"

namespace fastocr {

constexpr int kResGatherGroup = 8;      // ranges whose statistics a wave asks for at a time
constexpr float kRefSlack = 16.f;       // how far (log2 units) a logit may rise above its lane's reference before the reference moves

#define RES_DECLARE(J) f32x4 park_##J = f32x4{0.f, 0.f, 0.f, 0.f};
// image tile J of the wave: multiply, keep the weights, refill the tile's LDS slot
#define RES_STREAM_STEP(J)                                                                          \
    {                                                                                               \
        wait_and_read(ntext + (J), kb);                                                             \
        issue_img((J) + 2, ntext + (J));                                                            \
        park_##J = weights_of(kb, img_first(J) + tok_in_tile < r1);                                  \
        if ((J) + 1 >= nimg) goto img_done;                                                         \
    }
// tile J when a lane moves its reference (see weights_of): the weights kept so far follow
#define RES_RESCALE_STEP(J)                                                                         \
    {                                                                                               \
        _Pragma("unroll") for (int r = 0; r < 4; ++r) park_##J[r] *= alpha[r];                      \
    }
// tile J after the exchange: from the lane's reference to the sequence's normalisers, this lane's 4 heads summed;
// the partner lane's 4 heads of the same token go to a row of their own (a cross-lane move per
// tile would cost more than the second row does in the final sum)
#define RES_FINISH_STEP(J)                                                                          \
    {                                                                                               \
        float v = 0.f;                                                                              \
        _Pragma("unroll") for (int r = 0; r < 4; ++r) v += park_##J[r] * cf[r];                     \
        red[(2 * kvh + (lg & 1)) * R + img_first(J) - r0 + tok_in_tile] = v;                        \
        if ((J) + 1 >= nimg) goto fin_done;                                                         \
    }

// Exchange state lives in static device memory (zero when the module is loaded) rather than in
// the caller's workspace, which would have to be cleared by an extra launch before every call.
// g_res_stats: one 64-bit word {max, sum-exp} per (workgroup, head); zero means "not published
// yet" (a published word is never zero: the sum is positive, or the maximum is the finite
// stand-in for "no logit").  g_res_left: per sequence, how many of its ranges are done reading.
// The last range to finish zeroes the sequence's words and its count, so a slot is clean again
// when its call ends.  A slot belongs to a stream (or to a stream of a graph capture): calls that
// share one are ordered by their stream, so the next call starts on a clean slot.
// g_res_timeouts counts the waves that gave up waiting (fastocr_exchange_timeouts).
__device__ unsigned long long g_res_stats[kResSlots][kResMaxWg * kResMaxHq];
__device__ uint32_t g_res_left[kResSlots][kResMaxBatch];
__device__ uint32_t g_res_timeouts;          // waves that gave up waiting, since the module was loaded
__device__ uint32_t g_res_done[kResSlots][kResMaxBatch];     // fused top-k: ranges of a sequence whose scores are out

bool resident_select_fits(const Shape &s) { return s.bv.max_vis_len <= kSelMaxKeys; }

bool resident_plan(const Shape &s, int num_cu, ResidentPlan *plan)
{
    const int Hkv = s.kv.n_kv_heads;
    if (!s.fast || (s.kv.head_dim != 128 && s.kv.head_dim != 64) || Hkv < 1 || s.n_q_heads % Hkv != 0) return false;
    const int G = s.n_q_heads / Hkv;
    if (G > 8 || s.n_q_heads > kResMaxHq) return false;
    if (Hkv != 1 && Hkv != 2 && Hkv != 4 && Hkv != 8) return false;
    if (s.batch < 1 || s.batch > num_cu || s.batch > kResMaxBatch) return false;
    if (s.paged && s.kv.page_tokens < kResTile) return false;        // a tile may touch two pages at most
    if (s.kv.stride_token > (1 << 24)) return false;                 // 32 rows of bytes must fit 32 bits
    const int wpk = kResWaves / Hkv;
    const int unit = kResTile * wpk;                       // tokens of one round of a head's waves
    int nranges = num_cu / s.batch;
    const int N = s.bv.max_vis_len;
    int R = ((N + nranges - 1) / nranges + unit - 1) / unit * unit;
    if (R < unit) R = unit;
    if (R / unit > kResTmax) return false;
    nranges = (N + R - 1) / R;
    if (nranges < 1) nranges = 1;
    plan->nranges = nranges;
    plan->range_tokens = R;
    plan->wpk = wpk;
    return true;
}

size_t resident_workspace_bytes(const Shape &s, const ResidentPlan &p)
{
    size_t bytes = (size_t)s.batch * p.nranges * sizeof(float);                        // image-mass partials
    bytes += (size_t)s.batch * 2 * sizeof(int32_t);                                    // where each sequence's partials are
    return bytes;
}

template <int D, bool PAGED, bool SELECT>
__global__ __launch_bounds__(kResThreads) void score_resident_kernel(
    SelectArgs sel_args /* first: read straight from the kernel-argument segment when the select starts */,
    KvDev kv, BatchDev bv, const uint16_t *__restrict__ q, int Hq, int G, float scale_log2,
    int batch, int nranges_uniform, int R_uniform, int sync_slot, long long spin_ticks,
    float *__restrict__ scores, float *__restrict__ lse_out, float *__restrict__ mass_part,
    int32_t *__restrict__ mass_meta, uint32_t *__restrict__ gave_up_flag)
{
    static_assert(sizeof(unsigned char[kResWaves][2][8192]) >= (size_t)kSelLdsBytes, "the select reuses the tile buffers");
    __shared__ __align__(16) unsigned char smem[kResWaves][2][8192];
    __shared__ float sm_m[kResWaves][8], sm_z[kResWaves][8];
    __shared__ float sm_red[kResWaves];
    __shared__ int sm_met, sm_last;

    // wave-uniform quantities are kept in scalar registers: tile bookkeeping, addresses and loop
    // exits then cost no vector instructions
    static_assert(D == 128 || D == 64, "head_dim 128 or 64");
    constexpr int KS = D / 32;             // k-steps of a logit
    constexpr int NL = D / 16;             // 1 KB load instructions per 32-token tile
    constexpr int RPL = 32 / NL;           // rows one load instruction brings
    constexpr int CPR = D / 8;             // 16-byte chunks of a row
    constexpr int ROWB = 2 * D;            // bytes of a row
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;                      // the lane in the matrix products
    const int lrow = lane / CPR, lslot = lane % CPR;               // the lane in a load: row of the load's group, chunk slot in LDS
    const int Hkv = kv.n_kv_heads;
    const int wpk = kResWaves / Hkv;
    const int kvh = wave % Hkv, sub = wave / Hkv;

    // which sequence and which of its ranges (all wave-uniform)
    const RangeAlloc ra = resident_alloc(bv, batch, gridDim.x, nranges_uniform, R_uniform, kResTile * wpk, blockIdx.x);
    if (!ra.active) return;
    const int rng = ra.rng, b = ra.b, nranges = ra.nr, R = ra.R, wg0 = ra.wg0;
    const int S = ra.S, v0 = ra.v0, N = ra.N;
    const int Tn = S - N;

    // image tiles of this wave: tile ti = sub + j*wpk of the range, j = 0 .. nimg-1
    const int r0 = rng * R, r1 = min(N, r0 + R);
    const int nt_range = r1 > r0 ? (r1 - r0 + kResTile - 1) / kResTile : 0;
    const int nimg = min(nt_range > sub ? (nt_range - sub + wpk - 1) / wpk : 0, kResTmax);
    // text tiles of this wave: u = slot + i*nslots
    const int ntt = (Tn + kResTile - 1) / kResTile;
    const int slot = rng * wpk + sub, nslots = nranges * wpk;
    const int ntext = ntt > slot ? (ntt - slot + nslots - 1) / nslots : 0;

    // Q as the A operand (rows 0..7 for the tile's first 16 tokens, rows 8..15 for the second 16)
    u32x4 qlo[KS], qhi[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        qlo[kk] = u32x4{0u, 0u, 0u, 0u};
        qhi[kk] = u32x4{0u, 0u, 0u, 0u};
        const int hl = li, hh = li - 8;
        if (hl < G && hl < 8)
            qlo[kk] = *reinterpret_cast<const u32x4 *>(q + ((int64_t)b * Hq + (int64_t)kvh * G + hl) * D + 8 * (4 * kk + lg));
        if (hh >= 0 && hh < G)
            qhi[kk] = *reinterpret_cast<const u32x4 *>(q + ((int64_t)b * Hq + (int64_t)kvh * G + hh) * D + 8 * (4 * kk + lg));
    }
    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(kv.k);

    // The waves of the grid advance in lock step and their streams start at addresses that differ
    // by large powers of two, so each wave walks its image tiles in a rotated order (park slot x
    // holds tile x + rot) to spread the grid over the memory channels.
    const int rot = nimg > 0 ? (wave * 5 + rng * 3 + b * 7) % nimg : 0;
    auto img_first = [&](int x) {                                                  // span-relative
        int j = x + rot;
        j = j >= nimg ? j - nimg : j;
        return r0 + (sub + j * wpk) * kResTile;
    };
    auto text_first = [&](int x) { return (slot + x * nslots) * kResTile; };       // text-relative

    // A tile goes into LDS slot (sequence number & 1) of the wave, rows of 2 D bytes one after the
    // other: load e brings rows RPL e .. RPL e + RPL - 1 (4 rows of 256 bytes, or 8 of 128), lane
    // (lrow, lslot) one 16-byte chunk of row r = RPL e + lrow, which lands at slot + 1024 e + 16 lane,
    // i.e. in chunk slot lslot of its row.  The chunk it fetches is lslot ^ f(r), so that slot x of a row
    // holds chunk x ^ f(r): f(r) = r & 15 (D 128) or (r >> 1) & 7 (D 64, two rows to 64 banks) makes the
    // MFMA operand reads conflict-free.  f(RPL e + lrow) = fl ^ 4 (e & NV-1) with fl = lrow or lrow >> 1.
    // Rows past the end of a ragged tile are clamped to its last row.  Addresses are a wave-uniform
    // 64-bit base (scalar registers) plus a 32-bit byte offset per lane.
    constexpr int NV = D == 128 ? 4 : 2;                 // distinct chunk permutations over the loads of a tile
    const int64_t seq_base = row_offset<false>(kv, b, 0, kvh);
    const uint32_t stride_b = (uint32_t)kv.stride_token * 2u;            // bytes; 32 rows fit 32 bits (host-checked)
    const uint32_t rowoff_row = (uint32_t)lrow * stride_b;
    const int fl = D == 128 ? lrow : (lrow >> 1);
    uint32_t chunk_b[NV];                                // byte offset of this lane's chunk, by e & (NV - 1)
#pragma unroll
    for (int k = 0; k < NV; ++k) chunk_b[k] = 16u * (uint32_t)((lslot ^ fl) ^ (4 * k));
    const unsigned char *kbytes = reinterpret_cast<const unsigned char *>(kv.k);

    // rows first_tok .. first_tok + rv - 1 of the sequence, contiguous token indices
    // paged caches: a tile's two block-table entries are fetched while the tile before it is
    // issued, so the latency of those scalar loads is not in front of the tile's row loads
    int ahead_tok = -1, ahead_pg = 0, ahead_a = 0, ahead_b = 0;
    auto pages_ahead = [&](int first_tok) {
        const int32_t *bt = kv.block_table + (int64_t)b * kv.max_pages;
        ahead_tok = first_tok;
        ahead_pg = (int)((uint32_t)first_tok / (uint32_t)kv.page_tokens);
        ahead_a = bt[min(ahead_pg, kv.max_pages - 1)];
        ahead_b = bt[min(ahead_pg + 1, kv.max_pages - 1)];
    };
    auto issue_run = [&](int first_tok, int rv, int seq_no) {
        unsigned char *dst = smem[wave][seq_no & 1];
        const uint32_t limit = (uint32_t)(rv - 1) * stride_b;
        if (PAGED) {
            const int pt = kv.page_tokens;
            if (ahead_tok != first_tok) pages_ahead(first_tok);
            const int pg0 = ahead_pg, in0 = first_tok - pg0 * pt;
            const int64_t pa = ahead_a, pb = ahead_b;
            // row r of the tile lives at base_a + r*stride while in0 + r < pt, else at base_b + r*stride
            const unsigned char *base_a = kbytes + 2 * (pa * kv.stride_page + (int64_t)kvh * kv.stride_head + (int64_t)in0 * kv.stride_token);
            const unsigned char *base_b = kbytes + 2 * (pb * kv.stride_page + (int64_t)kvh * kv.stride_head + (int64_t)(in0 - pt) * kv.stride_token);
            const uint32_t split = (uint32_t)(pt - in0) * stride_b;      // first byte offset of the second page
#pragma unroll
            for (int e = 0; e < NL; ++e) {
                const uint32_t ro = min(rowoff_row + (uint32_t)(RPL * e) * stride_b, limit);
                const unsigned char *base = ro >= split ? base_b : base_a;
                lds_dma16(reinterpret_cast<const uint16_t *>(base + (ro + chunk_b[e & (NV - 1)])), dst + 1024 * e);
            }
        } else {
            const unsigned char *base = kbytes + 2 * (seq_base + (int64_t)first_tok * kv.stride_token);
#pragma unroll
            for (int e = 0; e < NL; ++e) {
                const uint32_t ro = min(rowoff_row + (uint32_t)(RPL * e) * stride_b, limit);
                lds_dma16(reinterpret_cast<const uint16_t *>(base + (ro + chunk_b[e & (NV - 1)])), dst + 1024 * e);
            }
        }
    };
    // image tile x of the wave.  Past the last one the issue stays unconditional (the reader's
    // "at most NL loads outstanding" wait counts on it) but fetches a row of the query, which
    // is in cache, instead of cache rows that nobody will use.
    const uint16_t *qrow = q + ((int64_t)b * Hq + (int64_t)kvh * G) * D;
    auto issue_img = [&](int x, int seq_no) {
        if (x >= nimg) {
            unsigned char *dst = smem[wave][seq_no & 1];
#pragma unroll
            for (int e = 0; e < NL; ++e) lds_dma16(qrow + chunk_b[e & (NV - 1)] / 2, dst + 1024 * e);
            return;
        }
        const int jf = img_first(x);
        issue_run(v0 + jf, min(kResTile, r1 - jf), seq_no);
        if (PAGED && x + 1 < nimg) pages_ahead(v0 + img_first(x + 1));
    };
    // text tile x of the wave: text positions map to tokens with a gap at the image span, so the
    // rows are addressed one by one
    auto issue_text = [&](int x, int seq_no) {
        const int tf = text_first(min(x, ntext - 1));
        unsigned char *dst = smem[wave][seq_no & 1];
#pragma unroll
        for (int e = 0; e < NL; ++e) {
            const int tc = min(tf + RPL * e + lrow, Tn - 1);
            const int tok = tc < v0 ? tc : tc + N;
            lds_dma16(kbase + row_offset<PAGED>(kv, b, tok, kvh) + chunk_b[e & (NV - 1)] / 2, dst + 1024 * e);
        }
    };

    const int hbase = 4 * (lg & 1);
    const int tok_in_tile = li + 16 * (lg >> 1);
    // Softmax weights are kept relative to a reference per lane and head that is fixed by the lane's
    // first live logit, so neither a running maximum nor a second pass of exponentials is needed, and
    // what is parked in the registers is the weight itself.  The exponent logit - ref is rounded to
    // fp32, half an ulp of its own size: relative to the true maximum the weights that matter have
    // exponents near 0, relative to a far reference they do not, and the weight's relative error is
    // that rounding times ln 2.  So a logit more than kRefSlack above the reference moves the reference
    // there and rescales what the lane holds: exponents stay below 16 (error <= 3.3e-7 of the weight,
    // what the two-kernel path reaches; with a slack of 64 a score of 0.3 was off by 1.3e-6), and a
    // lane moves once per 11 nats its logits rise above its first one -- rarely.
    float ref[4], z[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { ref[r] = kMinusHuge; z[r] = 0.f; }
    RES_EACH_TILE(RES_DECLARE)

    // LDS byte addresses of this lane's B-operand chunks, one per k-step (row li of slot 0; row 16 + li
    // has the same f and lies 16 rows further on)
    uint32_t rd_addr[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
        rd_addr[kk] = lds_address(&smem[wave][0][0]) + li * ROWB + ((((4 * kk + lg) ^ (D == 128 ? li : (li >> 1))) & (CPR - 1)) << 4);

    // Tile number seq_no of the wave has landed once at most the NL loads of the next tile are
    // outstanding; read it in the MFMA B layout.  The reads are written in assembly together with
    // their waits: the compiler does not order LDS reads after loads that land in LDS by
    // themselves (left to itself it waits for ALL outstanding loads, the prefetch included), and
    // it must not move the products above the wait either.
    auto wait_and_read = [&](int seq_no, u32x4(&kb)[2 * KS]) {
        const uint32_t so = (seq_no & 1) * 8192;
        if constexpr (D == 64) {
            asm volatile(
                "s_waitcnt vmcnt(4)\n\t"
                "ds_read_b128 %0, %4\n\t"
                "ds_read_b128 %1, %5\n\t"
                "ds_read_b128 %2, %4 offset:2048\n\t"
                "ds_read_b128 %3, %5 offset:2048\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&v"(kb[0]), "=&v"(kb[1]), "=&v"(kb[2]), "=&v"(kb[3])
                : "v"(rd_addr[0] + so), "v"(rd_addr[1] + so)
                : "memory");
        } else
        asm volatile(
            "s_waitcnt vmcnt(8)\n\t"
            "ds_read_b128 %0, %8\n\t"
            "ds_read_b128 %1, %9\n\t"
            "ds_read_b128 %2, %10\n\t"
            "ds_read_b128 %3, %11\n\t"
            "ds_read_b128 %4, %8 offset:4096\n\t"
            "ds_read_b128 %5, %9 offset:4096\n\t"
            "ds_read_b128 %6, %10 offset:4096\n\t"
            "ds_read_b128 %7, %11 offset:4096\n\t"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(kb[0]), "=&v"(kb[1]), "=&v"(kb[2]), "=&v"(kb[3]), "=&v"(kb[4]), "=&v"(kb[5]), "=&v"(kb[6]), "=&v"(kb[7])
            : "v"(rd_addr[0] + so), "v"(rd_addr[1] + so), "v"(rd_addr[2] + so), "v"(rd_addr[3] + so)
            : "memory");
    };
    // weights 2^(logit - ref) of this lane's token for its 4 heads (logits in the log2 domain); dead
    // positions come out 0
    auto weights_of = [&](u32x4(&kb)[2 * KS], bool live) -> f32x4 {
        f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qlo[kk]),
                                                        __builtin_bit_cast(bf16x8, kb[kk]), s, 0, 0, 0);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qhi[kk]),
                                                        __builtin_bit_cast(bf16x8, kb[KS + kk]), s, 0, 0, 0);
        bool moved = false;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s[r] = live ? s[r] * scale_log2 : -INFINITY;
            if (ref[r] == kMinusHuge) ref[r] = fmaxf(s[r], kMinusHuge);          // the first live logit
            moved = moved || s[r] - ref[r] > kRefSlack;
        }
        if (__builtin_amdgcn_ballot_w64(moved) != 0ull) {
            float alpha[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool mv = s[r] - ref[r] > kRefSlack;
                alpha[r] = mv ? fast_exp2(ref[r] - s[r]) : 1.f;
                ref[r] = mv ? s[r] : ref[r];
                z[r] *= alpha[r];
            }
            RES_EACH_TILE(RES_RESCALE_STEP)
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s[r] = fast_exp2(s[r] - ref[r]);
            z[r] += s[r];
        }
        return s;
    };

    // ---- stream: text tiles (statistics only), then image tiles (weights parked in registers) ----
    // The wave's tiles are numbered 0 .. ntext + nimg - 1 in that order; tile n uses slot n & 1 and
    // two tiles are always in flight.
    u32x4 kb[2 * KS];
    if (ntext + nimg > 0) {
        // the first two tiles
        if (ntext > 0) issue_text(0, 0); else issue_img(0, 0);
        if (ntext > 1) issue_text(1, 1); else if (nimg > 0) issue_img(1 - ntext, 1); else issue_text(1, 1);
        for (int x = 0; x < ntext; ++x) {
            wait_and_read(x, kb);
            if (x + 2 < ntext || nimg == 0) issue_text(x + 2, x); else issue_img(x + 2 - ntext, x);
            (void)weights_of(kb, text_first(x) + tok_in_tile < Tn);
        }
    }
    if (nimg > 0) {
        RES_EACH_TILE(RES_STREAM_STEP)
    }
img_done:
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the trailing refills must not land later

    // The other ranges' statistics of this wave's heads are asked for at once: with the chip's memory
    // queues full of other workgroups' streams a load takes microseconds to come back, and for the
    // ranges that finish late everybody else's words are there already -- the answer then arrives
    // while this range reduces and publishes its own.
    unsigned long long *stats = g_res_stats[sync_slot] + (int64_t)wg0 * Hq;
    const StatRows<kResGatherGroup> early = resident_heads_request<kResGatherGroup>(stats, rng, nranges, Hq, G, kvh);

    // ---- range statistics: lanes -> waves -> workgroup -> workspace ------------------------------
    // over the 16 lanes of a row (the tile's tokens li) with DPP moves -- pairs, quads, the mirrored half,
    // the mirrored row -- then over the two rows that hold the same heads (lanes 32 apart) with a half
    // swap: first the largest reference, then the sums brought to it
    float m[4];           // the wave's common reference per head
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float M = ref[r];
        M = fmaxf(M, dpp_move<kDppXor1>(M));
        M = fmaxf(M, dpp_move<kDppXor2>(M));
        M = fmaxf(M, dpp_move<kDppHalfMirror>(M));
        M = fmaxf(M, dpp_move<kDppRowMirror>(M));
        M = with_lane_xor32(M, [](float a, float b) { return fmaxf(a, b); });
        float Z = z[r] * fast_exp2(ref[r] - M);
        Z += dpp_move<kDppXor1>(Z);
        Z += dpp_move<kDppXor2>(Z);
        Z += dpp_move<kDppHalfMirror>(Z);
        Z += dpp_move<kDppRowMirror>(Z);
        Z = with_lane_xor32(Z, [](float a, float b) { return a + b; });
        m[r] = M;
        z[r] = Z;
    }
    if (li == 0 && lg < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { sm_m[wave][hbase + r] = m[r]; sm_z[wave][hbase + r] = z[r]; }
    }
    if (threadIdx.x == 0) sm_met = 1;
    __syncthreads();
    // publish this range's statistics (resident.hpp: every word is its own "ready" flag)
    resident_publish(stats + (int64_t)rng * Hq, sm_m, sm_z, Hq, G, Hkv, wpk);

    // ---- the log-sum-exp of this wave's heads over the whole sequence (lane 8s + x: head x of the group) ----
    float l2;
    {
        float M, Z;
        const bool ok = resident_heads_gather<kResGatherGroup>(stats, rng, nranges, Hq, G, Hkv, wpk, kvh, sm_m, sm_z, spin_ticks,
                                                               M, Z, &early);
        if (!ok && lane == 0) {
            sm_met = 0;
            __hip_atomic_fetch_add(&g_res_timeouts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (gave_up_flag) __hip_atomic_store(gave_up_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        l2 = Z > 0.f ? M + log2f(Z) : -INFINITY;
    }
    __syncthreads();      // whether every wave has met its ranges; the tile buffers are free for the head sums
    // This range is done reading: count it out.  The last one of the sequence (it has seen every
    // other one finish reading) clears the sequence's words and the count when the kernel ends.
    uint32_t *left = &g_res_left[sync_slot][b];
    // (the count's old value is only looked at when the kernel ends: nobody waits for the atomic)
    uint32_t left_before = 0u;
    if (threadIdx.x == 0) left_before = __hip_atomic_fetch_add(left, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    auto leave = [&]() {
        if (threadIdx.x == 0) sm_last = left_before == (uint32_t)nranges - 1u;
        __syncthreads();
        resident_retire(sm_last != 0, stats, nranges, Hq, left);
    };
    if (!sm_met) {
        // a range of the sequence never published (the grid was not resident as a whole): poison
        // this range's scores rather than publish numbers built on missing statistics
        for (int i = threadIdx.x; i < r1 - r0; i += kResThreads)
            store_score<SELECT>(&scores[(int64_t)b * bv.max_vis_len + r0 + i], __builtin_nanf(""));
        if (SELECT) resident_select_tail(scores, b, nranges, &g_res_done[sync_slot][b], &smem[0][0][0]);
        leave();
        return;
    }
    if (lse_out && rng == 0 && sub == 0 && lane < G) lse_out[(int64_t)b * Hq + kvh * G + lane] = l2 * kLn2;

    // ---- the parked weights brought to the normalisers, summed over the heads of each token ------
    float cf[4];          // from "relative to the lane's reference" to "relative to the head's normaliser"
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float la = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, l2), r));
        const float lb = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, l2), 4 + r));
        cf[r] = (hbase + r < G) ? fast_exp2(ref[r] - (hbase ? lb : la)) : 0.f;
    }
    float *red = reinterpret_cast<float *>(&smem[0][0][0]);          // [2 Hkv][R], at most 64 KB
    if (nimg > 0) {
        RES_EACH_TILE(RES_FINISH_STEP)
    }
fin_done:
    __syncthreads();
    float local = 0.f;
    const float inv = 1.0f / (float)Hq;
    for (int i = threadIdx.x; i < r1 - r0; i += kResThreads) {
        float a = 0.f;
        for (int g = 0; g < 2 * Hkv; ++g) a += red[g * R + i];
        a *= inv;
        store_score<SELECT>(&scores[(int64_t)b * bv.max_vis_len + r0 + i], a);
        local += a;
    }
    if (mass_part) {
        local = wave_sum(local);
        if (lane == 0) sm_red[wave] = local;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            for (int w = 0; w < kResWaves; ++w) t += sm_red[w];
            mass_part[wg0 + rng] = t;
            if (rng == 0) { mass_meta[2 * b] = wg0; mass_meta[2 * b + 1] = nranges; }
        }
    }
    if (SELECT) resident_select_tail(scores, b, nranges, &g_res_done[sync_slot][b], &smem[0][0][0]);
    leave();
}

// image mass of a sequence = the sum of its ranges' partial sums (their place comes from the kernel)
__global__ void resident_mass_kernel(const float *__restrict__ mass_part, const int32_t *__restrict__ mass_meta,
                                     float *__restrict__ img_mass)
{
    const int b = blockIdx.x;
    const int first = mass_meta[2 * b], n = mass_meta[2 * b + 1];
    float t = 0.f;
    for (int x = threadIdx.x; x < n; x += 64) t += mass_part[first + x];
    t = wave_sum(t);
    if (threadIdx.x == 0) img_mass[b] = t;
}

hipError_t score_resident_timeouts(uint32_t *n) { return hipMemcpyFromSymbol(n, HIP_SYMBOL(g_res_timeouts), sizeof(uint32_t)); }

hipError_t launch_score_resident(const Shape &s, const ResidentPlan &p, int sync_slot, uint32_t *flag, const void *q, float scale,
                                 float *scores, float *lse, float *img_mass, void *ws, hipStream_t stream,
                                 const SelectArgs *select)
{
    if (sync_slot < 0 || sync_slot >= kResSlots) return hipErrorInvalidValue;
    const int W = p.nranges * s.batch;                       // workgroups = range statistics slots
    float *mass_part = reinterpret_cast<float *>(ws);
    int32_t *mass_meta = reinterpret_cast<int32_t *>(mass_part + W);
    const float scale_log2 = scale * kLog2e;
    const int G = s.n_q_heads / s.kv.n_kv_heads;
    // a range waits at most this long for its sequence's other ranges (they run concurrently and
    // finish within microseconds of each other); past it the call's scores are NaN but it ends
    const long long spin_ticks = tune_spin_ticks();                  // 0.25 s unless overridden

    dim3 grid(W), block(kResThreads);
    const bool fuse = select && select->sel_idx;
    if (fuse && !resident_select_fits(s)) return hipErrorInvalidValue;
    const SelectArgs sa = fuse ? *select : SelectArgs{0.0, nullptr, nullptr, nullptr, nullptr, 0};
#define FASTOCR_RES(D, P, S) FASTOCR_LAUNCH(K_SCORE_LOGITS, (score_resident_kernel<D, P, S>), grid, block, 0, stream, sa, s.kv, s.bv, \
                       (const uint16_t *)q, s.n_q_heads, G, scale_log2, s.batch, p.nranges, p.range_tokens, \
                       sync_slot, spin_ticks, scores, lse, img_mass ? mass_part : nullptr, mass_meta, flag)
#define FASTOCR_RES_D(D) \
    if (s.paged) { if (fuse) FASTOCR_RES(D, true, true); else FASTOCR_RES(D, true, false); } \
    else         { if (fuse) FASTOCR_RES(D, false, true); else FASTOCR_RES(D, false, false); }
    if (s.kv.head_dim == 64) { FASTOCR_RES_D(64) } else { FASTOCR_RES_D(128) }
#undef FASTOCR_RES_D
#undef FASTOCR_RES
    if (img_mass) resident_mass_kernel<<<s.batch, 64, 0, stream>>>(mass_part, mass_meta, img_mass);
    return hipGetLastError();
}

}  // namespace fastocr
