// Decode attention over an explicit token list: split-K flash-decode for gfx950.
//
// One launch covers both branches of Eq. 2: the focal branch attends all cached tokens
// (dense), the non-focal branch attends the kept set T u F (gather: text before the image
// span, the selected image tokens, text after the span).  The attended list is cut into
// `nsplit` position ranges; a workgroup owns one (sequence, kv head, range), its four or
// eight waves walk 32-token tiles with a private online softmax each and merge through LDS.
// What leaves the workgroup depends on the mode (see kPartial / kDirect / kMerge below): an fp32
// partial (m, Z, acc[d]) that a second small kernel merges, the final output when the stream has
// one range, or -- pruned attention with a few ranges per stream -- a partial handed to the
// stream's last workgroup inside the same launch.
//
// bf16, head_dim 128 path: the G = Hq/Hkv query heads that share a kv head form the 16-wide
// side of v_mfma_f32_16x16x32_bf16 (rows beyond G are zero), tokens the other side.
//   QK^T : A = K tile (16 tokens x 32 dims), B = Q^T  -> C[token][head]
//   PV   : A = V^T (16 dims x 32 tokens),   B = P^T  -> C[dim][head]
// The C layout of the first product (lane = head, 4 tokens per lane group) is exactly the
// B layout the second one needs, so probabilities never cross lanes.  V rows are loaded
// coalesced (16 lanes x 16 B = one 256 B row) and transposed in registers with v_perm_b32.
// K is loaded the same coalesced way and re-laid to the A layout through a wave-private,
// XOR-swizzled LDS tile.
#include "kernels.hpp"
#include "combine.hpp"

namespace fastocr {

// How a workgroup's result leaves the kernel.
//   kPartial: an fp32 partial (m, Z, acc[d]) in the workspace; a merge kernel follows.
//   kDirect : the stream has a single range: the normalised output itself.
//   kMerge  : several ranges per stream, merged inside the launch.  Ranges 0 .. nsplit-2 publish
//             their partial as 64-bit words {value, tag} in static device memory with agent-scope
//             atomic stores; the stream's last range (dispatched after them) polls until every word
//             it needs carries this call's tag, merges and writes the output.  Every word is its
//             own "ready" flag, so nothing has to be ordered and no fence (an L2 write-back on this
//             chip) is needed.  The tag is the call's number on its (slot, stream number): every
//             workgroup of the call draws a ticket from a device-side counter by adding
//             kTicketUnit / nsplit to it, so one call adds kTicketUnit whatever its range count and
//             ticket / kTicketUnit is the same for all its workgroups, however late one of them
//             starts.  Calls that share a slot are enqueued on one stream (api.hip hands slots to
//             streams), so a call's last workgroup has drawn its ticket before the next call's first
//             one does: two calls never see the same number, a replayed HIP graph gets fresh tags
//             too, and a workgroup that publishes after its call's last range has given up waiting
//             still publishes under its own call's tag, which no later call accepts.  A word's place
//             depends on (stream number, range, element) only -- never on the call's shape -- so
//             whatever a word still holds was written under an older number of the same counter.
enum { kPartial = 0, kDirect = 1, kMerge = 2 };
constexpr int kMergeMaxSplits = 4;
constexpr unsigned long long kTicketUnit = 12;                  // divisible by every range count 2 .. kMergeMaxSplits
constexpr int kMergeMaxStreams = 128;
constexpr int kMergeMaxG = 8;
constexpr int kMergeStatsAt = kMergeMaxG * 128;                 // a partial: o[G][D] (D <= 128), then at a fixed place m[G], then Z[G]
constexpr int kMergePitch = kMergeMaxG * 130;                   // words per published partial, whatever G is
constexpr size_t kMergeWords = (size_t)kMergeMaxStreams * (kMergeMaxSplits - 1) * kMergePitch;   // per slot: 3.2 MB
__device__ unsigned long long g_merge_words[kMergeSlots][kMergeWords];
__device__ unsigned long long g_merge_ticket[kMergeSlots][kMergeMaxStreams];
__device__ uint32_t g_merge_timeouts;                        // sticky count of merges that gave up

// Where dim `dim` of head `head` sits in a wave's [16 heads][D] join buffer.  A head's row is a
// multiple of 64 LDS banks long, so with the plain order the 64 lanes of a store -- 16 heads x 4 lane
// groups whose dims differ by 32 -- would meet in two banks (a 32-way conflict on each of the 32
// stores per wave).  With the dim XORed by the head number and its bit 6 folded into bit 4 the 64
// lanes of a store fall into 64 different banks, and so do the 64 consecutive dims a wave reads.
template <int D>
__device__ __forceinline__ int join_slot(int head, int dim)
{
    if constexpr (D == 128) return dim ^ (head & 15) ^ ((dim & 64) >> 2);
    else return dim;
}

__device__ __forceinline__ unsigned long long tagged(float x, uint32_t tag)
{
    return (unsigned long long)__float_as_uint(x) | ((unsigned long long)tag << 32);
}


constexpr int kTile = 32;          // tokens per wave tile (two 16-token MFMA tiles)

// Row of the 32-token tile that lane group `lg` holds as element e of its 8-token k-block:
// elements 0..3 come from the first 16-token half, 4..7 from the second.
__device__ __forceinline__ int tile_row(int lg, int e) { return (e < 4) ? (4 * lg + e) : (16 + 4 * lg + (e - 4)); }

// -----------------------------------------------------------------------------------------
// MFMA kernel: bf16, head_dim D = 128 or 64, G <= 16.
// D = 64: rows are 128 bytes (8 chunks of 16), a 1 KB load instruction brings 8 rows, the logits take
// two k-steps and the output four 16-dim blocks.  K goes through the LDS tile as for D = 128 (pitch
// 128 bytes, chunk ^ ((row >> 1) & 7)).  V: P*V's A operand wants, in lane (li, lg), the 8 tokens of
// k-block lg for ONE dim -- rows i and i + 8 of the operand share a 16-byte chunk (chunk i & 7) and
// take its even / odd elements: row i is dim 8 (i & 7) + 2 t + (i >> 3) of block t.  Lanes li < 8
// load the k-block's first four tokens, lanes li >= 8 its last four, and the halves swap through
// a data-parallel-primitive move (lane ^ 8), so every V byte is still fetched once.
// -----------------------------------------------------------------------------------------
// kWaves waves per workgroup walk the range.  Dense: the workgroup's tiles are dealt to its waves
// in turn.  Gather: the attended list is cut into nsplit * kWaves contiguous pieces, one per wave,
// of equal length to within one token (or one tile, for short lists: see below) -- with a
// handful of tiles per wave, whole tiles would leave some waves a quarter more bytes than others.
template <int D, bool GATHER, bool PAGED, int kWaves, int MODE>
__global__ __launch_bounds__(64 * kWaves, 8 / kWaves) void attn_mfma_kernel(
    KvDev kv, BatchDev bv, const uint16_t *__restrict__ q, int Hq, int G, float scale_log2,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt, int64_t kmax,
    float *__restrict__ part_o, float *__restrict__ part_ml, int nsplit, uint16_t *__restrict__ out,
    float *__restrict__ lse, int merge_slot, long long spin_ticks, uint32_t *__restrict__ gave_up_flag)
{
    __shared__ __align__(16) unsigned char smem[kWaves][8192];
    __shared__ float sm_m[kWaves][16], sm_z[kWaves][16];
    __shared__ uint32_t sm_tag;

    static_assert(D == 128 || D == 64, "head_dim 128 or 64");
    constexpr int KS = D / 32;            // k-steps of the logits
    constexpr int NACC = D / 16;          // 16-dim blocks of the output
    constexpr int NL = D / 16;            // 1 KB load instructions per 32-token K (or V) tile
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;

    const int stream_id = b * gridDim.y + kvh;
    // this workgroup's ticket (see kMerge above), requested before anything else; the tag is only
    // needed after the tile loop and is put into LDS once the geometry (requested after it) is there
    unsigned long long ticket = 0;
    if (MODE == kMerge && threadIdx.x == 0)
        ticket = __hip_atomic_fetch_add(&g_merge_ticket[merge_slot][stream_id], kTicketUnit / (unsigned long long)nsplit,
                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    const SeqGeom geo = seq_geom(bv, b);
    int cnt = 0;
    const int32_t *sel = nullptr;
    if (GATHER) {
        cnt = min(max(sel_cnt[b], 0), (int)min((int64_t)geo.N, kmax));
        sel = sel_idx + (int64_t)b * kmax;
    }
    const int L = GATHER ? (geo.S - geo.N + cnt) : geo.S;
    if (MODE == kMerge && threadIdx.x == 0) {
        const uint32_t t = (uint32_t)(ticket / kTicketUnit) + 1u;
        sm_tag = t ? t : 1u;                  // zero is what never-written words hold
    }
    // this wave's tiles: tile i starts at position tile_pos(i) and ends before pend
    int wp0 = 0, pend = L, nt, tfirst = 0;
    if (GATHER) {
        // piece gw of nw: x units each, the first `rem` pieces one more.  A unit is a token when
        // that leaves a wave three tiles or more (the stream is then bound by memory and equal byte
        // counts matter), else a whole tile: a partial tile costs the load path as many
        // instructions as a full one, which is what bounds a short list.
        const int gw = split * kWaves + wave, nw = nsplit * kWaves;
        const int ntile = (L + kTile - 1) / kTile;
        const bool by_token = ntile >= 3 * nw;
        const int units = by_token ? L : ntile;
        const int x = units / nw, rem = units - x * nw;
        const int u0 = gw * x + min(gw, rem), u1 = u0 + x + (gw < rem ? 1 : 0);
        wp0 = by_token ? u0 : u0 * kTile;
        pend = by_token ? u1 : min(L, u1 * kTile);
        nt = (pend - wp0 + kTile - 1) / kTile;
    } else {
        const int ntile = (L + kTile - 1) / kTile;
        const int tps = (ntile + nsplit - 1) / nsplit;
        const int t1 = min(ntile, split * tps + tps);
        tfirst = split * tps + wave;
        nt = tfirst < t1 ? (t1 - 1 - tfirst) / kWaves + 1 : 0;
    }
    auto tile_pos = [&](int i) { return GATHER ? wp0 + i * kTile : (tfirst + i * kWaves) * kTile; };

    // Q as the B operand: lane (head li, k-block lg) holds dims 8*(4kk+lg) .. +7 for step kk.
    u32x4 qreg[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        qreg[kk] = u32x4{0u, 0u, 0u, 0u};
        if (li < G) {
            const uint16_t *qp = q + ((int64_t)b * Hq + (int64_t)kvh * G + li) * D + 8 * (4 * kk + lg);
            qreg[kk] = *reinterpret_cast<const u32x4 *>(qp);
        }
    }

    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(kv.k);
    const uint16_t *vbase = reinterpret_cast<const uint16_t *>(kv.v);

    // element offset of the row this lane looks up for the wave's tile i (row lane % 32; rows past
    // the end repeat the last one)
    auto rowoff_of = [&](int i) -> int64_t {
        int p = min(tile_pos(i) + (lane & 31), pend - 1);
        int tok = pos_to_token<GATHER>(p, geo, cnt, sel);
        return row_offset<PAGED>(kv, b, tok, kvh);
    };
    const int64_t seq_base = row_offset<false>(kv, b, 0, kvh);

    // D = 64: which of the k-block's halves this lane loads of V, and its chunk of a row
    const int vh = li >> 3, lc = lane & 7;
    auto load_tile = [&](int i, int64_t off, u32x4(&K)[NL], u32x4(&V)[NL]) {
#pragma unroll
        for (int e = 0; e < NL; ++e) {
            if constexpr (D == 128) {
                const int r = tile_row(lg, e);
                int64_t ro;
                if (GATHER || PAGED) ro = __shfl(off, r);
                else ro = seq_base + (int64_t)min(tile_pos(i) + r, L - 1) * kv.stride_token;
                V[e] = stream_load(vbase + ro + 8 * li);
                K[e] = stream_load(kbase + ro + 8 * li);
            } else {
                // V: row 16 vh + 4 lg + e (the k-block's tokens); K: rows 8e .. 8e+7, one per 8 lanes
                const int rv = 16 * vh + 4 * lg + e, rk = 8 * e + (lane >> 3);
                int64_t rov, rok;
                if (GATHER || PAGED) { rov = __shfl(off, rv); rok = __shfl(off, rk); }
                else {
                    rov = seq_base + (int64_t)min(tile_pos(i) + rv, L - 1) * kv.stride_token;
                    rok = seq_base + (int64_t)min(tile_pos(i) + rk, L - 1) * kv.stride_token;
                }
                V[e] = stream_load(vbase + rov + 8 * lc);
                K[e] = stream_load(kbase + rok + 8 * lc);
            }
        }
    };

    float m = -INFINITY, zl = 0.f;
    f32x4 acc[NACC];
#pragma unroll
    for (int t = 0; t < NACC; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int i, u32x4(&K)[NL], u32x4(&V)[NL]) {
        u32x4 ka[2 * KS];
        {
            unsigned char *sw = smem[wave];
#pragma unroll
            for (int e = 0; e < NL; ++e) {
                if constexpr (D == 128) {
                    const int r = tile_row(lg, e);
                    *reinterpret_cast<u32x4 *>(sw + r * 256 + ((li ^ (r & 15)) << 4)) = K[e];
                } else {
                    const int r = 8 * e + (lane >> 3);
                    *reinterpret_cast<u32x4 *>(sw + r * 128 + ((lc ^ ((r >> 1) & 7)) << 4)) = K[e];
                }
            }
            wave_lds_fence();
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int kk = 0; kk < KS; ++kk) {
                    const int c = 4 * kk + lg, r = 16 * T + li;
                    if constexpr (D == 128) ka[KS * T + kk] = *reinterpret_cast<const u32x4 *>(sw + r * 256 + (((c ^ li) & 15) << 4));
                    else ka[KS * T + kk] = *reinterpret_cast<const u32x4 *>(sw + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
                }
            wave_lds_fence();
        }
        f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kk]),
                                                         __builtin_bit_cast(bf16x8, qreg[kk]), s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[KS + kk]),
                                                         __builtin_bit_cast(bf16x8, qreg[kk]), s1, 0, 0, 0);
        }
        // lane (head li, group lg): s0[r] is token 4lg+r of the tile, s1[r] token 16+4lg+r
        float s[8];
        const int pbase = tile_pos(i) + 4 * lg;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s[r] = (pbase + r < pend) ? s0[r] * scale_log2 : -INFINITY;
            s[4 + r] = (pbase + 16 + r < pend) ? s1[r] * scale_log2 : -INFINITY;
        }
        float mx = s[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, s[e]);
        mx = rows_max(mx);
        const float m_new = fmaxf(m, mx);          // finite: every tile holds a valid position
        const float alpha = fast_exp2(m - m_new);
        float p[8], ps = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { p[e] = fast_exp2(s[e] - m_new); ps += p[e]; }
        zl = zl * alpha + ps;
        m = m_new;
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)p[e];
        if constexpr (D == 128) {
#pragma unroll
            for (int t = 0; t < NACC; ++t) {
                acc[t] *= alpha;
                const int w = t >> 1;
                const uint32_t selb = (t & 1) ? 0x07060302u : 0x05040100u;
                u32x4 a;
#pragma unroll
                for (int pp = 0; pp < 4; ++pp) a[pp] = __builtin_amdgcn_perm(V[2 * pp + 1][w], V[2 * pp][w], selb);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), pb, acc[t], 0, 0, 0);
            }
        } else {
            // fa[e]: this lane's chunk of token 4lg + e, sb[e]: of token 16 + 4lg + e -- one half loaded by
            // this lane, the other by lane ^ 8
            u32x4 fa[4], sb[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t own = V[e][w];
                    const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0x128, 0xf, 0xf, false);   // row_ror:8 = lane ^ 8
                    fa[e][w] = vh ? other : own;
                    sb[e][w] = vh ? own : other;
                }
            const uint32_t selb = vh ? 0x07060302u : 0x05040100u;      // rows 8 .. 15 of the operand take the odd elements
#pragma unroll
            for (int t = 0; t < NACC; ++t) {
                acc[t] *= alpha;
                u32x4 a;
                a[0] = __builtin_amdgcn_perm(fa[1][t], fa[0][t], selb);
                a[1] = __builtin_amdgcn_perm(fa[3][t], fa[2][t], selb);
                a[2] = __builtin_amdgcn_perm(sb[1][t], sb[0][t], selb);
                a[3] = __builtin_amdgcn_perm(sb[3][t], sb[2][t], selb);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), pb, acc[t], 0, 0, 0);
            }
        }
    };

    if (nt > 0) {
        // Two register buffers, software pipelined.  The prefetch is unconditional: a branch between
        // a load and the wait that matches it would make the compiler drain every outstanding load
        // at the join (and a copy of the step without the prefetch for the last tile costs more
        // registers than the kernel has).  Past the wave's last tile it fetches a single row (all
        // lanes the same address) instead of a tile.
        u32x4 KA[NL], VA[NL], KB[NL], VB[NL];
        int i = 0;
        const int last = nt - 1;
        if (!(GATHER || PAGED)) {
            load_tile(0, 0, KA, VA);
            while (true) {
                load_tile(min(i + 1, last), 0, KB, VB);
                compute(i, KA, VA);
                if (++i > last) break;
                load_tile(min(i + 1, last), 0, KA, VA);
                compute(i, KB, VB);
                if (++i > last) break;
            }
        } else {
            // Row offsets come from memory (selected indices, block table).  They are fetched a
            // whole group of tiles ahead and BEFORE that group's K/V loads are issued: loads return
            // in order, so waiting for an offset never waits for a tile issued after it.
            constexpr int kGroup = 4;
            int64_t offc[kGroup], offn[kGroup];
#pragma unroll
            for (int j = 0; j < kGroup; ++j) offc[j] = rowoff_of(min(j, last));
            load_tile(0, offc[0], KA, VA);
            while (true) {
#pragma unroll
                for (int j = 0; j < kGroup; ++j) offn[j] = rowoff_of(min(i + kGroup + j, last));
#pragma unroll
                for (int j = 0; j < kGroup; ++j) {
                    int64_t onext = (j + 1 < kGroup) ? offc[j + 1] : offn[0];
                    onext = (i + 1 <= last) ? onext : __shfl(onext, 0);
                    if ((j & 1) == 0) { load_tile(0, onext, KB, VB); compute(i, KA, VA); }
                    else              { load_tile(0, onext, KA, VA); compute(i, KB, VB); }
                    if (++i > last) goto tiles_done;
                }
#pragma unroll
                for (int j = 0; j < kGroup; ++j) offc[j] = offn[j];
            }
        }
    }
tiles_done:

    // ---- cross-wave merge through LDS -----------------------------------------------------
    zl = rows_sum(zl);
    float *buf = reinterpret_cast<float *>(smem[wave]);        // [16 heads][D dims], dims permuted per head (join_slot)
#pragma unroll
    for (int t = 0; t < NACC; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            // the operand row 4lg + r of block t: dim 8 row + t (D = 128), dim 8 (row & 7) + 2 t + (row >> 3) (D = 64)
            const int row = 4 * lg + r;
            const int dim = D == 128 ? 8 * row + t : 8 * (row & 7) + 2 * t + (row >> 3);
            buf[li * D + join_slot<D>(li, dim)] = acc[t][r];
        }
    if (lg == 0) { sm_m[wave][li] = m; sm_z[wave][li] = zl; }
    __syncthreads();
    const uint32_t tag = MODE == kMerge ? sm_tag : 0u;

    const int np = nsplit - 1;                                       // ranges that publish (kMerge)
    // the stream's published partials: kMergeMaxSplits - 1 fixed places of kMergePitch words
    unsigned long long *words = MODE == kMerge ? g_merge_words[merge_slot] + (int64_t)stream_id * (kMergeMaxSplits - 1) * kMergePitch : nullptr;
    for (int idx = threadIdx.x; idx < G * D; idx += 64 * kWaves) {
        const int hh = idx / D, c = idx % D;
        float M = sm_m[0][hh];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][hh]);
        float o = 0.f, Z = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float f = fast_exp2(sm_m[w][hh] - M);
                o += f * reinterpret_cast<const float *>(smem[w])[hh * D + join_slot<D>(hh, c)];
                Z += f * sm_z[w][hh];
            }
        }
        const int64_t bh = (int64_t)b * Hq + (int64_t)kvh * G + hh;
        if (MODE == kMerge && split < np) {
            unsigned long long *w = words + (int64_t)split * kMergePitch;
            __hip_atomic_store(w + idx, tagged(o, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (c == 0) {
                __hip_atomic_store(w + kMergeStatsAt + hh, tagged(M, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(w + kMergeStatsAt + kMergeMaxG + hh, tagged(Z, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else if (MODE == kMerge) {
            // the stream's last range: every other range's (o, m, Z) for this element, all requested
            // at once, again until each word carries this call's tag
            unsigned long long wo[kMergeMaxSplits - 1], wm[kMergeMaxSplits - 1], wz[kMergeMaxSplits - 1];
            const long long t_start = wall_clock64();
            bool ok = true;
            while (true) {
#pragma unroll
                for (int x = 0; x < kMergeMaxSplits - 1; ++x) {
                    if (x < np) {
                        const unsigned long long *w = words + (int64_t)x * kMergePitch;
                        wo[x] = __hip_atomic_load(w + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        wm[x] = __hip_atomic_load(w + kMergeStatsAt + hh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        wz[x] = __hip_atomic_load(w + kMergeStatsAt + kMergeMaxG + hh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                bool all = true;
#pragma unroll
                for (int x = 0; x < kMergeMaxSplits - 1; ++x)
                    if (x < np)
                        all = all && (uint32_t)(wo[x] >> 32) == tag && (uint32_t)(wm[x] >> 32) == tag && (uint32_t)(wz[x] >> 32) == tag;
                if (all) break;
                __builtin_amdgcn_s_sleep(1);
                if (wall_clock64() - t_start > spin_ticks) { ok = false; break; }
            }
            float Mt = M;
#pragma unroll
            for (int x = 0; x < kMergeMaxSplits - 1; ++x)
                if (x < np) Mt = fmaxf(Mt, __uint_as_float((uint32_t)wm[x]));
            float ot = 0.f, Zt = 0.f;
            if (Mt > -INFINITY) {
                const float f = fast_exp2(M - Mt);
                ot = f * o;
                Zt = f * Z;
#pragma unroll
                for (int x = 0; x < kMergeMaxSplits - 1; ++x) {
                    if (x < np) {
                        const float fx = fast_exp2(__uint_as_float((uint32_t)wm[x]) - Mt);
                        ot += fx * __uint_as_float((uint32_t)wo[x]);
                        Zt += fx * __uint_as_float((uint32_t)wz[x]);
                    }
                }
            }
            // a range that never published: no number is better than a wrong one
            out[bh * D + c] = ok ? f32_to_bf16_bits(Zt > 0.f ? ot / Zt : 0.f) : (uint16_t)0x7fc0;
            if (lse && c == 0) lse[bh] = !ok ? __builtin_nanf("") : (Zt > 0.f ? (Mt + log2f(Zt)) * kLn2 : -INFINITY);
            if (idx == 0 && !ok) {
                __hip_atomic_fetch_add(&g_merge_timeouts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (gave_up_flag) __hip_atomic_store(gave_up_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        } else if (MODE == kDirect) {
            out[bh * D + c] = f32_to_bf16_bits(Z > 0.f ? o / Z : 0.f);
            if (lse && c == 0) lse[bh] = Z > 0.f ? (M + log2f(Z)) * kLn2 : -INFINITY;
        } else {
            const int64_t ph = bh * nsplit + split;
            part_o[ph * D + c] = o;
            if (c == 0) { part_ml[ph * 2] = M; part_ml[ph * 2 + 1] = Z; }
        }
    }
}

// -----------------------------------------------------------------------------------------
// Generic kernel: any dtype / head_dim <= 256 / group size.  One wave per (range, query
// head, sequence); lanes over tokens for q.k, lanes over dims for p.V.  Plain FMAs.
// The fp32 cache's outputs are held to 1e-5 of their row maximum whatever the logits' size, so
// everything a long chain of roundings could spoil runs in fp64: the q.k sums (dot_row), the
// difference between a logit and the running maximum (exact in double; only the small difference
// is rounded to fp32 for the exponential), the sum of the weights and the p.V accumulators.  The
// kernel is off the hot path (none of the paper's models takes it) and stays latency-bound.
// -----------------------------------------------------------------------------------------
// acc[x] += sum_j p_j V[j][lane + 64 x] over the nv tokens of a tile; lane j holds token j's
// probability pj and row offset off.  Eight tokens' rows are requested before any is used (a row's
// address comes from another lane, so the compiler does not overlap the rows by itself); every load is
// unconditional -- components past d read the row's last component and are never stored, tokens
// past the tile's end repeat its last row with probability zero.
template <typename T, int NX>
__device__ __forceinline__ void pv_rows(const T *__restrict__ vbase, int64_t off, float pj, int nv, int d, int lane,
                                        double (&acc)[4])
{
    int cc[NX];
#pragma unroll
    for (int x = 0; x < NX; ++x) cc[x] = min(lane + 64 * x, d - 1);
    for (int j0 = 0; j0 < nv; j0 += 8) {
        float pb[8], vv[8][NX];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int jj = min(j0 + u, nv - 1);
            pb[u] = j0 + u < nv ? __shfl(pj, jj) : 0.f;
            const int64_t oj = __shfl(off, jj);
#pragma unroll
            for (int x = 0; x < NX; ++x) vv[u][x] = load_elem<T>(vbase + oj + cc[x]);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int x = 0; x < NX; ++x) acc[x] = fma((double)pb[u], (double)vv[u][x], acc[x]);
    }
}

template <typename T, bool GATHER, bool PAGED>
__global__ __launch_bounds__(64) void attn_generic_kernel(
    KvDev kv, BatchDev bv, const T *__restrict__ q, int Hq, double scale_log2,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt, int64_t kmax,
    float *__restrict__ part_o, float *__restrict__ part_ml, int nsplit, bool vec16)
{
    __shared__ float qs[256];
    const int lane = threadIdx.x;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int d = kv.head_dim;
    const int G = Hq / kv.n_kv_heads;
    const int g = h / G;

    const SeqGeom geo = seq_geom(bv, b);
    int cnt = 0;
    const int32_t *sel = nullptr;
    if (GATHER) {
        cnt = min(max(sel_cnt[b], 0), (int)min((int64_t)geo.N, kmax));
        sel = sel_idx + (int64_t)b * kmax;
    }
    const int L = GATHER ? (geo.S - geo.N + cnt) : geo.S;
    const int ntile = (L + 63) / 64;
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    for (int c = lane; c < d; c += 64) qs[c] = load_elem<T>(q + ((int64_t)b * Hq + h) * d + c);
    __syncthreads();

    const T *kbase = reinterpret_cast<const T *>(kv.k);
    const T *vbase = reinterpret_cast<const T *>(kv.v);
    float m = -INFINITY;                 // running maximum: an fp32 value, exact as a double
    double z = 0.0;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};

    for (int tile = t0; tile < t1; ++tile) {
        const int p = tile * 64 + lane;
        const bool valid = p < L;
        const int tok = pos_to_token<GATHER>(min(p, L - 1), geo, cnt, sel);
        const int64_t off = row_offset<PAGED>(kv, b, tok, g);
        const double sd = dot_row<T>(qs, kbase + off, d, vec16) * scale_log2;
        const float s = valid ? (float)sd : -INFINITY;
        const float m_new = fmaxf(m, wave_max(s));          // finite: every tile holds a valid position
        const float alpha = fast_exp2(m - m_new);
        // the weight from the exact difference: rounding it to fp32 costs 2^-24 of a number that is
        // small wherever the weight matters
        const float pj = valid ? fast_exp2((float)(sd - (double)m_new)) : 0.f;
        z = z * (double)alpha + (double)wave_sum(pj);
        m = m_new;
#pragma unroll
        for (int x = 0; x < 4; ++x) acc[x] *= (double)alpha;
        const int nv = min(64, L - tile * 64);
        if (d <= 64) pv_rows<T, 1>(vbase, off, pj, nv, d, lane, acc);
        else if (d <= 128) pv_rows<T, 2>(vbase, off, pj, nv, d, lane, acc);
        else pv_rows<T, 4>(vbase, off, pj, nv, d, lane, acc);
    }
    const int64_t ph = ((int64_t)b * Hq + h) * nsplit + split;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int c = lane + 64 * x;
        if (c < d) part_o[ph * d + c] = (float)acc[x];
    }
    if (lane == 0) { part_ml[ph * 2] = m; part_ml[ph * 2 + 1] = (float)z; }
}

// -----------------------------------------------------------------------------------------
// Merge of the per-range partials: out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) Z_s.
// -----------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_combine_kernel(
    const float *__restrict__ part_o, const float *__restrict__ part_ml, int nsplit, int d,
    T *__restrict__ out, float *__restrict__ lse)
{
    const int64_t bh = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;    // b*Hq + h
    const int c = threadIdx.x;
    const float *ml = part_ml + bh * nsplit * 2;
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, ml[2 * s]);
    float Z = 0.f, o = 0.f;
    if (M > -INFINITY) {
        for (int s = 0; s < nsplit; ++s) {
            const float f = fast_exp2(ml[2 * s] - M);
            Z += f * ml[2 * s + 1];
            if (c < d) o += f * part_o[(bh * nsplit + s) * d + c];
        }
    }
    if (c < d) store_elem<T>(out + bh * d + c, Z > 0.f ? o / Z : 0.f);
    if (lse && c == 0) lse[bh] = Z > 0.f ? (M + log2f(Z)) * kLn2 : -INFINITY;
}

// The same merge with the partials spread over the workgroup's threads (combine.hpp).
template <typename T>
__global__ __launch_bounds__(256) void attn_combine_wide_kernel(
    const float *__restrict__ part_o, const float *__restrict__ part_ml, int nsplit, int d,
    T *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ seq_meta, int wpk)
{
    __shared__ float sm_max[4];
    __shared__ float sm_z[256];
    __shared__ __align__(16) float sm_o[1024];
    combine_wide_body<T>(part_o, part_ml, nsplit, d, out, lse, seq_meta, wpk, blockIdx.x, blockIdx.y, gridDim.x,
                         CombineShared{sm_max, sm_z, sm_o});
}

// -----------------------------------------------------------------------------------------
// Host side
// -----------------------------------------------------------------------------------------
int attn_tile_tokens(const Shape &s) { return mfma_path(s) ? kTile * 4 : 64; }

size_t attn_workspace_bytes(const Shape &s, int nsplit)
{
    const size_t rows = (size_t)s.batch * s.n_q_heads * nsplit;
    return rows * (size_t)(s.kv.head_dim + 2) * sizeof(float);
}

bool attn_merges_in_kernel(const Shape &s, int nsplit)
{
    if (!mfma_path(s) || nsplit < 2 || nsplit > kMergeMaxSplits) return false;
    const size_t streams = (size_t)s.batch * s.kv.n_kv_heads;
    const size_t G = s.n_q_heads / s.kv.n_kv_heads;
    return streams <= (size_t)kMergeMaxStreams && G <= (size_t)kMergeMaxG;
}

template <bool GATHER, bool PAGED>
static void launch_mfma(int kid, const Shape &s, const void *q, float scale_log2, const int32_t *sel_idx,
                        const int32_t *sel_cnt, int64_t kmax, float *part_o, float *part_ml,
                        int nsplit, int merge_slot, uint32_t *flag, void *out, float *lse, hipStream_t stream)
{
    const int G = s.n_q_heads / s.kv.n_kv_heads;
    dim3 grid(nsplit, s.kv.n_kv_heads, s.batch);
    const bool merge = merge_slot >= 0 && nsplit > 1;
    const int slot = merge ? merge_slot : 0;
    // the stream's last range waits at most this long for the others (they run concurrently and
    // finish within microseconds of each other); past it the outputs are NaN but the call ends
    const long long spin_ticks = tune_spin_ticks();
#define FASTOCR_ATTN(DD, W, MODE) FASTOCR_LAUNCH(kid, (attn_mfma_kernel<DD, GATHER, PAGED, W, MODE>), grid, dim3(64 * W), 0, stream, \
        s.kv, s.bv, (const uint16_t *)q, s.n_q_heads, G, scale_log2, sel_idx, sel_cnt, kmax, part_o, part_ml, nsplit, \
        (uint16_t *)out, lse, slot, spin_ticks, flag)
    if (s.kv.head_dim == 64) {
        if (nsplit == 1) FASTOCR_ATTN(64, 8, kDirect);
        else if (merge) FASTOCR_ATTN(64, 8, kMerge);
        else if (tune_attn_waves() == 8) FASTOCR_ATTN(64, 8, kPartial);
        else FASTOCR_ATTN(64, 4, kPartial);
    }
    else if (nsplit == 1) FASTOCR_ATTN(128, 8, kDirect);       // one range per stream: eight waves, final output
    else if (merge) FASTOCR_ATTN(128, 8, kMerge);         // the stream's last range merges inside the launch
    else if (tune_attn_waves() == 8) FASTOCR_ATTN(128, 8, kPartial);
    else FASTOCR_ATTN(128, 4, kPartial);
#undef FASTOCR_ATTN
}

template <typename T, bool GATHER, bool PAGED>
static void launch_generic(int kid, const Shape &s, const void *q, double scale_log2, const int32_t *sel_idx,
                           const int32_t *sel_cnt, int64_t kmax, float *part_o, float *part_ml,
                           int nsplit, int, uint32_t *, void *, float *, hipStream_t stream)
{
    dim3 grid(nsplit, s.n_q_heads, s.batch), block(64);
    FASTOCR_LAUNCH(kid, (attn_generic_kernel<T, GATHER, PAGED>), grid, block, 0, stream,
        s.kv, s.bv, (const T *)q, s.n_q_heads, scale_log2, sel_idx, sel_cnt, kmax, part_o, part_ml, nsplit, s.vec16);
}

hipError_t attn_merge_timeouts(uint32_t *n) { return hipMemcpyFromSymbol(n, HIP_SYMBOL(g_merge_timeouts), sizeof(uint32_t)); }

hipError_t launch_attn(const Shape &s, const void *q, float scale, const int32_t *sel_idx,
                       const int32_t *sel_cnt, int64_t kmax, void *out, float *lse, void *ws,
                       int nsplit, int merge_slot, uint32_t *gave_up_flag, hipStream_t stream)
{
    const bool gather = sel_idx != nullptr;
    const bool merge = merge_slot >= 0 && attn_merges_in_kernel(s, nsplit);
    if (!merge) merge_slot = -1;
    const int d = s.kv.head_dim;
    float *part_o = reinterpret_cast<float *>(ws);
    float *part_ml = part_o + (size_t)s.batch * s.n_q_heads * nsplit * d;
    const float scale_log2f = scale * kLog2e;
    const double scale_log2d = (double)scale * 1.4426950408889634074;     // the fp64 kernels take the scale unrounded
    const int kid = gather ? K_SPARSE_ATTN : K_DENSE_ATTN;

#define FASTOCR_DISPATCH(FN, scale_log2, ...)                                                                      \
    do {                                                                                               \
        if (gather) { if (s.paged) FN<__VA_ARGS__ true, true>(kid, s, q, scale_log2, sel_idx, sel_cnt, kmax, part_o, part_ml, nsplit, merge_slot, gave_up_flag, out, lse, stream); \
                      else         FN<__VA_ARGS__ true, false>(kid, s, q, scale_log2, sel_idx, sel_cnt, kmax, part_o, part_ml, nsplit, merge_slot, gave_up_flag, out, lse, stream); } \
        else        { if (s.paged) FN<__VA_ARGS__ false, true>(kid, s, q, scale_log2, sel_idx, sel_cnt, kmax, part_o, part_ml, nsplit, merge_slot, gave_up_flag, out, lse, stream); \
                      else         FN<__VA_ARGS__ false, false>(kid, s, q, scale_log2, sel_idx, sel_cnt, kmax, part_o, part_ml, nsplit, merge_slot, gave_up_flag, out, lse, stream); } \
    } while (0)
    if (mfma_path(s)) {
        FASTOCR_DISPATCH(launch_mfma, scale_log2f, );
    } else if (s.dtype == DT_BF16) {
        FASTOCR_DISPATCH(launch_generic, scale_log2d, uint16_t, );
    } else {
        FASTOCR_DISPATCH(launch_generic, scale_log2d, float, );
    }
#undef FASTOCR_DISPATCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (mfma_path(s) && (nsplit == 1 || merge)) return hipSuccess;        // the kernel wrote the final output itself

    return launch_attn_combine(s, part_o, part_ml, nsplit, out, lse, stream);
}

hipError_t launch_attn_combine(const Shape &s, const float *part_o, const float *part_ml, int nsplit,
                               void *out, float *lse, hipStream_t stream, const int32_t *seq_meta, int wpk)
{
    const int d = s.kv.head_dim;
    dim3 grid(s.n_q_heads, s.batch), block(256);
    if (seq_meta && d % 4 != 0) return hipErrorInvalidValue;
    if (d % 4 == 0 && (nsplit >= 2 || seq_meta)) {
        // several partials per head: spread them over the workgroup's threads (two partials as well: its
        // form for few partials needs one memory round trip where the plain walk below needs two)
        if (s.dtype == DT_BF16)
            FASTOCR_LAUNCH(K_ATTN_COMBINE, attn_combine_wide_kernel<uint16_t>, grid, block, 0, stream, part_o, part_ml, nsplit, d, (uint16_t *)out, lse, seq_meta, wpk);
        else
            FASTOCR_LAUNCH(K_ATTN_COMBINE, attn_combine_wide_kernel<float>, grid, block, 0, stream, part_o, part_ml, nsplit, d, (float *)out, lse, seq_meta, wpk);
        return hipGetLastError();
    }
    if (s.dtype == DT_BF16)
        FASTOCR_LAUNCH(K_ATTN_COMBINE, attn_combine_kernel<uint16_t>, grid, block, 0, stream, part_o, part_ml, nsplit, d, (uint16_t *)out, lse);
    else
        FASTOCR_LAUNCH(K_ATTN_COMBINE, attn_combine_kernel<float>, grid, block, 0, stream, part_o, part_ml, nsplit, d, (float *)out, lse);
    return hipGetLastError();
}

}  // namespace fastocr
