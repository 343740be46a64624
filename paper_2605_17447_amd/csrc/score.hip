// Focal-layer scoring: head-averaged softmax attention of the current query over the whole
// cache, read at the image tokens (Eq. 1; text under Eq. 2).
//
// The average over heads is taken AFTER each head's softmax, so no score is final before
// every head's normaliser over all S keys is known.  Two kernels:
//   logits   : streams K once.  Per (sequence, kv head, token range) it computes the G query
//              heads' logits, parks them (fp32, log2 domain) in the workspace and reduces a
//              per-range (max, sum-exp) per head.
//   finalize : merges the per-range statistics into each head's log-sum-exp and writes
//              score_i = (1/Hq) sum_h 2^(logit_h,i - lse_h) for the image tokens.
// The K stream uses the same MFMA tiling as the attention kernel (tokens x heads tiles of
// v_mfma_f32_16x16x32_bf16) for bf16 / head_dim 128, and a plain fp32 kernel otherwise.
#include "kernels.hpp"

namespace fastocr {

constexpr int kTile = 32;          // tokens per wave tile

// parked logits: fp32 [sequence][kv head][token (pitch)][Gp], Gp = G rounded up to 4 heads
__host__ __device__ inline int park_heads(int G) { return (G + 3) / 4 * 4; }

// One workgroup per (token range, kv head, sequence); its four waves walk interleaved 32-token
// tiles.  A tile is loaded with 1 KB-contiguous 16-byte loads (4 rows of 256 B per instruction),
// re-laid through a wave-private XOR-swizzled LDS tile into the MFMA B layout, and multiplied
//     C[head][token] = Q (16 heads x 32 dims) * K^T (32 dims x 16 tokens)   (v_mfma_f32_16x16x32_bf16)
// so that a lane ends up with 4 consecutive heads of one token: the parked row [token][Gp] is
// written with one 16-byte store per lane and no transposition.
//   GR = 8 : the group's heads fill rows 0..7 for the tile's first 16 tokens and rows 8..15 for
//            its second 16 tokens (the same accumulator, Q placed in the upper rows for the
//            second product): all 64 lanes hold live logits, one 1 KB store per tile.
//   GR = 16: heads fill all 16 rows; two accumulators per tile.
// Each lane keeps a running (max, sum-exp) for its 4 heads; lanes, waves and ranges are merged
// at the end.
// D = 64 (rows of 128 bytes): a load instruction brings 8 rows, the LDS tile has a pitch of 128
// bytes with chunk ^ ((row >> 1) & 7), and the product takes two k-steps per 16-token half.
template <int D, bool PAGED, int GR, int kWaves, int NBUF>
__global__ __launch_bounds__(64 * kWaves) void score_mfma_kernel(
    KvDev kv, BatchDev bv, const uint16_t *__restrict__ q, int Hq, int G, float scale_log2,
    float *__restrict__ logits, int64_t pitch, float *__restrict__ part_ml, int nsplit)
{
    __shared__ __align__(16) unsigned char smem[kWaves][8192];
    __shared__ float sm_m[kWaves][16], sm_z[kWaves][16];

    static_assert(D == 128 || D == 64, "head_dim 128 or 64");
    constexpr int KS = D / 32;            // k-steps per product
    constexpr int NL = D / 16;            // 1 KB load instructions per 32-token tile
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int Gp = park_heads(G);

    const SeqGeom geo = seq_geom(bv, b);
    const int L = geo.S;
    const int ntile = (L + kTile - 1) / kTile;
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    // Q as the A operand: lane (row li, k-block lg) holds dims 32*kk + 8*lg .. +7 of step kk.
    u32x4 qlo[KS], qhi[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        qlo[kk] = u32x4{0u, 0u, 0u, 0u};
        qhi[kk] = u32x4{0u, 0u, 0u, 0u};
        const int hl = li, hh = li - 8;
        if (hl < G && (GR == 16 || hl < 8)) {
            const uint16_t *qp = q + ((int64_t)b * Hq + (int64_t)kvh * G + hl) * D + 8 * (4 * kk + lg);
            qlo[kk] = *reinterpret_cast<const u32x4 *>(qp);
        }
        if (GR == 8 && hh >= 0 && hh < G) {
            const uint16_t *qp = q + ((int64_t)b * Hq + (int64_t)kvh * G + hh) * D + 8 * (4 * kk + lg);
            qhi[kk] = *reinterpret_cast<const u32x4 *>(qp);
        }
    }
    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(kv.k);
    const int64_t seq_base = row_offset<false>(kv, b, 0, kvh);

    auto rowoff_of = [&](int tile) -> int64_t {
        int p = min(tile * kTile + (lane & 31), L - 1);
        return row_offset<PAGED>(kv, b, p, kvh);
    };

    // load e covers rows 4e .. 4e+3 of the tile (D = 128: lane group lg takes row 4e+lg, lane li its 16-byte
    // chunk) or rows 8e .. 8e+7 (D = 64: one row per 8 lanes)
    constexpr int CH = D / 8;                      // 16-byte chunks per row
    const int lrow = lane / CH, lchunk = lane % CH;
    auto load_tile = [&](int tile, int64_t off, u32x4(&K)[NL]) {
#pragma unroll
        for (int e = 0; e < NL; ++e) {
            const int r = (64 / CH) * e + lrow;
            int64_t ro;
            if (PAGED) ro = __shfl(off, r);
            else ro = seq_base + (int64_t)min(tile * kTile + r, L - 1) * kv.stride_token;
            K[e] = stream_load(kbase + ro + 8 * lchunk);
        }
    };
    // byte offset of chunk c of row r in the wave's LDS tile
    auto lds_at = [&](int r, int c) { return D == 128 ? r * 256 + (((c ^ r) & 15) << 4) : r * 128 + ((c ^ ((r >> 1) & 7)) << 4); };

    // heads of this lane: hbase .. hbase+3 ; token of the tile: li (+16 in the upper lane groups for GR = 8)
    const int hbase = (GR == 8) ? 4 * (lg & 1) : 4 * lg;
    const int tok_in_tile = (GR == 8) ? li + 16 * (lg >> 1) : li;
    const bool park = hbase < Gp;
    float m[4], z[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { m[r] = kMinusHuge; z[r] = 0.f; }
    float *lpark = logits + ((int64_t)b * kv.n_kv_heads + kvh) * pitch * Gp + hbase;

    auto compute = [&](int tile, u32x4(&K)[NL]) {
        unsigned char *sw = smem[wave];
#pragma unroll
        for (int e = 0; e < NL; ++e) {
            const int r = (64 / CH) * e + lrow;
            *reinterpret_cast<u32x4 *>(sw + lds_at(r, lchunk)) = K[e];
        }
        wave_lds_fence();
        u32x4 kb[2 * KS];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                kb[KS * T + kk] = *reinterpret_cast<const u32x4 *>(sw + lds_at(16 * T + li, 4 * kk + lg));
        wave_lds_fence();
        const int p0 = tile * kTile;
        if (GR == 8) {
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qlo[kk]),
                                                            __builtin_bit_cast(bf16x8, kb[kk]), s, 0, 0, 0);
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qhi[kk]),
                                                            __builtin_bit_cast(bf16x8, kb[KS + kk]), s, 0, 0, 0);
            const int p = p0 + tok_in_tile;
            const bool valid = p < L;
#pragma unroll
            for (int r = 0; r < 4; ++r) s[r] = valid ? s[r] * scale_log2 : -INFINITY;
            if (park) *reinterpret_cast<f32x4 *>(lpark + (int64_t)p * Gp) = s;     // p < pitch
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float mn = fmaxf(m[r], s[r]);
                z[r] = z[r] * fast_exp2(m[r] - mn) + fast_exp2(s[r] - mn);
                m[r] = mn;
            }
        } else {
            f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qlo[kk]),
                                                             __builtin_bit_cast(bf16x8, kb[kk]), s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qlo[kk]),
                                                             __builtin_bit_cast(bf16x8, kb[KS + kk]), s1, 0, 0, 0);
            }
            const int p = p0 + li;
            const bool v0 = p < L, v1 = p + 16 < L;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s0[r] = v0 ? s0[r] * scale_log2 : -INFINITY;
                s1[r] = v1 ? s1[r] * scale_log2 : -INFINITY;
            }
            if (park) {
                *reinterpret_cast<f32x4 *>(lpark + (int64_t)p * Gp) = s0;
                *reinterpret_cast<f32x4 *>(lpark + (int64_t)(p + 16) * Gp) = s1;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float mn = fmaxf(m[r], fmaxf(s0[r], s1[r]));
                z[r] = z[r] * fast_exp2(m[r] - mn) + fast_exp2(s0[r] - mn) + fast_exp2(s1[r] - mn);
                m[r] = mn;
            }
        }
    };

    if (t0 + wave < t1) {
        // NBUF register buffers, software pipelined: a buffer is refilled (with the tile NBUF rounds
        // ahead) right after it has been consumed, so NBUF-1 tiles are in flight during a compute.
        // The refills are unconditional (past the end the last tile is loaded again) so that no
        // branch separates a load from the wait that matches it -- a conditional prefetch makes the
        // compiler drain every outstanding load at the join.
        u32x4 KB[NBUF][NL];
        int64_t off[NBUF];
        int tile = t0 + wave;
        const int last = tile + (t1 - 1 - tile) / kWaves * kWaves;
#pragma unroll
        for (int i = 0; i < NBUF; ++i) {
            const int tl = min(tile + i * kWaves, last);
            off[i] = PAGED ? rowoff_of(tl) : 0;
            load_tile(tl, off[i], KB[i]);
        }
        for (;;) {
#pragma unroll
            for (int i = 0; i < NBUF; ++i) {
                compute(tile, KB[i]);
                const int tl = min(tile + NBUF * kWaves, last);
                off[i] = PAGED ? rowoff_of(tl) : 0;
                load_tile(tl, off[i], KB[i]);
                tile += kWaves;
                if (tile > last) goto stream_done;
            }
        }
    }
stream_done:

    // ---- merge lanes that hold the same heads, then waves, then write the range's statistics ----
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) softmax_merge(m[r], z[r], __shfl_xor(m[r], o), __shfl_xor(z[r], o));
        if (GR == 8) softmax_merge(m[r], z[r], __shfl_xor(m[r], 32), __shfl_xor(z[r], 32));
    }
    if (li == 0 && (GR == 16 || lg < 2)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { sm_m[wave][hbase + r] = m[r]; sm_z[wave][hbase + r] = z[r]; }
    }
    __syncthreads();
    if (threadIdx.x < G) {
        const int hh = threadIdx.x;
        float M = sm_m[0][hh];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][hh]);
        float Z = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) Z += fast_exp2(sm_m[w][hh] - M) * sm_z[w][hh];
        const int64_t ph = ((int64_t)b * Hq + (int64_t)kvh * G + hh) * nsplit + split;
        part_ml[ph * 2] = M;
        part_ml[ph * 2 + 1] = Z;
    }
}

// Generic: one wave per (range, query head, sequence), lanes over tokens.  The q.k sums run in
// fp64 (dot_row) and are scaled there; the logit is rounded to fp32 once, when it is parked.
template <typename T, bool PAGED>
__global__ __launch_bounds__(64) void score_generic_kernel(
    KvDev kv, BatchDev bv, const T *__restrict__ q, int Hq, double scale_log2,
    float *__restrict__ logits, int64_t pitch, float *__restrict__ part_ml, int nsplit, bool vec16)
{
    __shared__ float qs[256];
    const int lane = threadIdx.x;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int d = kv.head_dim;
    const int G = Hq / kv.n_kv_heads, Gp = park_heads(G);
    const int g = h / G;
    const SeqGeom geo = seq_geom(bv, b);
    const int L = geo.S;
    const int ntile = (L + 63) / 64;
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    for (int c = lane; c < d; c += 64) qs[c] = load_elem<T>(q + ((int64_t)b * Hq + h) * d + c);
    __syncthreads();
    const T *kbase = reinterpret_cast<const T *>(kv.k);
    float *lrow = logits + ((int64_t)b * kv.n_kv_heads + g) * pitch * Gp + (h - g * G);   // [token][Gp]
    float m = kMinusHuge, z = 0.f;
    for (int tile = t0; tile < t1; ++tile) {
        const int p = tile * 64 + lane;
        const bool valid = p < L;
        const int64_t off = row_offset<PAGED>(kv, b, min(p, L - 1), g);
        const float s = valid ? (float)(dot_row<T>(qs, kbase + off, d, vec16) * scale_log2) : -INFINITY;
        lrow[(int64_t)p * Gp] = s;                       // p < pitch: pitch is a multiple of 64
        const float m_new = fmaxf(m, wave_max(s));
        z = z * fast_exp2(m - m_new) + wave_sum(fast_exp2(s - m_new));
        m = m_new;
    }
    if (lane == 0) {
        const int64_t ph = ((int64_t)b * Hq + h) * nsplit + split;
        part_ml[ph * 2] = m;
        part_ml[ph * 2 + 1] = z;
    }
}

// Finalize: per-head log-sum-exp from the range statistics, then the head average
//     score_i = (1/Hq) sum_h 2^(logit_h,i - lse_h)
// read back from the parked [token][Gp] rows.  LP lanes share a token (one 16-byte quad of heads
// per kv head each), so that a wave's loads cover contiguous memory.
constexpr int kFinThreads = 256;

__host__ __device__ inline int fin_lanes_per_token(int Gp) { return Gp == 8 ? 2 : (Gp == 16 ? 4 : 1); }

__global__ __launch_bounds__(kFinThreads) void score_finalize_kernel(
    BatchDev bv, int Hq, int n_kv_heads, const float *__restrict__ logits, int64_t pitch,
    const float *__restrict__ part_ml, int nsplit, float *__restrict__ scores,
    float *__restrict__ lse, float *__restrict__ mass_part)
{
    extern __shared__ float lse2[];                    // [Hq]
    __shared__ float red[kFinThreads / 64];
    const int b = blockIdx.y;
    const SeqGeom geo = seq_geom(bv, b);
    // every head's log-sum-exp from its nsplit range statistics: 8 lanes share a head and walk every
    // 8th range (a serial walk is bound by load latency once there are dozens of ranges)
    for (int h0 = 0; h0 < Hq; h0 += kFinThreads / 8) {
        const int h = h0 + (threadIdx.x >> 3), part = threadIdx.x & 7;
        float M = kMinusHuge, Z = 0.f;
        if (h < Hq) {
            const float *ml = part_ml + ((int64_t)b * Hq + h) * nsplit * 2;
            for (int s = part; s < nsplit; s += 8) softmax_merge(M, Z, ml[2 * s], ml[2 * s + 1]);
        }
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) softmax_merge(M, Z, __shfl_xor(M, o), __shfl_xor(Z, o));
        if (h < Hq && part == 0) {
            const float l2 = Z > 0.f ? M + log2f(Z) : -INFINITY;
            lse2[h] = l2;
            if (lse && blockIdx.x == 0) lse[(int64_t)b * Hq + h] = l2 * kLn2;
        }
    }
    __syncthreads();
    const int G = Hq / n_kv_heads, Gp = park_heads(G);
    const int LP = fin_lanes_per_token(Gp);
    const int nq = Gp / 4 / LP;                        // 16-byte quads per lane per kv head
    const int i = (blockIdx.x * kFinThreads + threadIdx.x) / LP;
    const int sub = threadIdx.x % LP;
    float acc = 0.f;
    if (i < geo.N) {
        const float *lp = logits + ((int64_t)b * n_kv_heads * pitch + geo.v0 + i) * Gp;
        for (int g = 0; g < n_kv_heads; ++g) {
            const float *row = lp + (int64_t)g * pitch * Gp;
            for (int qd = 0; qd < nq; ++qd) {
                const int x0 = 4 * (sub * nq + qd);
                const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(row + x0));
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (x0 + r < G) acc += fast_exp2(v[r] - lse2[g * G + x0 + r]);
            }
        }
    }
    for (int o = 1; o < LP; o <<= 1) acc += __shfl_xor(acc, o);
    float sc = 0.f;
    if (i < geo.N && sub == 0) {
        sc = acc / (float)Hq;
        scores[(int64_t)b * bv.max_vis_len + i] = sc;
    }
    if (mass_part) {
        float w = wave_sum(sc);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            for (int x = 0; x < kFinThreads / 64; ++x) t += red[x];
            mass_part[(int64_t)b * gridDim.x + blockIdx.x] = t;
        }
    }
}

__global__ void mass_reduce_kernel(const float *__restrict__ mass_part, int nblk, float *__restrict__ img_mass)
{
    const int b = blockIdx.x;
    float t = 0.f;
    for (int x = threadIdx.x; x < nblk; x += 64) t += mass_part[(int64_t)b * nblk + x];
    t = wave_sum(t);
    if (threadIdx.x == 0) img_mass[b] = t;
}

// -----------------------------------------------------------------------------------------
int score_tile_tokens(const Shape &s) { return mfma_path(s) ? kTile : 64; }

static int fin_blocks(const Shape &s)
{
    const int LP = fin_lanes_per_token(park_heads(s.n_q_heads / s.kv.n_kv_heads));
    const int per = kFinThreads / LP;
    return max(1, (s.bv.max_vis_len + per - 1) / per);
}

static size_t parked_floats(const Shape &s)
{
    const int Gp = park_heads(s.n_q_heads / s.kv.n_kv_heads);
    return (size_t)s.batch * s.kv.n_kv_heads * (size_t)logit_pitch(s.bv.max_seq_len) * Gp;
}

size_t score_workspace_bytes(const Shape &s, int nsplit)
{
    size_t bytes = parked_floats(s) * sizeof(float);
    bytes += (size_t)s.batch * s.n_q_heads * (size_t)nsplit * 2 * sizeof(float);
    bytes += (size_t)s.batch * fin_blocks(s) * sizeof(float);
    return bytes;
}

hipError_t launch_score(const Shape &s, const void *q, float scale, float *scores, float *lse,
                        float *img_mass, void *ws, int nsplit, hipStream_t stream)
{
    const int64_t pitch = logit_pitch(s.bv.max_seq_len);
    const size_t rows = (size_t)s.batch * s.n_q_heads;
    float *logits = reinterpret_cast<float *>(ws);
    float *part_ml = logits + parked_floats(s);
    float *mass_part = part_ml + rows * nsplit * 2;
    const float scale_log2 = scale * kLog2e;
    const int G = s.n_q_heads / s.kv.n_kv_heads;

    if (mfma_path(s)) {
        dim3 grid(nsplit, s.kv.n_kv_heads, s.batch);
#define FASTOCR_SCORE(DD, P, GR) FASTOCR_LAUNCH(K_SCORE_LOGITS, (score_mfma_kernel<DD, P, GR, 4, 2>), grid, dim3(256), 0, stream, \
        s.kv, s.bv, (const uint16_t *)q, s.n_q_heads, G, scale_log2, logits, pitch, part_ml, nsplit)
        if (s.kv.head_dim == 64) {
            if (s.paged) { if (G <= 8) FASTOCR_SCORE(64, true, 8); else FASTOCR_SCORE(64, true, 16); }
            else         { if (G <= 8) FASTOCR_SCORE(64, false, 8); else FASTOCR_SCORE(64, false, 16); }
        }
        else if (s.paged) { if (G <= 8) FASTOCR_SCORE(128, true, 8); else FASTOCR_SCORE(128, true, 16); }
        else              { if (G <= 8) FASTOCR_SCORE(128, false, 8); else FASTOCR_SCORE(128, false, 16); }
#undef FASTOCR_SCORE
    } else {
        dim3 grid(nsplit, s.n_q_heads, s.batch), block(64);
#define FASTOCR_SCORE(T, P) FASTOCR_LAUNCH(K_SCORE_LOGITS, (score_generic_kernel<T, P>), grid, block, 0, stream, \
        s.kv, s.bv, (const T *)q, s.n_q_heads, (double)scale * 1.4426950408889634074, logits, pitch, part_ml, nsplit, s.vec16)
        if (s.dtype == DT_BF16) { if (s.paged) FASTOCR_SCORE(uint16_t, true); else FASTOCR_SCORE(uint16_t, false); }
        else                    { if (s.paged) FASTOCR_SCORE(float, true); else FASTOCR_SCORE(float, false); }
#undef FASTOCR_SCORE
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    const int nblk = fin_blocks(s);
    dim3 fgrid(nblk, s.batch), fblock(kFinThreads);
    FASTOCR_LAUNCH(K_SCORE_FINALIZE, score_finalize_kernel, fgrid, fblock, (size_t)s.n_q_heads * sizeof(float), stream,
        s.bv, s.n_q_heads, s.kv.n_kv_heads, logits, pitch, part_ml, nsplit, scores, lse, img_mass ? mass_part : nullptr);
    if (img_mass) mass_reduce_kernel<<<s.batch, 64, 0, stream>>>(mass_part, nblk, img_mass);
    return hipGetLastError();
}

}  // namespace fastocr
