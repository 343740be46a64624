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

extern int g_tune_k_via_lds;
extern int g_tune_dbg;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 32;
constexpr int kWaves = 4;

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int tile_row(int lg, int e) { return (e < 4) ? (4 * lg + e) : (16 + 4 * lg + (e - 4)); }

template <bool PAGED, bool KLDS>
__global__ __launch_bounds__(256, 3) void score_mfma_kernel(
    KvDev kv, BatchDev bv, const uint16_t *__restrict__ q, int Hq, int G, float scale_log2,
    float *__restrict__ logits, int64_t pitch, float *__restrict__ part_ml, int nsplit, int dbg)
{
    __shared__ __align__(16) unsigned char smem[kWaves][8192];
    __shared__ float sm_m[kWaves][16], sm_z[kWaves][16];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int li = lane & 15, lg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;

    const SeqGeom geo = seq_geom(bv, b);
    const int L = geo.S;
    const int ntile = (L + kTile - 1) / kTile;
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    u32x4 qreg[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        qreg[kk] = u32x4{0u, 0u, 0u, 0u};
        if (li < G) {
            const uint16_t *qp = q + ((int64_t)b * Hq + (int64_t)kvh * G + li) * 128 + 8 * (4 * kk + lg);
            qreg[kk] = *reinterpret_cast<const u32x4 *>(qp);
        }
    }
    const uint16_t *kbase = reinterpret_cast<const uint16_t *>(kv.k);
    const int64_t seq_base = row_offset<false>(kv, b, 0, kvh);

    auto rowoff_of = [&](int tile) -> int64_t {
        int p = min(tile * kTile + (lane & 31), L - 1);
        return row_offset<PAGED>(kv, b, p, kvh);
    };

    auto load_tile = [&](int tile, int64_t off, u32x4(&K)[8]) {
        if (KLDS) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = tile_row(lg, e);
                int64_t ro;
                if (PAGED) ro = __shfl(off, r);
                else ro = seq_base + (int64_t)min(tile * kTile + r, L - 1) * kv.stride_token;
                K[e] = *reinterpret_cast<const u32x4 *>(kbase + ro + 8 * li);
            }
        } else {
#pragma unroll
            for (int T = 0; T < 2; ++T) {
                const int r = 16 * T + li;
                int64_t ro;
                if (PAGED) ro = __shfl(off, r);
                else ro = seq_base + (int64_t)min(tile * kTile + r, L - 1) * kv.stride_token;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    K[4 * T + kk] = *reinterpret_cast<const u32x4 *>(kbase + ro + 8 * (4 * kk + lg));
            }
        }
    };

    float m = -INFINITY, zl = 0.f;
    float *ltile = logits + ((int64_t)b * kv.n_kv_heads + kvh) * pitch * G;    // [token][G]

    auto compute = [&](int tile, u32x4(&K)[8]) {
        u32x4 ka[8];
        if (KLDS) {
            unsigned char *sw = smem[wave];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = tile_row(lg, e);
                *reinterpret_cast<u32x4 *>(sw + r * 256 + ((li ^ (r & 15)) << 4)) = K[e];
            }
            wave_lds_fence();
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const int c = 4 * kk + lg;
                    ka[4 * T + kk] = *reinterpret_cast<const u32x4 *>(sw + (16 * T + li) * 256 + (((c ^ li) & 15) << 4));
                }
            wave_lds_fence();
        } else {
#pragma unroll
            for (int x = 0; x < 8; ++x) ka[x] = K[x];
        }
        f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kk]),
                                                         __builtin_bit_cast(bf16x8, qreg[kk]), s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[4 + kk]),
                                                         __builtin_bit_cast(bf16x8, qreg[kk]), s1, 0, 0, 0);
        }
        const int pbase = tile * kTile + 4 * lg;
        f32x4 a, c2;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            a[r] = (pbase + r < L) ? s0[r] * scale_log2 : -INFINITY;
            c2[r] = (pbase + 16 + r < L) ? s1[r] * scale_log2 : -INFINITY;
        }
        if (!(dbg & 1)) {
            // Park the tile's logits token-major ([token][G heads]): staged through LDS so that the
            // wave writes one contiguous run of 32*G floats with 16-byte stores.
            float *st = reinterpret_cast<float *>(smem[wave]);
            if (li < G) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    st[(4 * lg + r) * G + li] = a[r];
                    st[(16 + 4 * lg + r) * G + li] = c2[r];
                }
            }
            wave_lds_fence();
            float *dst = ltile + (int64_t)((dbg & 8) ? (tile & 3) : tile) * kTile * G;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int o = 4 * (lane + 64 * x);
                if (o < kTile * G && (!(dbg & 16) || (tile & 4))) *reinterpret_cast<f32x4 *>(dst + o) = *reinterpret_cast<const f32x4 *>(st + o);
            }
            wave_lds_fence();
        }
        float mx = fmaxf(fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])), fmaxf(fmaxf(c2[0], c2[1]), fmaxf(c2[2], c2[3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx);
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) ps += fast_exp2(a[r] - m_new) + fast_exp2(c2[r] - m_new);
        zl = zl * fast_exp2(m - m_new) + ps;
        m = m_new;
    };

    if (t0 + wave < t1) {
        // Two register buffers, software pipelined: the loads of the next tile are issued before the
        // current one is consumed.  They are issued unconditionally (past the end the last tile is
        // loaded again) so that no branch separates a load from the wait that matches it -- a
        // conditional prefetch makes the compiler drain every outstanding load at the join.
        u32x4 KA[8], KB[8];
        int tile = t0 + wave;
        const int last = tile + (t1 - 1 - tile) / kWaves * kWaves;
        int64_t off_a = 0, off_b = 0;
        if (PAGED) off_a = rowoff_of(tile);
        load_tile(tile, off_a, KA);
        if (PAGED) off_b = rowoff_of(min(tile + kWaves, last));
        while (true) {
            load_tile(min(tile + kWaves, last), off_b, KB);
            if (PAGED) off_a = rowoff_of(min(tile + 2 * kWaves, last));
            compute(tile, KA);
            tile += kWaves;
            if (tile > last) break;
            load_tile(min(tile + kWaves, last), off_a, KA);
            if (PAGED) off_b = rowoff_of(min(tile + 2 * kWaves, last));
            compute(tile, KB);
            tile += kWaves;
            if (tile > last) break;
        }
    }

    zl += __shfl_xor(zl, 16);
    zl += __shfl_xor(zl, 32);
    if (lg == 0) { sm_m[wave][li] = m; sm_z[wave][li] = zl; }
    __syncthreads();
    if (threadIdx.x < G) {
        const int hh = threadIdx.x;
        float M = sm_m[0][hh];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][hh]);
        float Z = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < kWaves; ++w) Z += fast_exp2(sm_m[w][hh] - M) * sm_z[w][hh];
        }
        const int64_t ph = ((int64_t)b * Hq + (int64_t)kvh * G + hh) * nsplit + split;
        part_ml[ph * 2] = M;
        part_ml[ph * 2 + 1] = Z;
    }
}

// Generic: one wave per (range, query head, sequence), lanes over tokens.
template <typename T, bool PAGED>
__global__ __launch_bounds__(64) void score_generic_kernel(
    KvDev kv, BatchDev bv, const T *__restrict__ q, int Hq, float scale_log2,
    float *__restrict__ logits, int64_t pitch, float *__restrict__ part_ml, int nsplit)
{
    __shared__ float qs[256];
    const int lane = threadIdx.x;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int d = kv.head_dim;
    const int g = h / (Hq / kv.n_kv_heads);
    const SeqGeom geo = seq_geom(bv, b);
    const int L = geo.S;
    const int ntile = (L + 63) / 64;
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    for (int c = lane; c < d; c += 64) qs[c] = load_elem<T>(q + ((int64_t)b * Hq + h) * d + c);
    __syncthreads();
    const T *kbase = reinterpret_cast<const T *>(kv.k);
    const int G = Hq / kv.n_kv_heads;
    float *lrow = logits + ((int64_t)b * kv.n_kv_heads + g) * pitch * G + (h - g * G);   // [token][G]
    float m = -INFINITY, z = 0.f;
    for (int tile = t0; tile < t1; ++tile) {
        const int p = tile * 64 + lane;
        const bool valid = p < L;
        const int64_t off = row_offset<PAGED>(kv, b, min(p, L - 1), g);
        float s = 0.f;
        for (int c = 0; c < d; ++c) s = fmaf(qs[c], load_elem<T>(kbase + off + c), s);
        s = valid ? s * scale_log2 : -INFINITY;
        lrow[(int64_t)p * G] = s;                        // p < pitch: pitch is a multiple of 64
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

// Finalize: per-head log-sum-exp from the range statistics, then the head average.
constexpr int kFinThreads = 256;

__global__ __launch_bounds__(kFinThreads) void score_finalize_kernel(
    BatchDev bv, int Hq, int n_kv_heads, const float *__restrict__ logits, int64_t pitch,
    const float *__restrict__ part_ml, int nsplit, float *__restrict__ scores,
    float *__restrict__ lse, float *__restrict__ mass_part)
{
    extern __shared__ float lse2[];                    // [Hq]
    __shared__ float red[kFinThreads / 64];
    const int b = blockIdx.y;
    const SeqGeom geo = seq_geom(bv, b);
    for (int h = threadIdx.x; h < Hq; h += kFinThreads) {
        const float *ml = part_ml + ((int64_t)b * Hq + h) * nsplit * 2;
        float M = -INFINITY;
        for (int s = 0; s < nsplit; ++s) M = fmaxf(M, ml[2 * s]);
        float Z = 0.f;
        if (M > -INFINITY)
            for (int s = 0; s < nsplit; ++s) Z += fast_exp2(ml[2 * s] - M) * ml[2 * s + 1];
        const float l2 = Z > 0.f ? M + log2f(Z) : -INFINITY;
        lse2[h] = l2;
        if (lse && blockIdx.x == 0) lse[(int64_t)b * Hq + h] = l2 * kLn2;
    }
    __syncthreads();
    const int i = blockIdx.x * kFinThreads + threadIdx.x;
    float sc = 0.f;
    if (i < geo.N) {
        // logits are parked as [sequence][kv head][token][G]
        const int G = Hq / n_kv_heads;
        const float *lp = logits + ((int64_t)b * n_kv_heads * pitch + geo.v0 + i) * G;
        float acc = 0.f;
        for (int g = 0; g < n_kv_heads; ++g) {
            const float *lg_ = lp + (int64_t)g * pitch * G;
            for (int x = 0; x < G; ++x) acc += fast_exp2(lg_[x] - lse2[g * G + x]);
        }
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

static int fin_blocks(const Shape &s) { return max(1, (s.bv.max_vis_len + kFinThreads - 1) / kFinThreads); }

size_t score_workspace_bytes(const Shape &s, int nsplit)
{
    const size_t rows = (size_t)s.batch * s.n_q_heads;
    size_t bytes = rows * (size_t)logit_pitch(s.bv.max_seq_len) * sizeof(float);
    bytes += rows * (size_t)nsplit * 2 * sizeof(float);
    bytes += (size_t)s.batch * fin_blocks(s) * sizeof(float);
    return bytes;
}

hipError_t launch_score(const Shape &s, const void *q, float scale, float *scores, float *lse,
                        float *img_mass, void *ws, int nsplit, hipStream_t stream)
{
    const int64_t pitch = logit_pitch(s.bv.max_seq_len);
    const size_t rows = (size_t)s.batch * s.n_q_heads;
    float *logits = reinterpret_cast<float *>(ws);
    float *part_ml = logits + rows * pitch;
    float *mass_part = part_ml + rows * nsplit * 2;
    const float scale_log2 = scale * kLog2e;
    const int G = s.n_q_heads / s.kv.n_kv_heads;

    timer_begin(K_SCORE_LOGITS, stream);
    if (mfma_path(s)) {
        dim3 grid(nsplit, s.kv.n_kv_heads, s.batch), block(256);
#define FASTOCR_SCORE(P, KL) score_mfma_kernel<P, KL><<<grid, block, 0, stream>>>( \
        s.kv, s.bv, (const uint16_t *)q, s.n_q_heads, G, scale_log2, logits, pitch, part_ml, nsplit, g_tune_dbg)
        if (s.paged) { if (g_tune_k_via_lds) FASTOCR_SCORE(true, true); else FASTOCR_SCORE(true, false); }
        else         { if (g_tune_k_via_lds) FASTOCR_SCORE(false, true); else FASTOCR_SCORE(false, false); }
#undef FASTOCR_SCORE
    } else {
        dim3 grid(nsplit, s.n_q_heads, s.batch), block(64);
#define FASTOCR_SCORE(T, P) score_generic_kernel<T, P><<<grid, block, 0, stream>>>( \
        s.kv, s.bv, (const T *)q, s.n_q_heads, scale_log2, logits, pitch, part_ml, nsplit)
        if (s.dtype == DT_BF16) { if (s.paged) FASTOCR_SCORE(uint16_t, true); else FASTOCR_SCORE(uint16_t, false); }
        else                    { if (s.paged) FASTOCR_SCORE(float, true); else FASTOCR_SCORE(float, false); }
#undef FASTOCR_SCORE
    }
    timer_end(K_SCORE_LOGITS, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    timer_begin(K_SCORE_FINALIZE, stream);
    const int nblk = fin_blocks(s);
    dim3 fgrid(nblk, s.batch), fblock(kFinThreads);
    score_finalize_kernel<<<fgrid, fblock, (size_t)s.n_q_heads * sizeof(float), stream>>>(
        s.bv, s.n_q_heads, s.kv.n_kv_heads, logits, pitch, part_ml, nsplit, scores, lse, img_mass ? mass_part : nullptr);
    if (img_mass) mass_reduce_kernel<<<s.batch, 64, 0, stream>>>(mass_part, nblk, img_mass);
    timer_end(K_SCORE_FINALIZE, stream);
    return hipGetLastError();
}

}  // namespace fastocr
