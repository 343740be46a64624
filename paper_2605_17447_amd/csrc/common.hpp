// Shared device-side plumbing of the FastOCR HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fastocr {

// Kernel-side copies of the C-ABI views (plain data, passed by value).
struct KvDev {
    const void *k;
    const void *v;
    int64_t stride_token, stride_head, stride_seq, stride_page;   // elements
    const int32_t *block_table;
    int32_t max_pages, page_tokens;
    int32_t n_kv_heads, head_dim;
};

struct BatchDev {
    const int32_t *seq_len, *vis_start, *vis_len;
    int32_t max_seq_len, max_vis_len;
};

// Sequence geometry, clamped to the host-side bounds the grids and workspaces were sized
// with, so that a bad device-side length can never drive a read or write out of range.
struct SeqGeom {
    int S;    // tokens in the sequence
    int v0;   // first image token
    int N;    // image tokens
};

// from the three per-sequence entries as loaded (clamped into what the batch's maxima allow)
__device__ __forceinline__ SeqGeom seq_geom_of(const BatchDev &bv, int seq_len, int vis_start, int vis_len)
{
    SeqGeom g;
    g.S = min(max(seq_len, 0), bv.max_seq_len);
    g.v0 = min(max(vis_start, 0), g.S);
    g.N = min(min(max(vis_len, 0), g.S - g.v0), bv.max_vis_len);
    return g;
}

__device__ __forceinline__ SeqGeom seq_geom(const BatchDev &bv, int b)
{
    return seq_geom_of(bv, bv.seq_len[b], bv.vis_start[b], bv.vis_len[b]);
}

// Element offset of (sequence b, token j, kv head g, component 0).
template <bool PAGED>
__device__ __forceinline__ int64_t row_offset(const KvDev &kv, int b, int j, int g)
{
    if (PAGED) {
        int pg = j / kv.page_tokens;
        int in = j - pg * kv.page_tokens;
        pg = min(pg, kv.max_pages - 1);
        int64_t page = kv.block_table[(int64_t)b * kv.max_pages + pg];
        return page * kv.stride_page + (int64_t)in * kv.stride_token + (int64_t)g * kv.stride_head;
    }
    return (int64_t)b * kv.stride_seq + (int64_t)j * kv.stride_token + (int64_t)g * kv.stride_head;
}

// Position p of the attended list -> token index of the sequence.
//   dense : identity.
//   gather: [text before the span][selected image tokens][text after the span]
template <bool GATHER>
__device__ __forceinline__ int pos_to_token(int p, const SeqGeom &g, int cnt, const int32_t *sel)
{
    if (!GATHER) return p;
    // The index is loaded unconditionally (slot clamped into the row, which always holds at
    // least one entry) and the case is chosen arithmetically: a load inside a branch would make
    // the compiler drain every outstanding prefetch at the join.
    const int slot = min(max(p - g.v0, 0), max(cnt - 1, 0));
    int i = sel[slot];
    i = min(max(i, 0), max(g.N - 1, 0));
    const int mid = g.v0 + i;
    const int tail = p - cnt + g.N;
    return (p < g.v0) ? p : ((p < g.v0 + cnt) ? mid : tail);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b)
{
    return __uint_as_float(((uint32_t)b) << 16);
}

// round-to-nearest-even fp32 -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_elem(const T *p);
template <> __device__ __forceinline__ float load_elem<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_elem<uint16_t>(const uint16_t *p) { return bf16_bits_to_f32(*p); }

template <typename T> __device__ __forceinline__ void store_elem(T *p, float x);
template <> __device__ __forceinline__ void store_elem<float>(float *p, float x) { *p = x; }
template <> __device__ __forceinline__ void store_elem<uint16_t>(uint16_t *p, float x) { *p = f32_to_bf16_bits(x); }

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (shifts
// within rows of 16 lanes, then the last lane of a row broadcast into the following rows): six
// full-rate VALU additions instead of six round trips through the LDS crossbar.
__device__ __forceinline__ int wave_scan_incl(int x)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);      // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);      // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);      // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);      // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);      // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);      // row_bcast:31 into rows 2 and 3
    return x;
}

// A lane's value together with that of the lane 16 (32) away, for commutative reductions: gfx950 swaps
// rows of 16 lanes (halves of 32) between two registers in one VALU instruction, where a general
// lane permute is a trip through the LDS crossbar.  Of the two results one is the lane's own value and
// the other its partner's (which is which depends on the lane's row, and does not matter to op).
template <typename Op>
__device__ __forceinline__ float with_lane_xor16(float x, Op op)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return op(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
template <typename Op>
__device__ __forceinline__ float with_lane_xor32(float x, Op op)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return op(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
// max / sum over the lanes that differ in bits 4 and 5 of the lane number (the four rows of a wave)
__device__ __forceinline__ float rows_max(float x)
{
    auto mx = [](float a, float b) { return fmaxf(a, b); };
    return with_lane_xor32(with_lane_xor16(x, mx), mx);
}
__device__ __forceinline__ float rows_sum(float x)
{
    auto add = [](float a, float b) { return a + b; };
    return with_lane_xor32(with_lane_xor16(x, add), add);
}

// exp2 with exp2(-inf) = 0 and no NaN for (-inf) - (-inf) handled by the callers
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// <q, row> over d components, accumulated in fp64: a product of two fp32 (or bf16) values is exact in
// double and the sum of up to 256 of them carries a relative error near 2^-53, so the logit is
// the exactly rounded one whichever way the row is fetched.  (A single fp32 chain over d left the
// logit off by about sqrt(d) 2^-24 of the largest partial sum, which is the relative error of the
// token's weight: 1.2e-5 on logits near 30.)  vec16: the row starts 16-byte aligned and d covers
// whole 16-byte pieces, so it is fetched 16 bytes per load instead of one element per load.
template <typename T>
__device__ __forceinline__ double dot_row(const float *__restrict__ qs, const T *__restrict__ row, int d, bool vec16)
{
    double s = 0.0;
    if (vec16) {
        constexpr int E = 16 / (int)sizeof(T);
        for (int c = 0; c < d; c += E) {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(row + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (sizeof(T) == 2) {
                    s = fma((double)qs[c + 2 * e], (double)__uint_as_float(w[e] << 16), s);
                    s = fma((double)qs[c + 2 * e + 1], (double)__uint_as_float(w[e] & 0xffff0000u), s);
                } else {
                    s = fma((double)qs[c + e], (double)__uint_as_float(w[e]), s);
                }
            }
        }
    } else {
        for (int c = 0; c < d; ++c) s = fma((double)qs[c], (double)load_elem<T>(row + c), s);
    }
    return s;
}

// LDS traffic of one wave executes in order; this only stops the compiler from moving the reads
// of other lanes' data above the writes that produce it.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// K and V are read once per call: non-temporal loads stream measurably faster on this chip and
// keep the cache lines that are reused (queries, indices, partials, parked logits) in place.
__device__ __forceinline__ u32x4 stream_load(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// Finite stand-in for "no logit yet": keeps 2^(m - m') free of inf - inf.
constexpr float kMinusHuge = -1.0e30f;

// (max, sum-exp) of two disjoint sets of base-2 logits -> of their union
__device__ __forceinline__ void softmax_merge(float &m, float &z, float mo, float zo)
{
    const float M = fmaxf(m, mo);
    z = z * fast_exp2(m - M) + zo * fast_exp2(mo - M);
    m = M;
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Workspace layout helpers shared by host and device code -------------------------------

// logits are parked with a row pitch that is a multiple of 64 tokens
__host__ __device__ inline int64_t logit_pitch(int max_seq_len) { return ((int64_t)max_seq_len + 63) / 64 * 64; }

}  // namespace fastocr
