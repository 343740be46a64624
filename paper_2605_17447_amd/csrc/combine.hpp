// Merge of attention partials spread over a workgroup's threads, as a device function: the merge kernel
// of attn.hip is this body, and so are the extra workgroups of the launch that runs a focal layer's
// top-k (topk.hip) -- the two depend only on the one-pass kernel before them, so they share a launch.
#pragma once
#include "common.hpp"

namespace fastocr {

constexpr int kCombineFew = 32;        // up to this many partials per head the merge takes its one-round-trip form

struct CombineShared {
    float *max4;        // [4]
    float *z;           // [256]
    float *o;           // [1024], 16-byte aligned: [split lane][d], SL * d <= 1024 as DL >= d/4
};

// out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) Z_s for head h of sequence b (head_dim a multiple
// of 4, at most 256).  Threads 0 .. 255 of the workgroup work -- a thread is (split lane, dim lane): it
// walks every SL-th partial with 16-byte loads, four of them in flight, and the split lanes are then
// added through LDS in a fixed order (a serial walk is bound by memory latency once a head has more
// than a handful of partials) -- but every thread of the workgroup must call: there are workgroup
// barriers inside.  seq_meta: the partials of sequence b are those of workgroups seq_meta[2b] ..
// + seq_meta[2b+1] of the one-pass focal kernel, wpk partials each.
template <typename T>
__device__ __forceinline__ void combine_wide_body(const float *__restrict__ part_o, const float *__restrict__ part_ml, int nsplit, int d,
                                                  T *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ seq_meta,
                                                  int wpk, int h, int b, int Hq, const CombineShared &sh)
{
    float *sm_max = sh.max4, *sm_z = sh.z, *sm_o = sh.o;
    const int64_t bh = (int64_t)b * Hq + h;
    const int t = threadIdx.x;
    const bool works = t < 256;
    // partial s of this head: statistics at ml[s * ml_step], accumulator at po[s * o_step]
    const float *ml = part_ml + bh * nsplit * 2;
    const float *pbase = part_o + bh * nsplit * d;
    int64_t ml_step = 2, o_step = d;
    if (seq_meta) {
        const int64_t first = (int64_t)seq_meta[2 * b] * wpk;
        nsplit = seq_meta[2 * b + 1] * wpk;
        ml = part_ml + (first * Hq + h) * 2;
        pbase = part_o + (first * Hq + h) * d;
        ml_step = 2 * (int64_t)Hq;
        o_step = (int64_t)Hq * d;
    }
    // dim lanes: the power of two covering d/4 (1 .. 64); split lanes: the rest of the 256 threads
    const int nd4 = d / 4;
    int DL = 1;
    while (DL < nd4) DL <<= 1;
    const int SL = 256 / DL;
    const int dl = t & (DL - 1), sl = t / DL;
    const bool live = works && dl < nd4;          // this thread holds a (split lane, dim lane) of the merge

    float Z = 0.f, M;
    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
    if (nsplit <= kCombineFew && nsplit <= 4 * SL) {
        // A handful of partials (a short list cut fine): one memory round trip instead of two.  The
        // thread's (at most four) accumulators are requested first, from clamped addresses; then every
        // thread reads all the maxima itself -- the same addresses across the workgroup, requests that
        // travel together with the others -- instead of waiting for a reduction through LDS.
        f32x4 a[4];
        float mm[4], zz[4];
        const int dc = dl < nd4 ? dl : nd4 - 1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int sk = sl + k * SL < nsplit ? sl + k * SL : 0;
            a[k] = *reinterpret_cast<const f32x4 *>(pbase + 4 * dc + sk * o_step);
            mm[k] = ml[sk * ml_step];
            zz[k] = ml[sk * ml_step + 1];
        }
        M = -INFINITY;
        for (int x = 0; x < nsplit; ++x) M = fmaxf(M, ml[x * ml_step]);
        if (M > -INFINITY && live) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (sl + k * SL < nsplit) {
                    const float f = fast_exp2(mm[k] - M);
                    Z += f * zz[k];
                    o += a[k] * f;
                }
            }
        }
    } else {
        float mloc = -INFINITY;
        if (works)
            for (int s = t; s < nsplit; s += 256) mloc = fmaxf(mloc, ml[s * ml_step]);
        mloc = wave_max(mloc);
        if (works && (t & 63) == 0) sm_max[t >> 6] = mloc;
        __syncthreads();
        M = fmaxf(fmaxf(sm_max[0], sm_max[1]), fmaxf(sm_max[2], sm_max[3]));
        if (M > -INFINITY && live) {
            const float *po = pbase + 4 * dl;
#pragma unroll 4
            for (int s = sl; s < nsplit; s += SL) {
                const float f = fast_exp2(ml[s * ml_step] - M);
                Z += f * ml[s * ml_step + 1];
                const f32x4 a = *reinterpret_cast<const f32x4 *>(po + s * o_step);
                o += a * f;
            }
        }
    }
    if (live) *reinterpret_cast<f32x4 *>(&sm_o[sl * d + 4 * dl]) = o;
    if (works && dl == 0) sm_z[sl] = Z;
    __syncthreads();
    if (t < d) {
        float acc = 0.f, zt = 0.f;
        for (int x = 0; x < SL; ++x) { acc += sm_o[x * d + t]; zt += sm_z[x]; }
        store_elem<T>(out + bh * d + t, zt > 0.f ? acc / zt : 0.f);
        if (lse && t == 0) lse[bh] = zt > 0.f ? (M + log2f(zt)) * kLn2 : -INFINITY;
    }

}

}  // namespace fastocr
