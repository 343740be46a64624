// Plain streaming kernels of known size: the measured HBM ceiling next to the attention
// kernels, and the reference that calibrates the profiler's fetch/write byte counters.
#include "kernels.hpp"

namespace fastocr {

__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4 *__restrict__ src,
                                                           u32x4 *__restrict__ dst, size_t n16,
                                                           uint32_t *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        if (dst) { dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d; }
        else acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) {
        const u32x4 a = src[i];
        if (dst) dst[i] = a;
        else acc ^= a;
    }
    // keeps the read-only variant's loads alive; the value is never expected to match
    if (!dst && (acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && sink) sink[0] = acc[0];
}

hipError_t launch_stream_probe(const void *src, void *dst, size_t bytes, void *sink, hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    stream_probe_kernel<<<256 * 8, 256, 0, stream>>>(reinterpret_cast<const u32x4 *>(src),
                                                     reinterpret_cast<u32x4 *>(dst), n16,
                                                     reinterpret_cast<uint32_t *>(sink));
    return hipGetLastError();
}

}  // namespace fastocr
