// Pieces shared by the two kernels that keep a focal layer's logits in registers
// (score_resident.hip, focal_fused.hip): geometry constants, the tile-list macro, the
// global -> LDS copy and the cross-lane moves.
#pragma once
#include "kernels.hpp"

namespace fastocr {

constexpr int kResWaves = 8;
constexpr int kResThreads = 64 * kResWaves;
constexpr int kResTmax = 32;          // image tiles per wave held in registers
constexpr int kResTile = 32;
constexpr int kResMaxHq = 64;
constexpr int kResSlots = 32;         // barrier slots: calls that may overlap on one GPU
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
constexpr int kDppRor8 = 0x128;         // lane i <- lane i ^ 8

}  // namespace fastocr
