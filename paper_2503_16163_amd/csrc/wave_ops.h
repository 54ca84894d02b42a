// Lane exchanges inside a wave on the vector ALU (DPP) and the byte transposition shared by the
// integer-matrix-core kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specache {
namespace {

// lane exchange patterns inside a row of 16 lanes
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;
constexpr int kDppRowRor8 = 0x128;              // lane i <-> lane i ^ 8 inside a row of 16

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// bytes p = 0..3 of four 32-bit words, gathered per byte position: out[p] = (y0.p, y1.p, y2.p, y3.p)
__device__ __forceinline__ void byte_planes(uint32_t y0, uint32_t y1, uint32_t y2, uint32_t y3, uint32_t out[4]) {
    const uint32_t a_lo = __builtin_amdgcn_perm(y1, y0, 0x05010400u), a_hi = __builtin_amdgcn_perm(y1, y0, 0x07030602u);
    const uint32_t b_lo = __builtin_amdgcn_perm(y3, y2, 0x05010400u), b_hi = __builtin_amdgcn_perm(y3, y2, 0x07030602u);
    out[0] = __builtin_amdgcn_perm(b_lo, a_lo, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(b_lo, a_lo, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(b_hi, a_hi, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(b_hi, a_hi, 0x07060302u);
}

// The lanes of a wave run in lockstep and LDS serves one wave's accesses in order: a wave-level
// fence is all an exchange through a wave-private LDS area needs.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace
}  // namespace specache
