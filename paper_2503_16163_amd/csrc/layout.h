// Device data layout of the low-bit cache C' and helpers shared by the kernels.
//
// All sizes are per (batch, KV head) "row" of a layer; head_dim D = 128.
//
// K codes (keys are grouped per channel over g tokens; Section 2.1 / 4.1):
//   tiles of 512 tokens = 16 sub-groups of 32 tokens.  A token's 128 codes occupy
//   4*BITS dwords; dword W holds the 32/BITS channels c with c / (32/BITS) == W.  A tile
//   is laid out as [dword W][2 halves][64 lanes][16 bytes]: lane = 4*G + k for sub-group
//   G and quad lane k, and the lane's 16 bytes in half hf are dword W of its tokens
//   32*G + 8*k + 4*hf + {0,1,2,3}.  The scoring wave owns a tile and walks W: each lane
//   scores the 8 consecutive tokens 8*k .. 8*k+7 of one sub-group, every load is 1 KB
//   contiguous across the wave, and the four lanes of a quad share one group's
//   multipliers.  Inside a dword the code of channel c sits at bit
//   8*(w % 4) + BITS*(w / 4), w = c % (32/BITS): masking with
//   (2^BITS - 1) * 0x01010101 << BITS*h leaves four codes, one per byte, each scaled by
//   2^(BITS*h); v_cvt_f32_ubyte{0..3} turns them into floats and the power of two is
//   folded into the multiplier.  Byte b of that mask is channel 4*h + b of the dword,
//   i.e. channel % 4 == b.
// K metadata: per token group j, 128 dwords = min | max << 16 (16-bit patterns of the
//   cache dtype), stored as [channel % 4][channel / 4] so that the quad lane k = c % 4
//   reads the channels it multiplies as consecutive dwords; scale and zero-point are
//   derived on use.
// V codes (values are grouped per token over g channels):
//   blocks of 32 tokens, each block = [2 halves of 16 tokens][16*BITS lanes][16 B];
//   byte t of a lane's 16 bytes is token 16*half + t and holds the 8/BITS
//   channels c with c / (8/BITS) == lane, channel c at bit BITS * (c % (8/BITS)).
//   The same mask-and-convert form then yields four tokens of one channel.
// V metadata: [token][channel group m] one dword = min | max << 16.
// Residual ring, staging slots and the pinned host store share one row format:
//   512 bytes per token = K row (128 x 16 bit) then V row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specache {

constexpr int kD = 128;          // head_dim
constexpr int kRowBytes = 512;   // one 16-bit (K,V) pair
constexpr int kBlockTokens = 32; // tokens per V code block / per K sub-group
constexpr int kTileTokens = 512; // tokens per K code tile

__host__ __device__ constexpr int code_block_bytes(int bits) { return 512 * bits; }
__host__ __device__ constexpr int k_tile_bytes(int bits) { return kTileTokens * 16 * bits; }

// ---- 16-bit -> float, exact --------------------------------------------------
template <bool BF16>
__device__ __forceinline__ float widen16(uint32_t bits16) {
    if constexpr (BF16) {
        return __uint_as_float(bits16 << 16);
    } else {
        _Float16 h;
        uint16_t u = (uint16_t)bits16;
        __builtin_memcpy(&h, &u, 2);
        return (float)h;
    }
}

// ---- Eq. 2 / Eq. 3: scale and zero-point from the stored (min, max) -----------
// Every step is a single IEEE binary32 operation (no contraction): the integer
// codes depend on it.
// plain_one_bit selects, for BITS == 1, the unmodified form (Eq. 2 with B = 1: z = min,
// s = max - min; the "original" 1-bit KIVI of Section 4.4 / Table 5) instead of Eq. 3.
template <int BITS>
__device__ __forceinline__ void derive_scale_zero(float mn, float mx, bool plain_one_bit, float& s, float& z) {
    const float range = __fsub_rn(mx, mn);
    if constexpr (BITS == 1) {
        const float z3 = __fmul_rn(__fadd_rn(__fmul_rn(3.0f, mn), mx), 0.25f);
        z = plain_one_bit ? mn : z3;
        s = plain_one_bit ? range : __fmul_rn(range, 0.5f);
    } else {
        constexpr float cB = (float)(1.0 / (double)((1 << BITS) - 1));
        z = mn;
        s = __fmul_rn(range, cB);
    }
}

template <int BITS>
__device__ __forceinline__ uint32_t quantize_one(float x, float s, float z) {
    if (s == 0.0f) return 0u;
    const float t = __fdiv_rn(__fsub_rn(x, z), s);
    const float r = floorf(__fadd_rn(t, 0.5f));
    int c = (int)r;
    c = c < 0 ? 0 : c;
    c = c > ((1 << BITS) - 1) ? ((1 << BITS) - 1) : c;
    return (uint32_t)c;
}

// ---- K code addressing ---------------------------------------------------------
template <int BITS>
__host__ __device__ __forceinline__ int k_dword_of_channel(int c) { return c / (32 / BITS); }
template <int BITS>
__host__ __device__ __forceinline__ int k_bit_of_channel(int c) {
    const int w = c % (32 / BITS);
    return 8 * (w % 4) + BITS * (w / 4);
}
// byte offset, inside a row's K code area, of dword W of token t
template <int BITS>
__host__ __device__ __forceinline__ size_t k_dword_offset(int t, int W) {
    const int tile = t / kTileTokens, u = t % kTileTokens;
    const int lane = 4 * (u / 32) + (u % 32) / 8, slot = u % 8;
    return (size_t)tile * k_tile_bytes(BITS) + ((size_t)(W * 2 + slot / 4) * 64 + lane) * 16 + (size_t)(slot % 4) * 4;
}
// dword index, inside a token group's 128 metadata dwords, of channel c
__host__ __device__ __forceinline__ int k_meta_index(int c) { return (c % 4) * 32 + c / 4; }

// ---- V code addressing ---------------------------------------------------------
template <int BITS>
__host__ __device__ __forceinline__ int v_lane_of_channel(int c) { return c / (8 / BITS); }
template <int BITS>
__host__ __device__ __forceinline__ int v_bit_of_channel(int c) {
    return BITS * (c % (8 / BITS));
}
// byte offset, inside a row's V code area, of the byte of (token t, lane L)
template <int BITS>
__host__ __device__ __forceinline__ size_t v_byte_offset(int t, int L) {
    const int blk = t / kBlockTokens, tok = t % kBlockTokens, half = tok / 16, tt = tok % 16;
    return (size_t)blk * code_block_bytes(BITS) + ((size_t)half * (16 * BITS) + L) * 16 + tt;
}

// Offload of one new token by the scoring launch's extra workgroup of a row (Appendix A "Decoding":
// the new pair goes to the CPU copy; it also joins the 16-bit residual): 32 lanes x 16 B move the
// 512-byte (K,V) pair.  True when this workgroup was that extra one.
template <typename View>
__device__ __forceinline__ bool append_tail_block(const View& L, int row) {
    if (L.tail_k == nullptr || blockIdx.x != gridDim.x - 1) return false;
    const int part = threadIdx.x;
    if (part < 32) {
        const uint4 v = reinterpret_cast<const uint4*>(part < 16 ? L.tail_k : L.tail_v)[(size_t)row * 16 + (part & 15)];
        const int t = L.tail_N0;
        reinterpret_cast<uint4*>(L.host)[((size_t)row * L.max_seq + t) * 32 + part] = v;
        reinterpret_cast<uint4*>(L.ring)[((size_t)row * L.R + (t % L.R)) * 32 + part] = v;
    }
    return true;
}

// order-preserving map float -> uint32 (larger float <=> larger key); -0 joins +0
__device__ __forceinline__ uint32_t float_to_key(float f) {
    const uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace specache
