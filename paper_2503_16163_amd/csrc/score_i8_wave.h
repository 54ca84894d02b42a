// The scoring of one wave's 128 tokens on the integer matrix cores (see score_i8.hip for the
// formulation): shared by the scoring kernel and by the kernel that scores and attends in one pass.
#pragma once
#include "kernels.h"
#include "layout.h"
#include "wave_ops.h"

namespace specache {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kI8Waves = 4;
constexpr int kPieceStride = 36;                          // dwords: 32 channel quads of one byte plane + pad
constexpr int kSubStride = 2 * 4 * kPieceStride + 8;      // dwords: [row][byte plane] of one sub-group + pad
constexpr int kWaveDwords = 4 * kSubStride;
constexpr int kResBlock = 64 + 4;                         // dwords between the result blocks of (sub-group, row, half)
static_assert(kWaveDwords >= 16 * kResBlock, "the result exchange reuses the multiplier area");

__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    return fmaxf(v, dpp_move<kDppMirror>(v));
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    return v + dpp_move<kDppMirror>(v);
}

__device__ __forceinline__ uint32_t comp_i8(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// Logits of the two query rows for the 128 tokens of wave `wave` of tile `tile` of a row (sub0 = 16 tile +
// 4 wave < n_sub sub-groups of 32 quantised tokens).  area: kWaveDwords dwords of LDS private to the wave;
// fin: [4 sub-groups][2 rows] (scale back, zero-point sum), private to the wave.  On return lane
// (sub-group sgO = lane / 16, row rO = (lane / 8) % 2, quad = lane % 8) holds in o[0..3] the logits of row rO
// for tokens 32 (sub0 + sgO) + 4 quad .. + 3; sub-groups at or beyond n_sub hold copies of the last one.
// Two hooks for a caller with work of its own to interleave: loaded() is called once the wave's loads are
// requested (work that waits for earlier loads of the caller fits there), between() once the multipliers are
// built and read back, before the contraction (loads requested there travel while the matrix cores work).
struct NoHook { __device__ void operator()() const {} };
template <int BITS, bool BF16, typename Loaded = NoHook, typename Between = NoHook>
__device__ __forceinline__ void score_i8_wave(const LayerView& L, const uint16_t* __restrict__ q, int row, int tile, int wave,
                                              int lane, int n_sub, float sm_scale, uint32_t* area, float2 (*fin_w)[2],
                                              float o[4], Loaded&& loaded = Loaded(), Between&& between = Between()) {
    constexpr int NW = 4 * BITS;               // code dwords per token
    constexpr int LD = NW / 4;                 // code dwords a lane quarter loads per token: 2 (2-bit) or 1 (1-bit)
    const int sub0 = tile * 16 + 4 * wave;     // this wave's first sub-group
    // ---- code dwords, requested first -----------------------------------------------------
    // lane = (MFMA row rA, channel quarter qd); row rA is layout lane 16 wave + rA of the tile.
    const int rA = lane & 15, qd = lane >> 4;
    int lam = 16 * wave + rA;
    if (tile * 16 + lam / 4 >= n_sub) lam = ((n_sub - 1) % 16) * 4 + (lam & 3);   // past the end: a valid sub-group again
    const uint8_t* kc_lane = L.kc + (size_t)row * L.kc_stride + (size_t)tile * k_tile_bytes(BITS) + (size_t)lam * 16;
    uint4 cw[LD][2];
#pragma unroll
    for (int i = 0; i < LD; ++i)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
            cw[i][hf] = *reinterpret_cast<const uint4*>(kc_lane + (size_t)((4 * i + qd) * 2 + hf) * 1024);

    // ---- multipliers: lane (sub-group sgP, u) folds channel quads 2u and 2u + 1 of that sub-group
    const int sgP = lane >> 4, u = lane & 15;
    const int subP = sub0 + sgP < n_sub ? sub0 + sgP : n_sub - 1;
    const int group_of_sub = subP * kBlockTokens / L.group;     // the sub-groups of one token group share its metadata
    const uint32_t* km_p = L.km + (size_t)row * L.km_stride + (size_t)group_of_sub * kD + 2 * u;
    uint2 mt[4];                                               // (min, max) of channels 4 (2u + mq) + b, mq = .x/.y
#pragma unroll
    for (int b = 0; b < 4; ++b) mt[b] = *reinterpret_cast<const uint2*>(km_p + b * 32);
    uint4 qraw[2];                                             // channels 8u .. 8u + 7 of both rows
#pragma unroll
    for (int r = 0; r < 2; ++r) qraw[r] = *reinterpret_cast<const uint4*>(q + ((size_t)row * 2 + r) * kD + 8 * u);

    loaded();

    float x[2][8], qz[2] = {0.0f, 0.0f}, mx[2] = {0.0f, 0.0f};
#pragma unroll
    for (int mq = 0; mq < 2; ++mq)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t m = mq ? mt[b].y : mt[b].x;
            float sc, z;
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), L.one_bit_plain, sc, z);
            const int e = 4 * mq + b;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const uint32_t pair = comp_i8(qraw[r], e / 2);
                const float qv = widen16<BF16>((e & 1) ? pair >> 16 : pair & 0xFFFFu) * sm_scale;
                x[r][e] = qv * sc;
                qz[r] = __builtin_fmaf(qv, z, qz[r]);
                mx[r] = fmaxf(mx[r], fabsf(x[r][e]));
            }
        }
    // the factor by which the codes of a channel quad arrive multiplied: 4^(quad % 2) for 2-bit
    // codes, 2^(quad % 4) for 1-bit codes
    float cls[2];
    if constexpr (BITS == 2) {
        cls[0] = 1.0f;
        cls[1] = 0.25f;
    } else {
        cls[0] = (u & 1) ? 0.25f : 1.0f;
        cls[1] = (u & 1) ? 0.125f : 0.5f;
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const float top = row16_max(mx[r]);
        qz[r] = row16_sum(qz[r]);
        // top < 2^(E - 126) with E its exponent field: x * 2^(156 - E) stays below 2^30
        uint32_t E = __float_as_uint(top) >> 23;
        E = E < 30u ? 30u : (E > 254u ? 254u : E);
        const float up = __uint_as_float((283u - E) << 23);
        if (u == 0) fin_w[sgP][r] = make_float2(__uint_as_float((E - 29u) << 23), qz[r]);
        const float up_c[2] = {up * cls[0], up * cls[1]};
#pragma unroll
        for (int mq = 0; mq < 2; ++mq) {
            uint32_t y[4], planes[4];
#pragma unroll
            for (int b = 0; b < 4; ++b)
                y[b] = ((uint32_t)(int)(x[r][4 * mq + b] * up_c[mq]) + 0x00808080u) ^ 0x00808080u;
            byte_planes(y[0], y[1], y[2], y[3], planes);
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) area[sgP * kSubStride + (r * 4 + pp) * kPieceStride + 2 * u + mq] = planes[pp];
        }
    }
    // The lanes of a wave run in lockstep and LDS serves one wave's accesses in order: a
    // wave-level fence is all the exchange needs.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // B operands of this lane: column (sub-group sgB, byte p), channel quarter qd; the 16 k-slots
    // of step ks are channel quads m0 .. m0 + 3 in the order the masked code bytes have
    const int sgB = (lane & 15) >> 2, p = lane & 3;
    v4i bop[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int m0 = BITS == 2 ? 16 * ks + 4 * qd : 8 * qd + 4 * ks;
#pragma unroll
        for (int r = 0; r < 2; ++r)
            bop[ks][r] = *reinterpret_cast<const v4i*>(area + sgB * kSubStride + (r * 4 + p) * kPieceStride + m0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();                 // every lane has read its B operands: the area is free
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    between();

    // ---- the contraction: per token (half hf, j of the lane's four) two k-steps, two rows.
    // Result register v of lane (column n, quarter qq) is MFMA row 4 qq + v: sub-group qq of the
    // wave, quad lane v, i.e. token 32 (sub0 + qq) + 8 v + 4 hf + j.  It is wanted where the
    // column's sub-group is qq too; those quads go to block (sub-group, row, hf) of the area as
    // [byte p][token j][quad lane v], the blocks 4 dwords further apart than their size so that
    // the lanes that read one position of 16 different blocks hit 16 different banks.
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4i acc[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                v4i a;
                if constexpr (BITS == 2) {
                    const uint32_t w = comp_i8(cw[ks][hf], j), t = w >> 4;
                    a = (v4i){(int)(w & 0x03030303u), (int)(w & 0x0C0C0C0Cu), (int)(t & 0x03030303u), (int)(t & 0x0C0C0C0Cu)};
                } else {
                    const uint32_t t = comp_i8(cw[0][hf], j) >> (4 * ks);
                    a = (v4i){(int)(t & 0x01010101u), (int)(t & 0x02020202u), (int)(t & 0x04040404u), (int)(t & 0x08080808u)};
                }
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    acc[r] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bop[ks][r], ks == 0 ? (v4i){0, 0, 0, 0} : acc[r], 0, 0, 0);
            }
            if (sgB == qd) {
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    *reinterpret_cast<v4i*>(area + ((qd * 2 + r) * 2 + hf) * kResBlock + (p * 4 + j) * 4) = acc[r];
            }
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- every lane finishes four consecutive tokens of one row: lane = (sub-group sgO, row rO,
    // ---- quad lane vO, half hfO), 8 lanes cover the 32 tokens of a sub-group in order
    const int sgO = lane >> 4, rO = (lane >> 3) & 1, vO = (lane >> 1) & 3, hfO = lane & 1;
    int s[4][4];   // [byte p][token j]
    const uint32_t* blk = area + ((sgO * 2 + rO) * 2 + hfO) * kResBlock + vO;
#pragma unroll
    for (int pp = 0; pp < 4; ++pp)
#pragma unroll
        for (int j = 0; j < 4; ++j) s[pp][j] = (int)blk[(pp * 4 + j) * 4];
    const float2 f = fin_w[sgO][rO];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float t = __builtin_fmaf((float)s[1][j], 256.0f, (float)s[0][j]);
        t = __builtin_fmaf((float)s[2][j], 65536.0f, t);
        t = __builtin_fmaf((float)s[3][j], 16777216.0f, t);
        o[j] = __builtin_fmaf(t, f.x, f.y);
    }
}

}  // namespace
}  // namespace specache
