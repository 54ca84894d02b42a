// Low-bit scoring of the two query rows of one query head per KV head (Appendix A "Decoding":
// A = Q K^T on the low-bit keys C' for the output token's and the speculative token's rows;
// Section 3.3) with the integer matrix cores.
//
// logit[r][i] = sum_c code[i][c] * x[r][j][c]  +  sum_c sm_scale q[r][c] z[j][c],
//               x[r][j][c] = sm_scale q[r][c] s[j][c],  j = i / g (keys are quantised per
//               channel over g tokens: the multipliers x are shared by a token group)
//
// On the vector ALUs this costs one multiply-accumulate per code and row plus a conversion per
// code, and that instruction count, not the 2.25 bits per code that come from HBM, bounds the
// kernel.  Here the first sum is an integer contraction, v_mfma_i32_16x16x64_i8:
//   A = codes: a code dword masked with 0x03030303 << 2h (1-bit: 0x01010101 << h) already is
//       four int8 operands, code or code << 2 (1-bit: code << (h % 4)); five vector
//       instructions turn a dword of 16 codes into the 16 bytes a lane feeds to one MFMA;
//   B = the multipliers of a token group as 32-bit fixed point relative to the largest |x| of
//       the (row, group), cut into its four bytes: column (sub-group, byte p) holds byte p of
//       every channel's multiplier, the low three re-centred to signed (x + 0x808080, then the
//       top bit of each flipped, leaves x = sum_p piece_p 256^p with signed pieces);
//   C = int32; the four byte columns are recombined in fp32, S3 2^24 + S2 2^16 + S1 2^8 + S0,
//       and scaled back.  Products and sums are exact; the only rounding is the truncation of x
//       to 2^-30 (2^-28 for the channels whose codes arrive shifted) of the group's largest
//       multiplier, below the rounding of an fp32 accumulation.
// The packed layout gives a lane the same code dword of four consecutive tokens, and 16 lanes
// of a wave-wide load four 32-token sub-groups; the 16 rows of an MFMA are therefore tokens of
// four different token groups.  The 16 columns take those four groups' multipliers (4 groups
// x 4 bytes), and of each 16 x 16 result only the blocks where row group = column group are
// used: three quarters of the matrix-core work is thrown away, which is cheap (32 MFMAs per
// 128 tokens) next to what the vector ALUs no longer do.
// A workgroup of four independent waves takes a 512-token tile, a wave 128 tokens of it with
// all channels.  Per wave: lane (sub-group, u) folds the multipliers of 8 channels for both
// rows, the 16 lanes of a sub-group agree on the largest |x| and the zero-point sum with DPP
// steps, bytes are transposed with v_perm_b32 and handed to the lanes that own the B columns
// through a wave-private LDS area; after the MFMAs the used blocks cross the same area once
// more so that every lane finishes four consecutive tokens of one row (16-byte stores).
// Measured on MI355X at 32 heads x 32768 keys, 2-bit codes: 13.4 us per launch (3.8 TB/s of
// packed keys and metadata; 4.7 TB/s counting the fp32 logits and keys it writes) against
// 19.0 us for the vector-ALU kernel, with 4.4 M instead of 8.4 M vector instructions.  The
// kernel is no longer bound by instruction issue: taking out the fold or the MFMAs does not
// change its time, taking out the code loads or the stores does (-1.9 and -2.3 us), an empty
// kernel of the same grid takes 4.5 us.  What helped on the way: accumulators of one token at
// a time, so that a wave fits 64 registers and all eight waves a SIMD gets are resident at
// once (14.8 us with four resident waves, 14.0 with six, 13.4 with eight).  What did not:
// waves that walk several tiles with the next tile's loads in flight (15.4 - 18.3 us: fewer
// waves, more registers), padding against LDS bank conflicts, and leaving out the key array
// (ArgTopK ranking the logits costs it more than the store saves here).
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kPieceStride = 36;                          // dwords: 32 channel quads of one byte plane + pad
constexpr int kSubStride = 2 * 4 * kPieceStride + 8;      // dwords: [row][byte plane] of one sub-group + pad
constexpr int kWaveDwords = 4 * kSubStride;
constexpr int kResBlock = 64 + 4;                         // dwords between the result blocks of (sub-group, row, half)
static_assert(kWaveDwords >= 16 * kResBlock, "the result exchange reuses the multiplier area");

// lane exchange patterns inside a row of 16 lanes
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
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

__device__ __forceinline__ uint32_t comp(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// bytes p = 0..3 of four 32-bit words, gathered per byte position: out[p] = (y0.p, y1.p, y2.p, y3.p)
__device__ __forceinline__ void byte_planes(uint32_t y0, uint32_t y1, uint32_t y2, uint32_t y3, uint32_t out[4]) {
    const uint32_t a_lo = __builtin_amdgcn_perm(y1, y0, 0x05010400u), a_hi = __builtin_amdgcn_perm(y1, y0, 0x07030602u);
    const uint32_t b_lo = __builtin_amdgcn_perm(y3, y2, 0x05010400u), b_hi = __builtin_amdgcn_perm(y3, y2, 0x07030602u);
    out[0] = __builtin_amdgcn_perm(b_lo, a_lo, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(b_lo, a_lo, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(b_hi, a_hi, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(b_hi, a_hi, 0x07060302u);
}

template <int BITS, bool BF16>
// at most 64 registers: all eight waves a SIMD gets are resident at once
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(8, 8))) void score_i8_kernel(LayerView L, const uint16_t* __restrict__ q, int Nq,
                                                               float sm_scale, float* __restrict__ logits,
                                                               size_t logit_stride, uint32_t* __restrict__ keys,
                                                               size_t key_stride) {
    constexpr int NW = 4 * BITS;               // code dwords per token
    constexpr int LD = NW / 4;                 // code dwords a lane quarter loads per token: 2 (2-bit) or 1 (1-bit)
    __shared__ __attribute__((aligned(16))) uint32_t xch[kWaves][kWaveDwords];
    __shared__ __attribute__((aligned(8))) float2 fin[kWaves][4][2];   // (scale back, zero-point sum) per (sub-group, row)

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.y, tile = blockIdx.x;
    if (append_tail_block(L, row)) return;   // the extra workgroup of a fused append
    const int n_sub = Nq / kBlockTokens;                       // quantised 32-token sub-groups
    const int sub0 = tile * 16 + 4 * wave;                     // this wave's first sub-group
    if (sub0 >= n_sub) return;                                 // the waves never meet at a barrier

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
                const uint32_t pair = comp(qraw[r], e / 2);
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
    uint32_t* area = xch[wave];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const float top = row16_max(mx[r]);
        qz[r] = row16_sum(qz[r]);
        // top < 2^(E - 126) with E its exponent field: x * 2^(156 - E) stays below 2^30
        uint32_t E = __float_as_uint(top) >> 23;
        E = E < 30u ? 30u : (E > 254u ? 254u : E);
        const float up = __uint_as_float((283u - E) << 23);
        if (u == 0) fin[wave][sgP][r] = make_float2(__uint_as_float((E - 29u) << 23), qz[r]);
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
                    const uint32_t w = comp(cw[ks][hf], j), t = w >> 4;
                    a = (v4i){(int)(w & 0x03030303u), (int)(w & 0x0C0C0C0Cu), (int)(t & 0x03030303u), (int)(t & 0x0C0C0C0Cu)};
                } else {
                    const uint32_t t = comp(cw[0][hf], j) >> (4 * ks);
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
    const float2 f = fin[wave][sgO][rO];
    float o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float t = __builtin_fmaf((float)s[1][j], 256.0f, (float)s[0][j]);
        t = __builtin_fmaf((float)s[2][j], 65536.0f, t);
        t = __builtin_fmaf((float)s[3][j], 16777216.0f, t);
        o[j] = __builtin_fmaf(t, f.x, f.y);
    }
    if (sub0 + sgO < n_sub) {
        const size_t i4 = (size_t)(sub0 + sgO) * kBlockTokens + 8 * vO + 4 * hfO;
        *reinterpret_cast<float4*>(logits + ((size_t)row * 2 + rO) * logit_stride + i4) = make_float4(o[0], o[1], o[2], o[3]);
        if (rO == 1)   // the speculative row ranks the positions
            *reinterpret_cast<uint4*>(keys + (size_t)row * key_stride + i4) =
                make_uint4(float_to_key(o[0]), float_to_key(o[1]), float_to_key(o[2]), float_to_key(o[3]));
    }
}

}  // namespace

bool score_uses_int8_matrix_cores(int G, int n_rows) { return G == 1 && n_rows == 2; }

hipError_t launch_score_i8(const LayerView& L, const void* q, int Nq, float sm_scale, float* logits,
                           size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (L.G != 1 || (L.bits != 1 && L.bits != 2) || (L.group != 32 && L.group != 64 && L.group != 128) || Nq % L.group != 0)
        return hipErrorInvalidValue;
    const dim3 grid((Nq + kTileTokens - 1) / kTileTokens + (L.tail_k ? 1 : 0), L.rows), block(64 * kWaves);
#define SPC_I8(B_, F_)                                                                                         \
    SPC_LAUNCH((score_i8_kernel<B_, F_>), grid, block, stream, L, (const uint16_t*)q, Nq, sm_scale, logits, \
               logit_stride, keys, key_stride)
    if (L.bits == 2) { if (L.bf16) SPC_I8(2, true); else SPC_I8(2, false); }
    else             { if (L.bf16) SPC_I8(1, true); else SPC_I8(1, false); }
#undef SPC_I8
    return hipGetLastError();
}

}  // namespace specache
