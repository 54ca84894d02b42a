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
#include "score_i8_wave.h"

namespace specache {
namespace {

constexpr int kWaves = kI8Waves;

template <int BITS, bool BF16>
// at most 64 registers: all eight waves a SIMD gets are resident at once
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(8, 8))) void score_i8_kernel(LayerView L, const uint16_t* __restrict__ q, int Nq,
                                                               float sm_scale, float* __restrict__ logits,
                                                               size_t logit_stride, uint32_t* __restrict__ keys,
                                                               size_t key_stride) {
    __shared__ __attribute__((aligned(16))) uint32_t xch[kWaves][kWaveDwords];
    __shared__ __attribute__((aligned(8))) float2 fin[kWaves][4][2];   // (scale back, zero-point sum) per (sub-group, row)

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.y, tile = blockIdx.x;
    if (append_tail_block(L, row)) return;   // the extra workgroup of a fused append
    const int n_sub = Nq / kBlockTokens;                       // quantised 32-token sub-groups
    const int sub0 = tile * 16 + 4 * wave;                     // this wave's first sub-group
    if (sub0 >= n_sub) return;                                 // the waves never meet at a barrier

    float o[4];
    score_i8_wave<BITS, BF16>(L, q, row, tile, wave, lane, n_sub, sm_scale, xch[wave], fin[wave], o);
    const int sgO = lane >> 4, rO = (lane >> 3) & 1, vO = (lane >> 1) & 3, hfO = lane & 1;
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
