// Low-bit scoring (Appendix A "Decoding": A = Q K^T on the low-bit keys C', read once
// for the output token's and the speculative token's query rows; Section 3.3).
//
// logit[r][i] = sm_scale * sum_c q[r][c] * (code[i][c] * s[j][c] + z[j][c]),  j = i / g
//             = sum_c (sm_scale q[r][c] s[j][c]) * code[i][c]  +  sum_c sm_scale q[r][c] z[j][c]
// Keys are quantised per channel over g tokens, so the folded multiplier
// qs[r][c] and the constant qz[r] are shared by the g tokens of a group.
//
// Mapping: one lane per token.  A wave covers two 32-token blocks (lanes 0-31 and
// 32-63); each half derives qs for its own group (4 channels per lane), spreads
// it through a wave-private LDS region into "quad layout" (lane l holds channel
// 4v + (l & 3) in register v), and the multiply-accumulate picks the channel
// with a DPP quad broadcast, so the multiplier costs no extra instruction.
// Codes become floats with v_cvt_f32_ubyte{0..3} after one mask per four codes.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

// acc[r] += sum_{b<4} float(byte b of mk) * q[r] read from quad lane b, for RC rows.
// The four conversions lead the block, so that the first DPP read is at least
// four VALU instructions after anything outside the block.
#define SPC_DPP(a, q, f, k) "v_fmac_f32_dpp " a ", " q ", " f " quad_perm:[" k "," k "," k "," k "] row_mask:0xf bank_mask:0xf\n"
#define SPC_CVT                          \
    "v_cvt_f32_ubyte0 %[f0], %[mk]\n"    \
    "v_cvt_f32_ubyte1 %[f1], %[mk]\n"    \
    "v_cvt_f32_ubyte2 %[f2], %[mk]\n"    \
    "v_cvt_f32_ubyte3 %[f3], %[mk]\n"
#define SPC_ROWS1(k, f) SPC_DPP("%[a0]", "%[q0]", f, k)
#define SPC_ROWS2(k, f) SPC_ROWS1(k, f) SPC_DPP("%[a1]", "%[q1]", f, k)
#define SPC_ROWS4(k, f) SPC_ROWS2(k, f) SPC_DPP("%[a2]", "%[q2]", f, k) SPC_DPP("%[a3]", "%[q3]", f, k)
#define SPC_ROWS8(k, f)                                                                            \
    SPC_ROWS4(k, f) SPC_DPP("%[a4]", "%[q4]", f, k) SPC_DPP("%[a5]", "%[q5]", f, k)                 \
    SPC_DPP("%[a6]", "%[q6]", f, k) SPC_DPP("%[a7]", "%[q7]", f, k)
#define SPC_BODY(ROWS) SPC_CVT ROWS("0", "%[f0]") ROWS("1", "%[f1]") ROWS("2", "%[f2]") ROWS("3", "%[f3]")

template <int RC>
__device__ __forceinline__ void fmac_block(float* acc, const float* q, uint32_t mk);

template <>
__device__ __forceinline__ void fmac_block<1>(float* acc, const float* q, uint32_t mk) {
    float f0, f1, f2, f3;
    asm(SPC_BODY(SPC_ROWS1)
        : [a0] "+v"(acc[0]), [f0] "=&v"(f0), [f1] "=&v"(f1), [f2] "=&v"(f2), [f3] "=&v"(f3)
        : [q0] "v"(q[0]), [mk] "v"(mk));
}
template <>
__device__ __forceinline__ void fmac_block<2>(float* acc, const float* q, uint32_t mk) {
    float f0, f1, f2, f3;
    asm(SPC_BODY(SPC_ROWS2)
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [f0] "=&v"(f0), [f1] "=&v"(f1), [f2] "=&v"(f2), [f3] "=&v"(f3)
        : [q0] "v"(q[0]), [q1] "v"(q[1]), [mk] "v"(mk));
}
template <>
__device__ __forceinline__ void fmac_block<4>(float* acc, const float* q, uint32_t mk) {
    float f0, f1, f2, f3;
    asm(SPC_BODY(SPC_ROWS4)
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]), [f0] "=&v"(f0),
          [f1] "=&v"(f1), [f2] "=&v"(f2), [f3] "=&v"(f3)
        : [q0] "v"(q[0]), [q1] "v"(q[1]), [q2] "v"(q[2]), [q3] "v"(q[3]), [mk] "v"(mk));
}
template <>
__device__ __forceinline__ void fmac_block<8>(float* acc, const float* q, uint32_t mk) {
    float f0, f1, f2, f3;
    asm(SPC_BODY(SPC_ROWS8)
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]), [a4] "+v"(acc[4]),
          [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]), [f0] "=&v"(f0), [f1] "=&v"(f1),
          [f2] "=&v"(f2), [f3] "=&v"(f3)
        : [q0] "v"(q[0]), [q1] "v"(q[1]), [q2] "v"(q[2]), [q3] "v"(q[3]), [q4] "v"(q[4]), [q5] "v"(q[5]),
          [q6] "v"(q[6]), [q7] "v"(q[7]), [mk] "v"(mk));
}

__device__ __forceinline__ float comp(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ __forceinline__ uint32_t comp(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

constexpr int kScoreWaves = 4;

template <int BITS, int GROUP, int G, int NROWS, bool BF16>
__global__ __launch_bounds__(64 * kScoreWaves) void score_kernel(LayerView L, const uint16_t* __restrict__ q,
                                                                 int Nq, float sm_scale,
                                                                 float* __restrict__ logits, size_t logit_stride,
                                                                 uint32_t* __restrict__ keys, size_t key_stride,
                                                                 int tiles_per_wave) {
    constexpr int NR = G * NROWS;              // query rows sharing this KV head
    constexpr int RC = NR > 8 ? 8 : NR;        // rows per multiply-accumulate block
    constexpr int HPD = (32 / BITS) / 4;       // masks per dword
    constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x01010101u;
    // +16 floats per half wave: the two halves of a wave read at the same offsets, the pad
    // puts them in different banks
    __shared__ float qs_lds[kScoreWaves][2][NR * kD + 16];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hw = lane >> 5, li = lane & 31;
    const int row = blockIdx.y;
    const int nb = Nq / kBlockTokens;
    const int n_tiles = (nb + 1) / 2;
    const uint8_t* kc_row = L.kc + (size_t)row * L.kc_stride;
    const uint32_t* km_row = L.km + (size_t)row * L.km_stride;

    // this lane's four channels of every query row, pre-scaled by sm_scale
    float qsc[NR][4];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const uint2 qb = *reinterpret_cast<const uint2*>(q + ((size_t)row * NR + r) * kD + 4 * li);
        qsc[r][0] = widen16<BF16>(qb.x & 0xFFFFu) * sm_scale;
        qsc[r][1] = widen16<BF16>(qb.x >> 16) * sm_scale;
        qsc[r][2] = widen16<BF16>(qb.y & 0xFFFFu) * sm_scale;
        qsc[r][3] = widen16<BF16>(qb.y >> 16) * sm_scale;
    }
    // the code of channel c = 4*li + cc arrives scaled by 2^(BITS*h), h = li % HPD
    const float unshift = __uint_as_float((uint32_t)(127 - BITS * (li % HPD)) << 23);

    const int tile0 = (blockIdx.x * kScoreWaves + wave) * tiles_per_wave;
    for (int it = 0; it < tiles_per_wave; ++it) {
        const int tile = tile0 + it;
        if (tile >= n_tiles) break;  // wave-uniform
        const int blk = 2 * tile + hw;
        const bool active = blk < nb;
        const int blk_c = active ? blk : nb - 1;
        const int j = (blk_c * kBlockTokens) / GROUP;

        uint4 cw[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p)
            cw[p] = *reinterpret_cast<const uint4*>(kc_row + (size_t)blk_c * code_block_bytes(BITS) + p * 512 + li * 16);
        const uint4 m4 = *reinterpret_cast<const uint4*>(km_row + (size_t)j * kD + 4 * li);

        float qz[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) qz[r] = 0.0f;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const uint32_t m = comp(m4, cc);
            float s, z;
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), s, z);
            const float sf = s * unshift;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                // quad layout: channel c = 16*T + 4*rr + k is word T*16 + k*4 + rr
                qs_lds[wave][hw][r * kD + (li / 4) * 16 + cc * 4 + (li % 4)] = qsc[r][cc] * sf;
                qz[r] = __builtin_fmaf(qsc[r][cc], z, qz[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
#pragma unroll
            for (int m = 16; m >= 1; m >>= 1) qz[r] += __shfl_xor(qz[r], m, 64);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        float acc[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r] = qz[r];

#pragma unroll
        for (int T = 0; T < 8; ++T) {
            float4 qv[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r)
                qv[r] = *reinterpret_cast<const float4*>(&qs_lds[wave][hw][r * kD + T * 16 + (lane & 3) * 4]);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int v = 4 * T + rr, W = v / HPD, h = v % HPD;
                const uint32_t mk = comp(cw[W / 4], W % 4) & (MASK << (BITS * h));
#pragma unroll
                for (int r0 = 0; r0 < NR; r0 += RC) {
                    float qr[RC];
#pragma unroll
                    for (int r = 0; r < RC; ++r) qr[r] = comp(qv[r0 + r], rr);
                    fmac_block<RC>(&acc[r0], qr, mk);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if (active) {
            const int i = blk * kBlockTokens + li;
            float best = -INFINITY;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                logits[((size_t)row * NR + r) * logit_stride + i] = acc[r];
                if (r % NROWS == NROWS - 1) best = fmaxf(best, acc[r]);
            }
            keys[(size_t)row * key_stride + i] = float_to_key(best);
        }
    }
}

template <int BITS, int GROUP, int G, int NROWS>
hipError_t launch3(const LayerView& L, const void* q, int Nq, float sm_scale, float* logits, size_t logit_stride,
                   uint32_t* keys, size_t key_stride, hipStream_t stream) {
    const int n_tiles = (Nq / kBlockTokens + 1) / 2;
    // aim at several workgroups per compute unit while keeping the per-wave set-up amortised
    int tpw = 4;
    while (tpw > 1 && (long)L.rows * ((n_tiles + kScoreWaves * tpw - 1) / (kScoreWaves * tpw)) < 2048) tpw >>= 1;
    const dim3 grid((n_tiles + kScoreWaves * tpw - 1) / (kScoreWaves * tpw), L.rows), block(64 * kScoreWaves);
    if (L.bf16)
        hipLaunchKernelGGL((score_kernel<BITS, GROUP, G, NROWS, true>), grid, block, 0, stream, L,
                           (const uint16_t*)q, Nq, sm_scale, logits, logit_stride, keys, key_stride, tpw);
    else
        hipLaunchKernelGGL((score_kernel<BITS, GROUP, G, NROWS, false>), grid, block, 0, stream, L,
                           (const uint16_t*)q, Nq, sm_scale, logits, logit_stride, keys, key_stride, tpw);
    return hipGetLastError();
}

template <int BITS, int GROUP>
hipError_t launch2(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                   size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
#define SPC_CASE(g_, n_)                                                                                    \
    if (L.G == g_ && n_rows == n_)                                                                          \
        return launch3<BITS, GROUP, g_, n_>(L, q, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    SPC_CASE(1, 1) SPC_CASE(1, 2) SPC_CASE(2, 1) SPC_CASE(2, 2) SPC_CASE(4, 1) SPC_CASE(4, 2) SPC_CASE(8, 1)
    SPC_CASE(8, 2)
#undef SPC_CASE
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_score(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                        size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (Nq <= 0) return hipSuccess;
    if (L.bits == 2 && L.group == 32) return launch2<2, 32>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 2 && L.group == 64) return launch2<2, 64>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 1 && L.group == 32) return launch2<1, 32>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 1 && L.group == 64) return launch2<1, 64>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
