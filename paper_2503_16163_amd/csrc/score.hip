// Low-bit scoring (Appendix A "Decoding": A = Q K^T on the low-bit keys C', read once
// for the output token's and the speculative token's query rows; Section 3.3).
//
// logit[r][i] = sm_scale * sum_c q[r][c] * (code[i][c] * s[j][c] + z[j][c]),  j = i / g
//             = sum_c (sm_scale q[r][c] s[j][c]) * code[i][c]  +  sum_c sm_scale q[r][c] z[j][c]
// Keys are quantised per channel over g tokens, so the folded multiplier
// qs[r][c] and the constant qz[r] are shared by the tokens of a group.
//
// Mapping: one workgroup of four waves per 512-token tile, each wave taking a quarter of
// the channels (code dwords) and wave 0 adding up the partial sums.  A lane scores 8
// consecutive tokens of one 32-token sub-group; the four lanes of a quad cover that
// sub-group and fold its multipliers straight from the metadata, quad lane k those of the
// channels with channel % 4 == k.  With one or two query rows the quad exchanges them through
// LDS (a wave-private area: one 8-byte write and two 16-byte reads per mask) so that they
// reach the multiply-accumulates as plain register operands; with more rows they stay in
// registers and are broadcast inside the quad with DPP moves, one per 8 tokens.  Codes
// become floats with v_cvt_f32_ubyte{0..3} after one mask per four codes.
// Measured on MI355X, with every load of the kernel served from cache: the kernel takes as
// long as with the loads from HBM less about a tenth, and its time follows the count of
// vector instructions (two multiply-accumulates and one conversion per code) at four clocks
// each; a DPP move costs more than twice that, which is why the LDS exchange pays.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

template <int B>
__device__ __forceinline__ float cvt_ubyte(uint32_t w) {
    float f;
    if constexpr (B == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(w));
    if constexpr (B == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(w));
    if constexpr (B == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(w));
    if constexpr (B == 3) asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(w));
    return f;
}

// value of quad lane K's register, in every lane of the quad
template <int K>
__device__ __forceinline__ float quad_bcast(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x55 * K, 0xf, 0xf, true));
}

__device__ __forceinline__ uint32_t comp(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

constexpr int kTok = 8;   // tokens per lane

constexpr int kScoreWaves = 4;   // waves per tile: each takes a quarter of the code dwords

template <int BITS, int G, int NROWS, bool BF16>
__global__ __launch_bounds__(64 * kScoreWaves) void score_kernel(LayerView L, const uint16_t* __restrict__ q, int Nq,
                                                                 float sm_scale, float* __restrict__ logits,
                                                                 size_t logit_stride, uint32_t* __restrict__ keys,
                                                                 size_t key_stride) {
    constexpr int NR = G * NROWS;              // query rows sharing this KV head
    constexpr int HPD = (32 / BITS) / 4;       // masks (= multiplier registers) per code dword
    constexpr int NW = 4 * BITS;               // code dwords per token
    constexpr int WPW = NW / kScoreWaves;      // code dwords per wave
    constexpr int NP = kTok * NR + NR;         // partial sums per lane: logits and the zero-point terms
    constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x01010101u;
    // query rows in quad layout [row][channel % 4][channel / 4], rows of 32 padded to 36 floats so
    // that the four quad lanes read different banks
    __shared__ __attribute__((aligned(16))) float qfq[NR][4][36];
    // Per wave: first the multipliers it folds, [sub-group][mask][channel % 4][row] with the
    // sub-groups 8 floats apart in bank space; once it has scored its share, its partial sums.
    constexpr bool kLdsMult = NR <= 2;
    constexpr int kMultQuad = WPW * HPD * 4 * NR + 8;
    constexpr int kWaveFloats = (kLdsMult && 16 * kMultQuad > NP * 64) ? 16 * kMultQuad : NP * 64;
    __shared__ __attribute__((aligned(16))) float wsm[kScoreWaves][kWaveFloats];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, k = lane & 3;
    const int row = blockIdx.y, tile = blockIdx.x;
    const int n_sub = Nq / kBlockTokens;                       // quantised 32-token sub-groups
    const int sub = tile * 16 + (lane >> 2);
    const bool active = sub < n_sub;
    const int sub_c = active ? sub : n_sub - 1;                // inactive lanes recompute the last sub-group
    const int lane_c = active ? lane : ((n_sub - 1) % 16) * 4 + k;
    const uint8_t* kc_lane = L.kc + (size_t)row * L.kc_stride + (size_t)tile * k_tile_bytes(BITS) + (size_t)lane_c * 16;
    const uint32_t* km_lane = L.km + (size_t)row * L.km_stride + (size_t)(sub_c * kBlockTokens / L.group) * kD + k * 32;

    // this wave's code dwords of the lane's 8 tokens (two 16-byte loads per dword, each 1 KB
    // contiguous across the wave) and the (min,max) pairs of their channels, requested up front
    uint4 cw[WPW][2], mt[WPW][HPD / 4];
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
        const int W = wave * WPW + i;
        cw[i][0] = *reinterpret_cast<const uint4*>(kc_lane + (size_t)(W * 2) * 1024);
        cw[i][1] = *reinterpret_cast<const uint4*>(kc_lane + (size_t)(W * 2 + 1) * 1024);
#pragma unroll
        for (int j = 0; j < HPD / 4; ++j) mt[i][j] = *reinterpret_cast<const uint4*>(km_lane + HPD * W + 4 * j);
    }

    for (int e = threadIdx.x; e < NR * kD; e += 64 * kScoreWaves) {
        const int r = e / kD, c = e % kD;
        qfq[r][c % 4][c / 4] = widen16<BF16>(q[(size_t)row * NR * kD + e]) * sm_scale;
    }
    __syncthreads();

    float acc[kTok][NR];
    float qz[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) qz[r] = 0.0f;
#pragma unroll
    for (int s = 0; s < kTok; ++s)
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[s][r] = 0.0f;

    if constexpr (kLdsMult) {
        // Every lane folds the multipliers of its channel class (channel % 4 == k) for all masks of
        // this wave and leaves them in LDS, from where the four lanes of the quad read all four
        // classes back as plain operands: the lanes of a wave run in lockstep and LDS serves one
        // wave's accesses in order, so no workgroup barrier is involved.
        float* mq = &wsm[wave][(lane >> 2) * kMultQuad];
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int W = wave * WPW + i;
#pragma unroll
            for (int h = 0; h < HPD; ++h) {
                const uint32_t m = comp(mt[i][h / 4], h % 4);
                float sc, z;
                derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), sc, z);
                const float sf = sc * __uint_as_float((uint32_t)(127 - BITS * h) << 23);
                float qs[NR];
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    const float qv = qfq[r][k][HPD * W + h];
                    qs[r] = qv * sf;
                    qz[r] = __builtin_fmaf(qv, z, qz[r]);
                }
                float* dst = mq + ((i * HPD + h) * 4 + k) * NR;
                if constexpr (NR == 2) *reinterpret_cast<float2*>(dst) = make_float2(qs[0], qs[1]);
                else dst[0] = qs[0];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
#pragma unroll
            for (int h = 0; h < HPD; ++h) {
                float b[4][NR];
                const float* src = mq + (i * HPD + h) * 4 * NR;
                if constexpr (NR == 2) {
                    const float4 t0 = *reinterpret_cast<const float4*>(src), t1 = *reinterpret_cast<const float4*>(src + 4);
                    b[0][0] = t0.x; b[0][1] = t0.y; b[1][0] = t0.z; b[1][1] = t0.w;
                    b[2][0] = t1.x; b[2][1] = t1.y; b[3][0] = t1.z; b[3][1] = t1.w;
                } else {
                    const float4 t0 = *reinterpret_cast<const float4*>(src);
                    b[0][0] = t0.x; b[1][0] = t0.y; b[2][0] = t0.z; b[3][0] = t0.w;
                }
                float f[kTok][4];
#pragma unroll
                for (int s = 0; s < kTok; ++s) {
                    const uint32_t mk = comp(cw[i][s / 4], s % 4) & (MASK << (BITS * h));
                    f[s][0] = cvt_ubyte<0>(mk);
                    f[s][1] = cvt_ubyte<1>(mk);
                    f[s][2] = cvt_ubyte<2>(mk);
                    f[s][3] = cvt_ubyte<3>(mk);
                }
#pragma unroll
                for (int r = 0; r < NR; ++r)
#pragma unroll
                    for (int s = 0; s < kTok; ++s) {
                        acc[s][r] = __builtin_fmaf(f[s][0], b[0][r], acc[s][r]);
                        acc[s][r] = __builtin_fmaf(f[s][1], b[1][r], acc[s][r]);
                        acc[s][r] = __builtin_fmaf(f[s][2], b[2][r], acc[s][r]);
                        acc[s][r] = __builtin_fmaf(f[s][3], b[3][r], acc[s][r]);
                    }
            }
        }
    } else {
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
        const int W = wave * WPW + i;
        float qv[NR][HPD];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int j = 0; j < HPD / 4; ++j) {
                const float4 t = *reinterpret_cast<const float4*>(&qfq[r][k][HPD * W + 4 * j]);
                qv[r][4 * j] = t.x; qv[r][4 * j + 1] = t.y; qv[r][4 * j + 2] = t.z; qv[r][4 * j + 3] = t.w;
            }
#pragma unroll
        for (int h = 0; h < HPD; ++h) {
            // multiplier of channel 4*(HPD*W + h) + k for every query row
            const uint32_t m = comp(mt[i][h / 4], h % 4);
            float sc, z;
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), sc, z);
            // the codes of mask h arrive scaled by 2^(BITS*h)
            const float sf = sc * __uint_as_float((uint32_t)(127 - BITS * h) << 23);
            float qs[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                qs[r] = qv[r][h] * sf;
                qz[r] = __builtin_fmaf(qv[r][h], z, qz[r]);
            }
            float f[kTok][4];
#pragma unroll
            for (int s = 0; s < kTok; ++s) {
                const uint32_t mk = comp(cw[i][s / 4], s % 4) & (MASK << (BITS * h));
                f[s][0] = cvt_ubyte<0>(mk);
                f[s][1] = cvt_ubyte<1>(mk);
                f[s][2] = cvt_ubyte<2>(mk);
                f[s][3] = cvt_ubyte<3>(mk);
            }
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const float b0 = quad_bcast<0>(qs[r]), b1 = quad_bcast<1>(qs[r]);
                const float b2 = quad_bcast<2>(qs[r]), b3 = quad_bcast<3>(qs[r]);
#pragma unroll
                for (int s = 0; s < kTok; ++s) {
                    acc[s][r] = __builtin_fmaf(f[s][0], b0, acc[s][r]);
                    acc[s][r] = __builtin_fmaf(f[s][1], b1, acc[s][r]);
                    acc[s][r] = __builtin_fmaf(f[s][2], b2, acc[s][r]);
                    acc[s][r] = __builtin_fmaf(f[s][3], b3, acc[s][r]);
                }
            }
        }
    }

    }

    // waves 1.. hand their partial sums to wave 0
    if (wave > 0) {
#pragma unroll
        for (int s = 0; s < kTok; ++s)
#pragma unroll
            for (int r = 0; r < NR; ++r) wsm[wave][(s * NR + r) * 64 + lane] = acc[s][r];
#pragma unroll
        for (int r = 0; r < NR; ++r) wsm[wave][(kTok * NR + r) * 64 + lane] = qz[r];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 1; w < kScoreWaves; ++w) {
#pragma unroll
        for (int s = 0; s < kTok; ++s)
#pragma unroll
            for (int r = 0; r < NR; ++r) acc[s][r] += wsm[w][(s * NR + r) * 64 + lane];
#pragma unroll
        for (int r = 0; r < NR; ++r) qz[r] += wsm[w][(kTok * NR + r) * 64 + lane];
    }
    // the zero-point term: sum over the quad's four channel classes
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        qz[r] += __shfl_xor(qz[r], 1, 64);
        qz[r] += __shfl_xor(qz[r], 2, 64);
    }

    if (active) {
        const int i0 = sub * kBlockTokens + kTok * k;          // first of this lane's 8 consecutive tokens
        float best[kTok];
#pragma unroll
        for (int s = 0; s < kTok; ++s) best[s] = -INFINITY;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            float o[kTok];
#pragma unroll
            for (int s = 0; s < kTok; ++s) {
                o[s] = acc[s][r] + qz[r];
                if (r % NROWS == NROWS - 1) best[s] = fmaxf(best[s], o[s]);
            }
            float4* dst = reinterpret_cast<float4*>(logits + ((size_t)row * NR + r) * logit_stride + i0);
            dst[0] = make_float4(o[0], o[1], o[2], o[3]);
            dst[1] = make_float4(o[4], o[5], o[6], o[7]);
        }
        uint4* kd = reinterpret_cast<uint4*>(keys + (size_t)row * key_stride + i0);
        kd[0] = make_uint4(float_to_key(best[0]), float_to_key(best[1]), float_to_key(best[2]), float_to_key(best[3]));
        kd[1] = make_uint4(float_to_key(best[4]), float_to_key(best[5]), float_to_key(best[6]), float_to_key(best[7]));
    }
}

template <int BITS, int G, int NROWS>
hipError_t launch3(const LayerView& L, const void* q, int Nq, float sm_scale, float* logits, size_t logit_stride,
                   uint32_t* keys, size_t key_stride, hipStream_t stream) {
    const dim3 grid((Nq + kTileTokens - 1) / kTileTokens, L.rows), block(64 * kScoreWaves);
    if (L.bf16)
        hipLaunchKernelGGL((score_kernel<BITS, G, NROWS, true>), grid, block, 0, stream, L, (const uint16_t*)q, Nq,
                           sm_scale, logits, logit_stride, keys, key_stride);
    else
        hipLaunchKernelGGL((score_kernel<BITS, G, NROWS, false>), grid, block, 0, stream, L, (const uint16_t*)q, Nq,
                           sm_scale, logits, logit_stride, keys, key_stride);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch2(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                   size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
#define SPC_CASE(g_, n_)                                                                                    \
    if (L.G == g_ && n_rows == n_)                                                                          \
        return launch3<BITS, g_, n_>(L, q, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    SPC_CASE(1, 1) SPC_CASE(1, 2) SPC_CASE(2, 1) SPC_CASE(2, 2) SPC_CASE(4, 1) SPC_CASE(4, 2) SPC_CASE(8, 1)
    SPC_CASE(8, 2)
#undef SPC_CASE
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_score(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                        size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (Nq <= 0) return hipSuccess;
    if (L.group != 32 && L.group != 64) return hipErrorInvalidValue;
    if (L.bits == 2) return launch2<2>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 1) return launch2<1>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
