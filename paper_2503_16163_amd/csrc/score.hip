// Low-bit scoring (Appendix A "Decoding": A = Q K^T on the low-bit keys C', read once
// for the output token's and the speculative token's query rows; Section 3.3).
//
// logit[r][i] = sm_scale * sum_c q[r][c] * (code[i][c] * s[j][c] + z[j][c]),  j = i / g
//             = sum_c (sm_scale q[r][c] s[j][c]) * code[i][c]  +  sum_c sm_scale q[r][c] z[j][c]
// Keys are quantised per channel over g tokens, so the folded multiplier
// qs[r][c] and the constant qz[r] are shared by the tokens of a group.
//
// Mapping: one workgroup of four waves per 512-token tile, each wave taking a quarter of
// the channels (code dwords).  A lane scores 8 consecutive tokens of one 32-token sub-group;
// the four lanes of a quad cover that sub-group and fold its multipliers straight from the
// metadata, quad lane k those of the channels with channel % 4 == k, and exchange them
// through a wave-private LDS area (one vector write and up to four 16-byte reads per mask)
// so that they reach the multiply-accumulates as plain register operands.  Codes become
// floats with v_cvt_f32_ubyte{0..3} after one mask per four codes.  Query rows are taken in
// passes of at most four (a pass converts the codes again, but 32 accumulators instead of up
// to 128 keep four waves per SIMD resident); after a pass the waves swap partial sums through
// the same LDS area and each finishes, stores and ranks two of the lane's eight tokens.
// Measured on MI355X, with every load of the kernel served from cache: the kernel takes as
// long as with the loads from HBM less about a tenth, and its time follows the count of
// vector instructions (per code one multiply-accumulate per query row and one conversion
// per pass) at four clocks each; a DPP move costs more than twice that, which is why the
// multipliers travel through LDS.
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

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
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
    constexpr int RH = NR < 4 ? NR : 4;        // query rows per pass
    constexpr int HPD = (32 / BITS) / 4;       // masks (= multiplier registers) per code dword
    constexpr int NW = 4 * BITS;               // code dwords per token
    constexpr int WPW = NW / kScoreWaves;      // code dwords per wave
    constexpr int TPW = kTok / kScoreWaves;    // tokens of a lane that one wave finishes
    constexpr bool kRowSplit = G == 1 && NROWS == 2;
    constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x01010101u;
    // query rows in quad layout [row][channel % 4][channel / 4], rows of 32 padded to 36 floats so
    // that the four quad lanes read different banks
    __shared__ __attribute__((aligned(16))) float qfq[NR][4][36];
    // Per wave: first the multipliers of a pass, [sub-group][mask][channel % 4][row] with the
    // sub-groups 8 floats apart in bank space; once it has scored its share, its partial sums.
    constexpr int kMultQuad = WPW * HPD * 4 * RH + 8;
    constexpr int kWaveFloats = 16 * kMultQuad > kTok * RH * 64 ? 16 * kMultQuad : kTok * RH * 64;
    __shared__ __attribute__((aligned(16))) float wsm[kScoreWaves][kWaveFloats];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, k = lane & 3;
    const int row = blockIdx.y, tile = blockIdx.x;
    if (append_tail_block(L, row)) return;   // the extra workgroup of a fused append
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

    float* mq = &wsm[wave][(lane >> 2) * kMultQuad];
    const int i0 = sub * kBlockTokens + kTok * k + TPW * wave;   // first of the tokens this wave finishes for the lane
    float best[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) best[t] = -INFINITY;

#pragma unroll 1
    for (int r0 = 0; r0 < NR; r0 += RH) {
        if constexpr (NR > RH) {
            // Everything derived from the loaded dwords is the same in every pass; hoisting it out of
            // the loop would cost the registers the passes are there to save, so the loads are
            // made to look pass-dependent.
#pragma unroll
            for (int i = 0; i < WPW; ++i) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    asm volatile("" : "+v"(cw[i][j].x), "+v"(cw[i][j].y), "+v"(cw[i][j].z), "+v"(cw[i][j].w));
#pragma unroll
                for (int j = 0; j < HPD / 4; ++j)
                    asm volatile("" : "+v"(mt[i][j].x), "+v"(mt[i][j].y), "+v"(mt[i][j].z), "+v"(mt[i][j].w));
            }
        }
        // Every lane folds the multipliers of its channel class for all masks of this wave and
        // leaves them in LDS, from where the four lanes of the quad read all four classes back:
        // the lanes of a wave run in lockstep and LDS serves one wave's accesses in order, so
        // no workgroup barrier is involved.
        float qz[RH];
#pragma unroll
        for (int r = 0; r < RH; ++r) qz[r] = 0.0f;
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int W = wave * WPW + i;
#pragma unroll
            for (int h = 0; h < HPD; ++h) {
                const uint32_t m = comp(mt[i][h / 4], h % 4);
                float sc, z;
                derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), L.one_bit_plain, sc, z);
                // the codes of mask h arrive scaled by 2^(BITS*h)
                const float sf = sc * __uint_as_float((uint32_t)(127 - BITS * h) << 23);
                float qs[RH];
#pragma unroll
                for (int r = 0; r < RH; ++r) {
                    const float qv = qfq[r0 + r][k][HPD * W + h];
                    qs[r] = qv * sf;
                    qz[r] = __builtin_fmaf(qv, z, qz[r]);
                }
                float* dst = mq + ((i * HPD + h) * 4 + k) * RH;
                if constexpr (RH == 4) *reinterpret_cast<float4*>(dst) = make_float4(qs[0], qs[1], qs[2], qs[3]);
                else if constexpr (RH == 2) *reinterpret_cast<float2*>(dst) = make_float2(qs[0], qs[1]);
                else dst[0] = qs[0];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        float acc[kTok][RH];
#pragma unroll
        for (int s = 0; s < kTok; ++s)
#pragma unroll
            for (int r = 0; r < RH; ++r) acc[s][r] = 0.0f;
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
#pragma unroll
            for (int h = 0; h < HPD; ++h) {
                float b[4][RH];
                const float* src = mq + (i * HPD + h) * 4 * RH;
#pragma unroll
                for (int v = 0; v < RH; ++v) {   // RH 16-byte reads cover [4 channel classes][RH rows]
                    const float4 t = *reinterpret_cast<const float4*>(src + 4 * v);
                    const float tv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) b[(4 * v + e) / RH][(4 * v + e) % RH] = tv[e];
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
                for (int r = 0; r < RH; ++r)
#pragma unroll
                    for (int s = 0; s < kTok; ++s) {
                        acc[s][r] = __builtin_fmaf(f[s][0], b[0][r], acc[s][r]);
                        acc[s][r] = __builtin_fmaf(f[s][1], b[1][r], acc[s][r]);
                        acc[s][r] = __builtin_fmaf(f[s][2], b[2][r], acc[s][r]);
                        acc[s][r] = __builtin_fmaf(f[s][3], b[3][r], acc[s][r]);
                    }
            }
        }
        // the zero-point term of this wave's channels: sum over the quad's four channel classes
#pragma unroll
        for (int r = 0; r < RH; ++r) {
            float v = qz[r];
            v += dpp_move<0xB1>(v);   // quad lanes 1 apart
            v += dpp_move<0x4E>(v);   // quad lanes 2 apart
#pragma unroll
            for (int s = 0; s < kTok; ++s) acc[s][r] += v;
        }
        // swap partial sums (the area is this wave's own: its multiplier reads are behind it)
#pragma unroll
        for (int s = 0; s < kTok; ++s)
#pragma unroll
            for (int r = 0; r < RH; ++r) wsm[wave][(s * RH + r) * 64 + lane] = acc[s][r];
        __syncthreads();
        if constexpr (kRowSplit) {
            // one KV head per query head, two rows: wave = (row, half of the lane's tokens), so that
            // logits and keys leave as 16-byte stores; the keys are the speculative row's alone
            const int r = wave & 1, hf = wave >> 1;
            float o[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int s = 4 * hf + t;
                float v = wsm[0][(s * RH + r) * 64 + lane];
#pragma unroll
                for (int w = 1; w < kScoreWaves; ++w) v += wsm[w][(s * RH + r) * 64 + lane];
                o[t] = v;
            }
            if (active) {
                const int i4 = sub * kBlockTokens + kTok * k + 4 * hf;
                *reinterpret_cast<float4*>(logits + ((size_t)row * NR + r) * logit_stride + i4) = make_float4(o[0], o[1], o[2], o[3]);
                if (r == NROWS - 1)
                    *reinterpret_cast<uint4*>(keys + (size_t)row * key_stride + i4) =
                        make_uint4(float_to_key(o[0]), float_to_key(o[1]), float_to_key(o[2]), float_to_key(o[3]));
            }
        } else {
#pragma unroll
            for (int r = 0; r < RH; ++r) {
                float o[TPW];
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const int s = TPW * wave + t;
                    float v = wsm[0][(s * RH + r) * 64 + lane];
#pragma unroll
                    for (int w = 1; w < kScoreWaves; ++w) v += wsm[w][(s * RH + r) * 64 + lane];
                    o[t] = v;
                    if ((r0 + r) % NROWS == NROWS - 1) best[t] = fmaxf(best[t], v);
                }
                static_assert(TPW == 2, "one 8-byte store per lane and row");
                if (active)
                    *reinterpret_cast<float2*>(logits + ((size_t)row * NR + r0 + r) * logit_stride + i0) = make_float2(o[0], o[1]);
            }
        }
        if (r0 + RH < NR) __syncthreads();   // partial sums consumed before the next pass reuses the area
    }
    if constexpr (!kRowSplit) {
        if (active)
            *reinterpret_cast<uint2*>(keys + (size_t)row * key_stride + i0) = make_uint2(float_to_key(best[0]), float_to_key(best[1]));
    }
}

template <int BITS, int G, int NROWS>
hipError_t launch3(const LayerView& L, const void* q, int Nq, float sm_scale, float* logits, size_t logit_stride,
                   uint32_t* keys, size_t key_stride, hipStream_t stream) {
    const dim3 grid((Nq + kTileTokens - 1) / kTileTokens + (L.tail_k ? 1 : 0), L.rows), block(64 * kScoreWaves);
    if (L.bf16)
        SPC_LAUNCH((score_kernel<BITS, G, NROWS, true>), grid, block, stream, L, (const uint16_t*)q, Nq,
                           sm_scale, logits, logit_stride, keys, key_stride);
    else
        SPC_LAUNCH((score_kernel<BITS, G, NROWS, false>), grid, block, stream, L, (const uint16_t*)q, Nq,
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
    if (L.group != 32 && L.group != 64 && L.group != 128) return hipErrorInvalidValue;
    if (L.bits == 4) return launch_score4(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    // two rows of one query head: the integer matrix cores take the contraction (it reads q 16 bytes at a
    // time; the C ABI rejects a q that is not 16-byte aligned)
    if (score_uses_int8_matrix_cores(L.G, n_rows) && !(kernel_choice() & kChoiceScoreValu))
        return launch_score_i8(L, q, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (score_uses_matrix_cores(L.G, n_rows))
        return launch_score_mfma(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 2) return launch2<2>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 1) return launch2<1>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
