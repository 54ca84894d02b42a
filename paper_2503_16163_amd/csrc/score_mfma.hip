// Low-bit scoring with 8 or 16 query rows per KV head (grouped-query attention, both query
// rows of Appendix A "Decoding") on the matrix cores.
//
// logit[r][i] = sum_c code[i][c] * (sm_scale q[r][c] s[j][c])  +  sum_c sm_scale q[r][c] z[j][c],  j = i / g
// With this many rows per KV head the first sum is a dense enough contraction: per 32 tokens
// and 32 channels one v_mfma_f32_16x16x32_f16 with
//   A = codes (rows: 16 tokens, columns: 32 channels), read from the packed dwords as f16
//       subnormals (a byte holding code << (8 - BITS), widened to 16 bits, is the f16 number
//       code * 2^(8 - BITS - 24); the codes are lifted to the top bits of their byte because
//       the matrix cores do not normalise subnormal operands before aligning products),
//   B = the folded multipliers of the token group, scaled by a power of two near the top of
//       the f16 range and split into hi + lo f16 (columns: (row r, hi | lo)),
//   C accumulating in fp32.
// A workgroup of four waves takes a 512-token tile, a wave 128 tokens of it (four sub-groups
// of 32) with all channels, so no sums cross waves.  The multipliers of a token group are
// folded once per group by the wave: each lane derives (s, z) of two channels into a
// wave-private LDS table, then builds the B operands of its column.  The zero-point term
// is a plain dot product per (row, group), summed over the four lanes of a column.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// lane exchange patterns inside a row of 16 lanes
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

// two bytes of w, each widened to 16 bits
template <int HI>
__device__ __forceinline__ uint32_t bytes_to_halves(uint32_t w) {
    return __builtin_amdgcn_perm(0u, w, HI ? 0x0c030c02u : 0x0c010c00u);
}

__device__ __forceinline__ float wave_max_nonneg(float v) {
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_move<kDppMirror>(v));
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

constexpr int kWaves = 4;
constexpr int kSubPerWave = (kTileTokens / kBlockTokens) / kWaves;   // 32-token sub-groups per wave

template <int BITS, int G, int NROWS, bool BF16>
__global__ __launch_bounds__(64 * kWaves) void score_mfma_kernel(LayerView L, const uint16_t* __restrict__ q, int Nq,
                                                                 float sm_scale, float* __restrict__ logits,
                                                                 size_t logit_stride, uint32_t* __restrict__ keys,
                                                                 size_t key_stride) {
    constexpr int NR = G * NROWS;
    constexpr int NT = NR / 8;                 // column tiles of 8 query rows x (hi, lo)
    constexpr int CPW = 32 / BITS;             // channels per code dword
    static_assert(NR % 8 == 0, "one column tile is 8 query rows");
    __shared__ __attribute__((aligned(16))) float sz[kWaves][2][kD];   // (s, z) of the wave's current token group

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int ic = lane & 15, kq = lane >> 4;
    const int row = blockIdx.y, tile = blockIdx.x;
    if (append_tail_block(L, row)) return;   // the extra workgroup of a fused append
    const int n_sub = Nq / kBlockTokens;

    // This lane's multipliers-to-be.  Column (r, hi | lo) needs sm_scale * q[r][32 kc + 8 kq + e],
    // e = 0..7, per chunk; the two lanes of a column pair share that work, the hi lane taking
    // e = 0..3 and the lo lane e = 4..7, and swap halves of their operands afterwards.  The
    // values are kept scaled by a power of two chosen from the row's largest |q| (|q'| < 2^7).
    const int hl = ic & 1;
    float qreg[NT][4][4];
    float q_unscale[NT];                       // the inverse of that power of two
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int r = 8 * nt + (ic >> 1);
        const uint16_t* qr = q + ((size_t)row * NR + r) * kD;
        float qa = 0.0f;
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
            const uint2 w = *reinterpret_cast<const uint2*>(qr + 32 * kc + 8 * kq + 4 * hl);
            const uint32_t wd[2] = {w.x, w.y};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = widen16<BF16>((wd[e / 2] >> (16 * (e % 2))) & 0xFFFFu) * sm_scale;
                qreg[nt][kc][e] = v;
                qa = fmaxf(qa, fabsf(v));
            }
        }
        // largest |q| of the row: over the pair and the four lanes of the column
        qa = fmaxf(qa, __shfl_xor(qa, 1, 64));
        qa = fmaxf(qa, __shfl_xor(qa, 16, 64));
        qa = fmaxf(qa, __shfl_xor(qa, 32, 64));
        const uint32_t eq = (__float_as_uint(qa) >> 23) & 0xFFu;       // |q| < 2^(eq - 126)
        int fq = 260 - (int)eq;                                        // field of 2^(133 - eq)
        fq = fq < 100 ? 100 : (fq > 224 ? 224 : fq);
        const float qscale = __uint_as_float((uint32_t)fq << 23);
        q_unscale[nt] = __uint_as_float((uint32_t)(254 - fq) << 23);
#pragma unroll
        for (int kc = 0; kc < 4; ++kc)
#pragma unroll
            for (int e = 0; e < 4; ++e) qreg[nt][kc][e] *= qscale;
    }

    // code bits of this lane's 8 channels of a 32-channel chunk: channel 32 kc + 8 kq + e is code
    // w' = 8 kq' + e of its dword (kq' = kq % (CPW / 8)), i.e. byte e % 4, field h0 + e / 4
    constexpr int KPD = CPW / 8;               // lanes kq that share one code dword
    const int h0 = 2 * (kq % KPD);
    uint32_t amask[2], ashift[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int h = h0 + u;
        amask[u] = (((1u << BITS) - 1u) * 0x01010101u) << (BITS * h);
        ashift[u] = (8 - BITS) - BITS * h;
    }
    constexpr float kUnlift = 1.0f / (float)(1 << (8 - BITS));

    uint4v bop[NT][4];
    float qz[NT], unscale[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        qz[nt] = 0.0f;
        unscale[nt] = 0.0f;
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) bop[nt][kc] = uint4v{0u, 0u, 0u, 0u};
    }
    int group_done = -1;

    for (int sg = 0; sg < kSubPerWave; ++sg) {
        const int sub = tile * 16 + wave * kSubPerWave + sg;       // 32-token sub-group of the row
        if (sub >= n_sub) break;                                   // uniform over the wave
        const int tok0 = sub * kBlockTokens;
        // ---- this sub-group's code dwords: row it = ic is tokens 2 ic and 2 ic + 1 of the sub-group ----
        // piece (dword W, half (ic % 4) / 2, lane 4 (sub % 16) + ic / 4), bytes 8 (ic % 2) .. + 7
        const uint8_t* kc_base = L.kc + (size_t)row * L.kc_stride + (size_t)tile * k_tile_bytes(BITS) +
                                 ((size_t)((ic % 4) / 2) * 64 + 4 * (sub % 16) + ic / 4) * 16 + 8 * (ic % 2);
        uint2 cw[4];
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
            const int W = (kc * 32 + 8 * kq) / CPW;
            cw[kc] = *reinterpret_cast<const uint2*>(kc_base + (size_t)(W * 2) * 1024);
        }

        // ---- multipliers of the token group (once per group) ----
        const int grp = tok0 / L.group;
        if (grp != group_done) {
            group_done = grp;
            const uint32_t* km = L.km + (size_t)row * L.km_stride + (size_t)grp * kD;
            const uint32_t m0 = km[k_meta_index(2 * lane)], m1 = km[k_meta_index(2 * lane + 1)];
            float s0, z0, s1, z1;
            derive_scale_zero<BITS>(widen16<BF16>(m0 & 0xFFFFu), widen16<BF16>(m0 >> 16), L.one_bit_plain, s0, z0);
            derive_scale_zero<BITS>(widen16<BF16>(m1 & 0xFFFFu), widen16<BF16>(m1 >> 16), L.one_bit_plain, s1, z1);
            // the table holds s scaled by a power of two chosen from the group's largest s (s' < 2^8),
            // so that q' s' < 2^15 sits near the top of the f16 range
            const float smax = wave_max_nonneg(fmaxf(s0, s1));
            const uint32_t es = (__float_as_uint(smax) >> 23) & 0xFFu;     // s < 2^(es - 126)
            int fs = 261 - (int)es;                                        // field of 2^(134 - es)
            fs = fs < 100 ? 100 : (fs > 224 ? 224 : fs);
            const float sscale = __uint_as_float((uint32_t)fs << 23);
            const float s_unscale = __uint_as_float((uint32_t)(254 - fs) << 23) * (kUnlift * 16777216.0f);   // 2^24 / (s scale 2^(8-BITS))
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // earlier reads of the table are done
            __builtin_amdgcn_wave_barrier();
            *reinterpret_cast<float2*>(&sz[wave][0][2 * lane]) = make_float2(s0 * sscale, s1 * sscale);
            *reinterpret_cast<float2*>(&sz[wave][1][2 * lane]) = make_float2(z0, z1);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                unscale[nt] = q_unscale[nt] * s_unscale;
                float zacc = 0.0f;
#pragma unroll
                for (int kc = 0; kc < 4; ++kc) {
                    const float4 sa = *reinterpret_cast<const float4*>(&sz[wave][0][32 * kc + 8 * kq + 4 * hl]);
                    const float4 za = *reinterpret_cast<const float4*>(&sz[wave][1][32 * kc + 8 * kq + 4 * hl]);
                    const float sv[4] = {sa.x, sa.y, sa.z, sa.w};
                    const float zv[4] = {za.x, za.y, za.z, za.w};
                    uint32_t keep[2], send[2];
#pragma unroll
                    for (int e2 = 0; e2 < 2; ++e2) {
                        const float q0 = qreg[nt][kc][2 * e2], q1 = qreg[nt][kc][2 * e2 + 1];
                        zacc = __builtin_fmaf(q0, zv[2 * e2], zacc);
                        zacc = __builtin_fmaf(q1, zv[2 * e2 + 1], zacc);
                        const float x0 = q0 * sv[2 * e2], x1 = q1 * sv[2 * e2 + 1];
                        // hi by truncation, lo = x - hi: hi + lo is x to 2^-21
                        const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(x0, x1));
                        const float h0f = widen16<false>(hi & 0xFFFFu), h1f = widen16<false>(hi >> 16);
                        const uint32_t lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(x0 - h0f, x1 - h1f));
                        // the hi lane keeps its hi halves and hands its lo halves to the lo lane, and vice versa
                        keep[e2] = hl ? lo : hi;
                        send[e2] = hl ? hi : lo;
                    }
                    const uint32_t r0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send[0], kDppXor1, 0xf, 0xf, true);
                    const uint32_t r1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send[1], kDppXor1, 0xf, 0xf, true);
                    // k-slots 0..3 come from the hi lane's channels, 4..7 from the lo lane's
                    bop[nt][kc] = hl ? uint4v{r0, r1, keep[0], keep[1]} : uint4v{keep[0], keep[1], r0, r1};
                }
                // the zero-point term of (row, group): the pair and the four lanes of the column hold a share each
                zacc += dpp_move<kDppXor1>(zacc);
                zacc += __shfl_xor(zacc, 16, 64);
                zacc += __shfl_xor(zacc, 32, 64);
                qz[nt] = zacc * q_unscale[nt];
            }
        }

        // ---- products: two row tiles (even and odd tokens) x four channel chunks ----
        float4v acc[2][NT];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const uint32_t w = mt == 0 ? cw[kc].x : cw[kc].y;
                const uint32_t ma = (w & amask[0]) << ashift[0], mb = (w & amask[1]) << ashift[1];
                const uint4v aop{bytes_to_halves<0>(ma), bytes_to_halves<1>(ma), bytes_to_halves<0>(mb), bytes_to_halves<1>(mb)};
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop),
                                                                         __builtin_bit_cast(half8, bop[nt][kc]), acc[mt][nt], 0, 0, 0);
            }
        }

        // ---- C rows 4 kq + v of tile mt are tokens 2 (4 kq + v) + mt: this lane's 8 consecutive tokens ----
        float best[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) best[t] = -INFINITY;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int r = 8 * nt + (ic >> 1);
            const bool last = (r % NROWS) == NROWS - 1;
            float o[8];
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    float val = acc[mt][nt][v];
                    val += dpp_move<kDppXor1>(val);                 // hi column + lo column
                    val = val * unscale[nt] + qz[nt];
                    o[2 * v + mt] = val;
                    best[2 * v + mt] = fmaxf(best[2 * v + mt], last ? val : -INFINITY);
                }
            if ((ic & 1) == 0) {
                float4* dst = reinterpret_cast<float4*>(logits + ((size_t)row * NR + r) * logit_stride + tok0 + 8 * kq);
                dst[0] = make_float4(o[0], o[1], o[2], o[3]);
                dst[1] = make_float4(o[4], o[5], o[6], o[7]);
            }
        }
        // selection key: maximum over the heads' last rows = over the 16 lanes of the column row
        // (both lanes of a pair hold the same value)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float b = best[t];
            b = fmaxf(b, dpp_move<kDppXor2>(b));
            b = fmaxf(b, dpp_move<kDppHalfMirror>(b));
            b = fmaxf(b, dpp_move<kDppMirror>(b));
            best[t] = b;
        }
        if (ic == 0) {
            uint4* kd = reinterpret_cast<uint4*>(keys + (size_t)row * key_stride + tok0 + 8 * kq);
            kd[0] = make_uint4(float_to_key(best[0]), float_to_key(best[1]), float_to_key(best[2]), float_to_key(best[3]));
            kd[1] = make_uint4(float_to_key(best[4]), float_to_key(best[5]), float_to_key(best[6]), float_to_key(best[7]));
        }
    }
}

template <int BITS, int G, int NROWS>
hipError_t launch_case(const LayerView& L, const void* q, int Nq, float sm_scale, float* logits, size_t logit_stride,
                       uint32_t* keys, size_t key_stride, hipStream_t stream) {
    const dim3 grid((Nq + kTileTokens - 1) / kTileTokens + (L.tail_k ? 1 : 0), L.rows), block(64 * kWaves);
    if (L.bf16)
        SPC_LAUNCH((score_mfma_kernel<BITS, G, NROWS, true>), grid, block, stream, L, (const uint16_t*)q, Nq,
                           sm_scale, logits, logit_stride, keys, key_stride);
    else
        SPC_LAUNCH((score_mfma_kernel<BITS, G, NROWS, false>), grid, block, stream, L, (const uint16_t*)q, Nq,
                           sm_scale, logits, logit_stride, keys, key_stride);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_bits(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                       size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (L.G == 4 && n_rows == 2) return launch_case<BITS, 4, 2>(L, q, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.G == 8 && n_rows == 1) return launch_case<BITS, 8, 1>(L, q, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.G == 8 && n_rows == 2) return launch_case<BITS, 8, 2>(L, q, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    return hipErrorInvalidValue;
}

}  // namespace

bool score_uses_matrix_cores(int G, int n_rows) { return G * n_rows >= 8 && (G * n_rows) % 8 == 0; }

hipError_t launch_score_mfma(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                             size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (L.bits == 2) return launch_bits<2>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    if (L.bits == 1) return launch_bits<1>(L, q, n_rows, Nq, sm_scale, logits, logit_stride, keys, key_stride, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
