// Mixed attention of Eq. 1 (Section 3.3) for one query head per KV head and the two query rows
// of a decode step, 1- or 2-bit values: the value side on the integer matrix cores, alone
// (attend_i8_kernel, after a scoring pass that left the logits in memory) or in one pass with the
// low-bit scoring of Appendix A "Decoding" (the same kernel with the scoring pass in front: the logits never leave the chip).
//
// Values are quantised per token over g channels (Section 2.1 / 4.1), so over the quantised
// positions of a chunk
//   sum_i p[r][i] V'[i][c] = sum_i (p[r][i] s[i][m]) code[i][c]  +  sum_i p[r][i] z[i][m],   m = c / g.
// The first sum is a contraction over tokens.  On the vector ALUs it costs a conversion per code
// and a multiply-accumulate per code and row, and that instruction count bounds the kernel (three
// times the time its bytes need).  Here it runs as v_mfma_i32_16x16x64_i8:
//   A = codes.  The packed layout gives a lane 16 consecutive tokens of four channels in 16 bytes;
//       masking with 0x03030303 or 0x0C0C0C0C (after a shift by 4 for the upper two channels) leaves
//       the 16 int8 operands of one channel as they stand, code or 4 x code: five vector
//       instructions per 64 codes.  The 16 rows of an MFMA are 16 channels four apart: one half
//       ("set") of the head's channels, two value groups at g = 32;
//   B = p s as 32-bit fixed point relative to the largest scale of the wave's tokens (p <= 1), cut
//       into four byte planes, the low three re-centred to signed: column (row r, group, plane).
//       With two rows, two groups and four planes the 16 columns are exactly full; of every result
//       the half whose column group matches the row's channel group is used;
//   C = int32, exact.  The planes are recombined in fp32 when the workgroup merges its waves.
// With 1-bit codes a byte holds 8 channels of a token and 16 code lanes are all 128 channels: the masks are
// 0x01010101 << j on the word and on the word shifted by 4 (operands code x 1, 2, 4, 8), eight products per
// token step, each run against the columns of either channel half; of a product's 16 rows the 8 code lanes
// of that half are kept.
// The zero-point term and the row sums stay on the vector ALUs (one multiply-add per token, group
// and row).
//
// A workgroup takes a chunk of 512 quantised positions (or, as in the vector-ALU kernel, 128 16-bit
// candidates: attend_extra_chunk); its four waves are independent, each with 128 tokens and its own
// softmax maximum, and meet once, at the end, to merge their (max, sum, sum p V) into the chunk's
// partial result.  Lane = (32-token sub-group, h, token quad): it holds the logits of four
// consecutive tokens of row h (the layout in which the scoring wave finishes them), exchanges the
// numerators with the lane that holds the other row (one DPP rotation), and prepares p s of both
// rows for the value groups of channel set h.
#include "attend_common.h"
#include "score_i8_wave.h"

namespace specache {
namespace {

constexpr int kI8Chunk = 512;                   // quantised tokens per workgroup
constexpr int kWaveTok = kI8Chunk / kWaves;     // 128
constexpr int kColStride = kWaveTok + 16;       // bytes between the B columns of a wave (pad: banks)
constexpr int kSetBytes = 16 * kColStride;      // the 16 columns (row, group of the set, plane) of a channel set
constexpr int kWaveArea = 2 * kSetBytes;        // bytes per wave; a set's results [2][4][4][16] int32 replace its columns
static_assert(kSetBytes >= 2 * 4 * 4 * 16 * 4, "a set's results reuse the set's operand columns");
static_assert(kWaveDwords * 4 >= kWaveArea, "the value phase reuses the scoring wave's exchange area");
constexpr int kWaveBitmapTopk = 256;            // up to here every wave builds the bitmap of its own tokens

// sum / max over the 8 lanes that share (sub-group, h): lanes differ in their low three bits
__device__ __forceinline__ float sum8(float v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    return v + dpp_move<kDppHalfMirror>(v);
}
__device__ __forceinline__ float max8(float v) {
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    return fmaxf(v, dpp_move<kDppHalfMirror>(v));
}

// what the waves of a workgroup hand to the merge
struct WaveOut {
    float m[kWaves][2];            // softmax maximum of the wave's tokens, per row
    float unscale[kWaves];         // 1 / fixed-point scale of the wave's B operands
    float part[kWaves][4][2][5];   // per (wave, sub-group, h): zero-point sums [rows x groups of the lane], cell 4: sum of row h
};

// The lane's share of a wave's value-side loads: packed codes of 16 tokens x 4 channels for two token steps
// and two channel sets, and (min, max) words.  The metadata is stored per token ([token][group]); every lane
// requests consecutive 16 bytes of it (so that a load instruction covers whole cache lines) and the wave
// then hands the words through its LDS area to the lanes that use them: the groups of channel set h for
// the lane's four tokens (value_meta_exchange).
template <int GROUP, int BITS>
struct ValueLoads {
    static constexpr int M = kD / GROUP, MPL = M >= 2 ? M / 2 : 1;
    uint4 vw[2][BITS];           // [token step][channel set] with 2 bits; one word per token step holds all channels with 1
    uint4 raw[M == 4 ? 2 : 1];
    uint32_t mw[4][MPL];
};

template <int GROUP, int BITS>
__device__ __forceinline__ void value_loads(const LayerView& L, int row, int c0, int w0, int nw, int lane, ValueLoads<GROUP, BITS>& v) {
    constexpr int M = kD / GROUP;
    const int sg = lane >> 4, l16 = lane & 15;
    const bool live = 32 * sg < nw;
    const size_t tok = (size_t)c0 + w0 + 32 * sg;                      // the sub-group's first token
    const uint32_t* vm_row = L.vm + (size_t)row * L.vm_stride;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    if constexpr (M == 4) {            // 16 bytes per token: lane l16 takes tokens l16 and 16 + l16
        v.raw[0] = live ? *reinterpret_cast<const uint4*>(vm_row + (tok + l16) * 4) : zero;
        v.raw[1] = live ? *reinterpret_cast<const uint4*>(vm_row + (tok + 16 + l16) * 4) : zero;
    } else if constexpr (M == 2) {     // 8 bytes per token: tokens 2 l16 and 2 l16 + 1
        v.raw[0] = live ? *reinterpret_cast<const uint4*>(vm_row + (tok + 2 * l16) * 2) : zero;
    } else {                           // 4 bytes per token: the lane's own four tokens
        v.raw[0] = (32 * sg + 4 * (lane & 7)) < nw ? *reinterpret_cast<const uint4*>(vm_row + tok + 4 * (lane & 7)) : zero;
    }
    // codes: lane (il = lane % 16, tg = lane / 16) reads, for token step ks and channel set s, the 16 tokens
    // 64 ks + 16 tg .. + 15 of code lane 16 s + il (channels 4 (16 s + il) .. + 3); with 1-bit codes of code
    // lane il (channels 8 il .. + 7)
    const int il = lane & 15, tg = lane >> 4;
    const uint8_t* vc_row = L.vc + (size_t)row * L.vc_stride;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int tw = 64 * ks + 16 * tg;                                  // inside the wave
        const size_t t16 = tw < nw ? (size_t)c0 + w0 + tw : (size_t)c0;    // past the end: the chunk's first tokens (p = 0 there)
        const uint8_t* base = vc_row + (t16 / kBlockTokens) * code_block_bytes(BITS) + ((t16 / 16) & 1) * (256 * BITS);
#pragma unroll
        for (int s = 0; s < BITS; ++s) v.vw[ks][s] = *reinterpret_cast<const uint4*>(base + (16 * s + il) * 16);
    }
}

// Metadata words from the lanes that loaded them to the lanes that use them, through the wave's LDS area
// (free at that point): [h][128 tokens] cells of the groups of channel set h, written per token, read as the
// lane's four consecutive tokens.
template <int GROUP, int BITS>
__device__ __forceinline__ void value_meta_exchange(ValueLoads<GROUP, BITS>& v, int lane, uint8_t* area) {
    constexpr int M = kD / GROUP;
    const int sg = lane >> 4, l16 = lane & 15, h = (lane >> 3) & 1, t0 = 32 * sg + 4 * (lane & 7);
    if constexpr (M == 4) {
        uint2* cells = reinterpret_cast<uint2*>(area);                 // [2][128] x 8 bytes
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int t = 32 * sg + 16 * e + l16;
            cells[t] = make_uint2(v.raw[e].x, v.raw[e].y);
            cells[128 + t] = make_uint2(v.raw[e].z, v.raw[e].w);
        }
        wave_sync();
        const uint4 a = *reinterpret_cast<const uint4*>(cells + 128 * h + t0), b = *reinterpret_cast<const uint4*>(cells + 128 * h + t0 + 2);
        v.mw[0][0] = a.x; v.mw[0][1] = a.y; v.mw[1][0] = a.z; v.mw[1][1] = a.w;
        v.mw[2][0] = b.x; v.mw[2][1] = b.y; v.mw[3][0] = b.z; v.mw[3][1] = b.w;
        wave_sync();
    } else if constexpr (M == 2) {
        uint32_t* cells = reinterpret_cast<uint32_t*>(area);           // [2][128] x 4 bytes
        const int t = 32 * sg + 2 * l16;
        cells[t] = v.raw[0].x;
        cells[128 + t] = v.raw[0].y;
        cells[t + 1] = v.raw[0].z;
        cells[128 + t + 1] = v.raw[0].w;
        wave_sync();
        const uint4 a = *reinterpret_cast<const uint4*>(cells + 128 * h + t0);
        v.mw[0][0] = a.x; v.mw[1][0] = a.y; v.mw[2][0] = a.z; v.mw[3][0] = a.w;
        wave_sync();
    } else {
        v.mw[0][0] = v.raw[0].x; v.mw[1][0] = v.raw[0].y; v.mw[2][0] = v.raw[0].z; v.mw[3][0] = v.raw[0].w;
    }
}

// Bits of the wave's 128 tokens that the staged index list names (they enter through the 16-bit chunks),
// built by the wave alone from an index list of at most 256 entries: the lane's four entries are requested
// with wave_bitmap_loads (positions relative to the wave's first token, -1 = none) and turned into wbits[4]
// by wave_bitmap_apply, once other loads are under way.
__device__ __forceinline__ void wave_bitmap_loads(const int32_t* __restrict__ idx_row, int topk, int first, int lane, int t[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int j = 64 * u + lane;
        t[u] = (idx_row && j < topk) ? idx_row[j] - first : -1;
    }
}
__device__ __forceinline__ void wave_bitmap_apply(const int t[4], int nw, int lane, uint32_t* wbits) {
    if (lane < 4) wbits[lane] = 0u;
    wave_sync();
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (t[u] >= 0 && t[u] < nw) atomicOr(&wbits[t[u] >> 5], 1u << (t[u] & 31));
    wave_sync();
}

// The value side of one wave: softmax numerators relative to the wave's maximum, B operands, zero-point and
// row sums, the contraction, and the results left in the wave's area for the merge.  lgv: the logits of the
// lane's four tokens of row h (-inf where not a candidate).  nw > 0.
template <int GROUP, int BITS, bool BF16>
__device__ __forceinline__ void value_wave(const ValueLoads<GROUP, BITS>& v, float lgv[4], bool one_bit_plain, int wave, int lane,
                                           uint8_t* area, WaveOut& out) {
    constexpr int M = kD / GROUP;                 // value groups per token: 4, 2, 1
    constexpr int MPL = M >= 2 ? M / 2 : 1;       // groups a lane prepares
    constexpr int RPL = M >= 2 ? 2 : 1;           // rows a lane prepares (one group only: each lane its own row)
    const int sg = lane >> 4, h = (lane >> 3) & 1, tg = lane >> 4;
    const int t0 = 32 * sg + 4 * (lane & 7);

    float mloc = fmaxf(fmaxf(lgv[0], lgv[1]), fmaxf(lgv[2], lgv[3]));
    mloc = max8(mloc);
    float mrow[2];
#pragma unroll
    for (int r = 0; r < 2; ++r)
        mrow[r] = fmaxf(fmaxf(lane_value(mloc, 8 * r), lane_value(mloc, 16 + 8 * r)),
                        fmaxf(lane_value(mloc, 32 + 8 * r), lane_value(mloc, 48 + 8 * r)));
    const float m_own = h ? mrow[1] : mrow[0];
    const float ms = m_own == -INFINITY ? 0.0f : m_own;
    float p[4], psum = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        p[j] = __expf(lgv[j] - ms);
        psum += p[j];
    }
    // numerators of both rows for the lane's tokens: pr[r][j]
    float pr[2][4];
    if constexpr (RPL == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float other = dpp_move<kDppRowRor8>(p[j]);
            pr[0][j] = h ? other : p[j];
            pr[1][j] = h ? p[j] : other;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) pr[0][j] = p[j];   // the lane's own row only
    }

    // scale and zero-point of the lane's (token, group) pairs; the wave's largest scale
    float sc[4][MPL], zp[4][MPL], smax = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int ml = 0; ml < MPL; ++ml) {
            derive_scale_zero<BITS>(widen16<BF16>(v.mw[j][ml] & 0xFFFFu), widen16<BF16>(v.mw[j][ml] >> 16), one_bit_plain, sc[j][ml], zp[j][ml]);
            smax = fmaxf(smax, sc[j][ml]);
        }
    const float top = wave_max(smax);
    // top < 2^(E - 126) with E its exponent field, p <= 1: p s 2^(156 - E) stays below 2^30
    uint32_t E = __float_as_uint(top) >> 23;
    E = E < 30u ? 30u : (E > 254u ? 254u : E);
    const float up = __uint_as_float((283u - E) << 23);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int ml = 0; ml < MPL; ++ml) sc[j][ml] *= up;

    // B columns: byte planes of p s, four tokens per dword; zero-point sums.  Column (set, row, group of the
    // set, plane); with one value group per token each lane fills its own row's columns of both sets.
    float zacc[RPL][MPL];
#pragma unroll
    for (int r = 0; r < RPL; ++r)
#pragma unroll
        for (int ml = 0; ml < MPL; ++ml) {
            uint32_t y[4], planes[4];
            float za = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                y[j] = ((uint32_t)(int)(pr[r][j] * sc[j][ml]) + 0x00808080u) ^ 0x00808080u;
                za = __builtin_fmaf(pr[r][j], zp[j][ml], za);
            }
            zacc[r][ml] = za;
            byte_planes(y[0], y[1], y[2], y[3], planes);
            const int rr = RPL == 2 ? r : h;
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                if constexpr (M >= 2) {
                    *reinterpret_cast<uint32_t*>(area + (((h * 2 + rr) * 2 + ml) * 4 + pp) * kColStride + t0) = planes[pp];
                } else {
                    *reinterpret_cast<uint32_t*>(area + ((rr * 2) * 4 + pp) * kColStride + t0) = planes[pp];
                    *reinterpret_cast<uint32_t*>(area + kSetBytes + ((rr * 2) * 4 + pp) * kColStride + t0) = planes[pp];
                }
            }
        }
    // partial sums of the 8 lanes that share (sub-group, h); the merge adds them up
    psum = sum8(psum);
#pragma unroll
    for (int r = 0; r < RPL; ++r)
#pragma unroll
        for (int ml = 0; ml < MPL; ++ml) zacc[r][ml] = sum8(zacc[r][ml]);
    if ((lane & 7) == 0) {
        float* dst = out.part[wave][sg][h];
#pragma unroll
        for (int r = 0; r < RPL; ++r)
#pragma unroll
            for (int ml = 0; ml < MPL; ++ml) dst[r * MPL + ml] = zacc[r][ml];
        dst[4] = psum;
    }
    if (lane == 0) {
        out.m[wave][0] = mrow[0];
        out.m[wave][1] = mrow[1];
        out.unscale[wave] = __uint_as_float((E - 29u) << 23);   // 2^(E - 156) = 1 / up
    }
    wave_sync();

    // the contraction, one channel set at a time: per token step one B operand and the masks of the code bytes
    const int bn = lane & 15;
    const int brow = bn >> 3, bml = (bn >> 2) & 1, bpp = bn & 3;
    if constexpr (BITS == 2) {
        // Result register e of lane (column bn, quarter tg) is MFMA row 4 tg + e: code lane 16 s + 4 tg + e, i.e.
        // channel 64 s + 16 tg + 4 e + j, whose value group is 2 s + tg / 2 (g = 32), s (g = 64) or 0.  The columns
        // of that group are kept: [row][plane][j][16 rows] int32 per set.
        const bool keep = M == 4 ? bml == (tg >> 1) : bml == 0;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v4i acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = (v4i){0, 0, 0, 0};
            uint8_t* set = area + s * kSetBytes;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const v4i b = *reinterpret_cast<const v4i*>(set + ((brow * 2 + (M == 4 ? bml : 0)) * 4 + bpp) * kColStride + 64 * ks + 16 * tg);
                const uint4 w = v.vw[ks][s];
                const uint4 t = make_uint4(w.x >> 4, w.y >> 4, w.z >> 4, w.w >> 4);
                const v4i a0 = {(int)(w.x & 0x03030303u), (int)(w.y & 0x03030303u), (int)(w.z & 0x03030303u), (int)(w.w & 0x03030303u)};
                const v4i a1 = {(int)(w.x & 0x0C0C0C0Cu), (int)(w.y & 0x0C0C0C0Cu), (int)(w.z & 0x0C0C0C0Cu), (int)(w.w & 0x0C0C0C0Cu)};
                const v4i a2 = {(int)(t.x & 0x03030303u), (int)(t.y & 0x03030303u), (int)(t.z & 0x03030303u), (int)(t.w & 0x03030303u)};
                const v4i a3 = {(int)(t.x & 0x0C0C0C0Cu), (int)(t.y & 0x0C0C0C0Cu), (int)(t.z & 0x0C0C0C0Cu), (int)(t.w & 0x0C0C0C0Cu)};
                acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a2, b, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a3, b, acc[3], 0, 0, 0);
            }
            wave_sync();   // every lane has read the set's B operands: its columns are free for the results
            if (keep) {
                int* res = reinterpret_cast<int*>(set);
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<v4i*>(res + (((brow * 4 + bpp) * 4 + j) * 16 + 4 * tg)) = acc[j];
            }
        }
    } else {
        // MFMA row 4 tg + e is code lane 4 tg + e, channels 8 (4 tg + e) .. + 7: channel half (set) tg / 2, value
        // group tg (g = 32), tg / 2 (g = 64) or 0.  Each set's columns run against all 16 code lanes and the 8 of
        // the set are kept: [row][plane][j = 0..7][8 code lanes] int32 per set, the size of the 2-bit results.
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint8_t* set = area + s * kSetBytes;
            v4i b[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                b[ks] = *reinterpret_cast<const v4i*>(set + ((brow * 2 + (M == 4 ? bml : 0)) * 4 + bpp) * kColStride + 64 * ks + 16 * tg);
            wave_sync();   // every lane holds the set's B operands: its columns are free for the results
            const bool keep = (tg >> 1) == s && (M == 4 ? bml == (tg & 1) : bml == 0);
#pragma unroll
            for (int jh = 0; jh < 2; ++jh) {
                v4i acc[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = (v4i){0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    uint4 w = v.vw[ks][0];
                    if (jh) w = make_uint4(w.x >> 4, w.y >> 4, w.z >> 4, w.w >> 4);
                    const v4i a0 = {(int)(w.x & 0x01010101u), (int)(w.y & 0x01010101u), (int)(w.z & 0x01010101u), (int)(w.w & 0x01010101u)};
                    const v4i a1 = {(int)(w.x & 0x02020202u), (int)(w.y & 0x02020202u), (int)(w.z & 0x02020202u), (int)(w.w & 0x02020202u)};
                    const v4i a2 = {(int)(w.x & 0x04040404u), (int)(w.y & 0x04040404u), (int)(w.z & 0x04040404u), (int)(w.w & 0x04040404u)};
                    const v4i a3 = {(int)(w.x & 0x08080808u), (int)(w.y & 0x08080808u), (int)(w.z & 0x08080808u), (int)(w.w & 0x08080808u)};
                    acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b[ks], acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b[ks], acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a2, b[ks], acc[2], 0, 0, 0);
                    acc[3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a3, b[ks], acc[3], 0, 0, 0);
                }
                if (keep) {
                    int* res = reinterpret_cast<int*>(set);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        *reinterpret_cast<v4i*>(res + (((brow * 4 + bpp) * 8 + 4 * jh + j) * 8 + 4 * (tg & 1))) = acc[j];
                }
            }
        }
    }
}

// a wave without tokens contributes nothing, in finite numbers
__device__ __forceinline__ void empty_wave(int wave, int lane, WaveOut& out) {
    if (lane < 40) (&out.part[wave][0][0][0])[lane] = 0.0f;
    if (lane == 0) {
        out.m[wave][0] = -INFINITY;
        out.m[wave][1] = -INFINITY;
        out.unscale[wave] = 0.0f;
    }
}

// Merge of the four waves of a chunk (after a workgroup barrier): thread = (row r, channel c).
template <int GROUP, int BITS>
__device__ __forceinline__ void merge_waves(const uint8_t* areas, int area_stride, const WaveOut& out, int tid, float* po,
                                            float* pml) {
    constexpr int M = kD / GROUP, MPL = M >= 2 ? M / 2 : 1;
    const int r = tid >> 7, c = tid & 127;
    // where the channel's sums sit in its set's results: 2 bits [row][plane][j = c % 4][code lane (c / 4) % 16],
    // 1 bit [row][plane][j = c % 8][code lane (c / 8) % 8]
    const int s = c >> 6, i = BITS == 2 ? (c >> 2) & 15 : (c >> 3) & 7, j = BITS == 2 ? c & 3 : c & 7;
    constexpr int NJ = BITS == 2 ? 4 : 8, NI = BITS == 2 ? 16 : 8;
    const int m = c / GROUP;
    const int hh = M >= 2 ? m / MPL : r, zi = M >= 2 ? r * MPL + m % MPL : 0;   // where the zero-point sum of (r, m) sits
    float mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mmax = fmaxf(mmax, out.m[w][r]);
    float o = 0.0f, lsum = 0.0f;
    // the masks leave a code where it sits in its nibble: 4 x code for odd channels (2 bits), 2^(c % 4) x code (1 bit)
    const float jscale = BITS == 2 ? ((j & 1) ? 0.25f : 1.0f) : __uint_as_float((uint32_t)(127 - (j & 3)) << 23);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const float mwv = out.m[w][r];
        const float e = mwv == -INFINITY ? 0.0f : __expf(mwv - mmax);
        const int* res = reinterpret_cast<const int*>(areas + w * area_stride + s * kSetBytes);
        float f[4];
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) f[pp] = (float)res[((r * 4 + pp) * NJ + j) * NI + i];
        float t = __builtin_fmaf(f[1], 256.0f, f[0]);
        t = __builtin_fmaf(f[2], 65536.0f, t);
        t = __builtin_fmaf(f[3], 16777216.0f, t);
        float zs = 0.0f, ls = 0.0f;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            zs += out.part[w][g4][hh][zi];
            ls += out.part[w][g4][r][4];
        }
        // a wave without tokens left its area as it was: whatever integers sit there are finite and weigh 0
        const float val = __builtin_fmaf(t, out.unscale[w] * jscale, zs);
        o = __builtin_fmaf(e, val, o);
        lsum = __builtin_fmaf(e, ls, lsum);
    }
    po[r * kD + c] = o;
    if (c == 0) {
        pml[2 * r] = mmax;
        pml[2 * r + 1] = lsum;
    }
}

// (row, chunk) of this workgroup: the 16-bit chunks are chains of dependent loads and are dispatched first
__device__ __forceinline__ void chunk_of_block(const AttendArgs& A, int rows, int bid, int& row, int& chunk) {
    const int n_extra = A.n_chunks - A.n_main;
    if (bid < rows * n_extra) {
        row = bid / n_extra;
        chunk = A.n_main + bid % n_extra;
    } else {
        const int id = bid - rows * n_extra;
        row = id / A.n_main;
        chunk = id % A.n_main;
    }
}

// Workgroup-wide bitmap of the chunk's staged positions, for index lists too long for every wave to walk
__device__ __forceinline__ void chunk_bitmap(const AttendArgs& A, int topk, int row, int c0, int n, int tid, uint32_t* maskbits) {
    if (tid < kI8Chunk / 32) maskbits[tid] = 0u;
    __syncthreads();
    if (A.slot_idx)
        for (int j = tid; j < topk; j += kThreads) {
            const int t = A.slot_idx[(size_t)row * topk + j] - c0;
            if (t >= 0 && t < n) atomicOr(&maskbits[t >> 5], 1u << (t & 31));
        }
    __syncthreads();
}

// Registers: the pass that also scores needs 84 to 88 (five waves per SIMD); compiled for six or eight it
// spills and runs slower (measured at the 7B shape: 28.6 us, 32 with two registers spilled, 58 with 34).
template <int GROUP, int BITS, bool BF16, bool FUSED>
__global__ __launch_bounds__(kThreads) void attend_i8_kernel(LayerView L, AttendArgs A, float sm_scale, uint32_t* __restrict__ keys,
                                                             size_t key_stride) {
    constexpr int NR = 2;
    constexpr int kAreaBytes = FUSED ? kWaveDwords * 4 : kWaveArea;        // per wave
    constexpr int kRegion = (kWaves * kAreaBytes) / 4 > extra_chunk_floats(NR) ? (kWaves * kAreaBytes) / 4 : extra_chunk_floats(NR);
    __shared__ __attribute__((aligned(16))) float smem[kRegion];
    __shared__ float red[kWaves * NR];
    __shared__ uint32_t maskbits[kI8Chunk / 32];
    __shared__ __attribute__((aligned(8))) float2 fin[FUSED ? kWaves : 1][4][2];
    __shared__ WaveOut wout;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n_tail = L.tail_k ? L.rows : 0;
    if ((int)blockIdx.x < n_tail) {
        // a launch that also appends the step's new token (Appendix A "Decoding": Offload of the new pair to the
        // CPU copy; it also joins the 16-bit residual): one more workgroup per row, 32 lanes x 16 bytes.  They are
        // dispatched first: the store to host memory crosses a link the prefetch keeps busy, and the launch
        // ends only when it has landed.
        const int r = blockIdx.x;
        if (tid < 32) {
            const uint4 v = reinterpret_cast<const uint4*>(tid < 16 ? L.tail_k : L.tail_v)[(size_t)r * 16 + (tid & 15)];
            reinterpret_cast<uint4*>(L.host)[((size_t)r * L.max_seq + L.tail_N0) * 32 + tid] = v;
            reinterpret_cast<uint4*>(L.ring)[((size_t)r * L.R + (L.tail_N0 % L.R)) * 32 + tid] = v;
        }
        return;
    }
    int row, chunk;
    chunk_of_block(A, L.rows, (int)blockIdx.x - n_tail, row, chunk);
    float* po = A.part_o + (((size_t)row * A.max_chunks + chunk) * NR) * kD;
    float* pml = A.part_ml + (((size_t)row * A.max_chunks + chunk) * NR) * 2;

    if (chunk >= A.n_main) {
        float m_row[NR], l_row[NR];
        attend_extra_chunk<NR, 2, BF16>(L, A, row, chunk, smem, red, m_row, l_row, po);
        if (tid < NR) {
            pml[2 * tid] = tid == 0 ? m_row[0] : m_row[1];
            pml[2 * tid + 1] = tid == 0 ? l_row[0] : l_row[1];
        }
        return;
    }

    // ------------------------------------------------------------------ quantised positions
    const int c0 = chunk * kI8Chunk;
    const int n = (A.Nq - c0) < kI8Chunk ? (A.Nq - c0) : kI8Chunk;   // multiple of 32, >= 32
    const int w0 = kWaveTok * wave;                                    // first token of the wave inside the chunk
    int nw = n - w0;                                                   // its valid tokens
    nw = nw < 0 ? 0 : (nw > kWaveTok ? kWaveTok : nw);
    const int sg = lane >> 4, h = (lane >> 3) & 1;
    const int t0 = 32 * sg + 4 * (lane & 7);                           // first of the lane's four tokens inside the wave
    const bool live = t0 < nw;
    uint8_t* area = reinterpret_cast<uint8_t*>(smem) + wave * kAreaBytes;
    const bool wave_maps = L.topk <= kWaveBitmapTopk;                  // uniform over the launch
    if (!wave_maps) chunk_bitmap(A, L.topk, row, c0, n, tid, maskbits);

    if (nw > 0) {   // wave-uniform
        ValueLoads<GROUP, BITS> v;
        float lgv[4];
        // everything this wave reads from global memory is requested before the first wait on any of it
        int ti[4];
        if (wave_maps) wave_bitmap_loads(A.slot_idx ? A.slot_idx + (size_t)row * L.topk : nullptr, L.topk, c0 + w0, lane, ti);
        if constexpr (!FUSED) {
            float4 lg4 = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (live) lg4 = *reinterpret_cast<const float4*>(A.logits + ((size_t)row * NR + h) * A.logit_stride + c0 + w0 + t0);
            value_loads<GROUP, BITS>(L, row, c0, w0, nw, lane, v);
            if (wave_maps) wave_bitmap_apply(ti, nw, lane, maskbits + 4 * wave);
            lgv[0] = lg4.x; lgv[1] = lg4.y; lgv[2] = lg4.z; lgv[3] = lg4.w;
        } else {
            // the low-bit logits of the wave's tokens (Appendix A "Decoding": A = Q K^T on C'); the value-side loads
            // are requested once the scoring operands are built and travel while the scoring contraction runs
            score_i8_wave<BITS, BF16>(L, A.q, row, chunk, wave, lane, A.Nq / kBlockTokens, sm_scale, reinterpret_cast<uint32_t*>(area),
                                   fin[wave], lgv,
                                   [&]() { if (wave_maps) wave_bitmap_apply(ti, nw, lane, maskbits + 4 * wave); },
                                   [&]() { value_loads<GROUP, BITS>(L, row, c0, w0, nw, lane, v); });
            if (live) {
                if (h == 1)   // the speculative row ranks the positions
                    *reinterpret_cast<uint4*>(keys + (size_t)row * key_stride + c0 + w0 + t0) =
                        make_uint4(float_to_key(lgv[0]), float_to_key(lgv[1]), float_to_key(lgv[2]), float_to_key(lgv[3]));
                if (A.logits_out)   // kept only when the caller asked for them (parity hook)
                    *reinterpret_cast<float4*>(A.logits_out + ((size_t)row * NR + h) * A.logit_stride + c0 + w0 + t0) =
                        make_float4(lgv[0], lgv[1], lgv[2], lgv[3]);
            }
            wave_sync();   // the scoring exchange is over: the area now serves the value side
        }
        value_meta_exchange<GROUP, BITS>(v, lane, area);
        const uint32_t mbits = maskbits[4 * wave + sg] >> (4 * (lane & 7));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (!live || ((mbits >> j) & 1u)) lgv[j] = -INFINITY;
        value_wave<GROUP, BITS, BF16>(v, lgv, L.one_bit_plain, wave, lane, area, wout);
    } else {
        empty_wave(wave, lane, wout);
    }
    __syncthreads();
    merge_waves<GROUP, BITS>(reinterpret_cast<const uint8_t*>(smem), kAreaBytes, wout, tid, po, pml);
}

}  // namespace

bool attend_uses_int8_matrix_cores(const LayerView& L, int n_rows) { return L.G == 1 && n_rows == 2 && (L.bits == 2 || L.bits == 1); }

// keys != null: the scoring pass runs inside the launch (logits are not read; they are written to logits_out if set)
hipError_t launch_attend_i8_partial(const LayerView& L, const void* q, int N, int Nq, float sm_scale, const float* logits,
                                    size_t logit_stride, const uint16_t* slot, const int32_t* slot_idx, const void* k_spec,
                                    const void* v_spec, const AttendScratch& scratch, uint32_t* keys, size_t key_stride,
                                    float* logits_out, hipStream_t stream) {
    if (!attend_uses_int8_matrix_cores(L, 2) || Nq % kBlockTokens) return hipErrorInvalidValue;
    AttendArgs A;
    A.q = (const uint16_t*)q;
    A.logits = logits;
    A.logits_out = logits_out;
    A.logit_stride = logit_stride;
    A.slot = slot;
    A.slot_idx = slot_idx;
    A.k_spec = (const uint16_t*)k_spec;
    A.v_spec = (const uint16_t*)v_spec;
    A.part_o = scratch.part_o;
    A.part_ml = scratch.part_ml;
    A.max_chunks = scratch.max_chunks;
    A.N = N;
    A.Nq = Nq;
    A.sm_scale = sm_scale;
    const int n_ex = (slot_idx ? L.topk : 0) + (N - Nq) + (k_spec ? 1 : 0);
    A.n_main = (Nq + kI8Chunk - 1) / kI8Chunk;
    A.n_chunks = A.n_main + (n_ex + kExtraChunk - 1) / kExtraChunk;
    if (A.n_chunks > A.max_chunks || A.n_chunks < 1) return hipErrorInvalidValue;
    const dim3 grid(A.n_chunks * L.rows + (L.tail_k ? L.rows : 0)), block(kThreads);
#define SPC_AI8_B(G_, B_, F_)                                                                                              \
    do {                                                                                                                   \
        if (keys) SPC_LAUNCH((attend_i8_kernel<G_, B_, F_, true>), grid, block, stream, L, A, sm_scale, keys, key_stride); \
        else SPC_LAUNCH((attend_i8_kernel<G_, B_, F_, false>), grid, block, stream, L, A, sm_scale, keys, key_stride);     \
    } while (0)
#define SPC_AI8(G_, F_)                    \
    do {                                   \
        if (L.bits == 2) SPC_AI8_B(G_, 2, F_); \
        else SPC_AI8_B(G_, 1, F_);         \
    } while (0)
    if (L.group == 32) { if (L.bf16) SPC_AI8(32, true); else SPC_AI8(32, false); }
    else if (L.group == 64) { if (L.bf16) SPC_AI8(64, true); else SPC_AI8(64, false); }
    else if (L.group == 128) { if (L.bf16) SPC_AI8(128, true); else SPC_AI8(128, false); }
    else return hipErrorInvalidValue;
#undef SPC_AI8_B
#undef SPC_AI8
    return hipGetLastError();
}

}  // namespace specache
