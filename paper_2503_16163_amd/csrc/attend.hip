// Mixed attention of Eq. 1 (Section 3.3): Attn([T_t, T'_{t+1}], C' u C_K).
//
// Candidates of a query row: quantised positions i < Nq (the prefetched 16-bit
// pair where i is in the slot's index list, the dequantised low-bit pair
// elsewhere), the 16-bit residual positions, and for the speculative row its own
// transient pair.  The low-bit logits were kept by the scoring pass.
//
// Split over the sequence: "main" workgroups take chunks of quantised positions,
// "extra" workgroups take the 16-bit candidates (staged pairs, residual, transient
// pair); each writes an un-normalised partial (max, sum, sum p*V) and a combine
// kernel merges them with the usual log-sum-exp rescaling.  Prefetched positions
// are removed from the main chunks by setting their logit to -inf in LDS; the
// staged pair then enters through the extra chunks, which is Eq. 1's "replace".
//
// Values are quantised per token over g channels, so for the main chunks
//   sum_i p_i V'[i][c] = sum_i (p_i s[i][m]) code[i][c] + sum_i p_i z[i][m],  m = c / g.
// With up to four query rows per KV head the first sum runs on the vector ALUs: a lane owns
// 8/BITS channels and reads 16 tokens of them as one 16-byte load; p_i s[i][m] comes from
// LDS (computed once per token by the softmax phase).  With 8 or 16 rows it is a dense
// enough contraction for the matrix cores (v_mfma_f32_16x16x32_f16, fp32 accumulation):
// the codes enter as f16 subnormals straight from the packed bytes, p_i s[i][m] as a
// hi + lo pair of f16.
#include "attend_common.h"

namespace specache {
namespace {

__host__ __device__ constexpr int main_chunk(int NR) { return NR <= 8 ? 512 : 256; }

template <int BITS, int GROUP, int G, int NROWS, bool BF16>
__global__ __launch_bounds__(kThreads) void attend_partial_kernel(LayerView L, AttendArgs A) {
    constexpr int NR = G * NROWS;
    constexpr int CH = main_chunk(NR);
    constexpr int M = kD / GROUP;            // value groups per token
    constexpr int CPB = 8 / BITS;            // channels per code byte (per lane)
    constexpr int LPB = 32 * BITS;           // lanes per 32-token block
    constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x01010101u;
    constexpr int TPT = (CH + kThreads - 1) / kThreads;   // chunk tokens per thread
    // With up to four query rows the value side runs on the vector ALUs, with more on the matrix
    // cores (kSplit).  One LDS region serves, in turn: for main chunks ps[M][CH][NR] (vector
    // path) or the planes p[CH][NR+1], z[CH][M], s[CH][M] (matrix path); for extra chunks
    // the areas of attend_extra_chunk; at the end o_lds[kWaves][NR][128] (vector path).
    // ps is stored in cells [16-token half block][value group m] of 16*NR floats plus one
    // 16-byte pad: the lanes of one LDS read differ only in (half block, m), i.e. in
    // consecutive cells, and the pad spreads those over distinct banks.
    constexpr bool kSplit = NR > 4;
    constexpr int kCell = 16 * NR + 4;
    constexpr int kPl = NR + 1;              // row pitch of the p plane: lanes of one read in distinct banks
    constexpr int kPlanes = CH * kPl + 2 * CH * M;
    constexpr int kPs = kSplit ? kPlanes : (CH / 16) * M * kCell, kOl = kWaves * NR * kD;
    // a workgroup is either a main or an extra chunk (16-bit candidates, attend_extra_chunk): both use
    // the one region, and LDS per workgroup decides how many chunks are resident per compute unit
    constexpr int kExtra = extra_chunk_floats(NR);
    constexpr int kMax1 = kExtra > kPs ? kExtra : kPs;
    constexpr int RH = NR;
    constexpr int kRegion = kMax1 > kOl ? kMax1 : kOl;
    __shared__ __attribute__((aligned(16))) float smem[kRegion];
    __shared__ float red[kWaves * NR * (1 + M)];
    __shared__ float red_sum[kWaves * NR];
    __shared__ float red_z[kWaves * NR * M];
    __shared__ float red_scale[kWaves];
    __shared__ uint32_t maskbits[CH / 32];

    float* ps = smem;                        // [CH/16][M] cells
    float* o_lds = smem;                     // [kWaves][NR][128]

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    // The 16-bit chunks are chains of dependent loads: they are dispatched first (all rows), the
    // quantised chunks after them.
    const int n_extra = A.n_chunks - A.n_main, rows = L.rows;
    int row, chunk;
    if ((int)blockIdx.x < rows * n_extra) {
        row = blockIdx.x / n_extra;
        chunk = A.n_main + blockIdx.x % n_extra;
    } else {
        const int id = blockIdx.x - rows * n_extra;
        row = id / A.n_main;
        chunk = id % A.n_main;
    }
    float m_row[NR], l_row[NR];
    float* po = A.part_o + (((size_t)row * A.max_chunks + chunk) * NR) * kD;
    float* pml = A.part_ml + (((size_t)row * A.max_chunks + chunk) * NR) * 2;

    if (chunk < A.n_main) {
        // ------------------------------------------------------------ quantised positions
        const int c0 = chunk * CH;
        const int n = (A.Nq - c0) < CH ? (A.Nq - c0) : CH;   // multiple of 32
        const uint8_t* vc_row = L.vc + (size_t)row * L.vc_stride + (size_t)(c0 / kBlockTokens) * code_block_bytes(BITS);
        const uint32_t* vm_row = L.vm + (size_t)row * L.vm_stride;
        const int units = (n / kBlockTokens) * LPB;
        const int within = lane % LPB;                       // position inside a block
        const int Lc = within % (16 * BITS);                 // code lane: channels Lc*CPB .. +CPB-1
        const int mgrp = (Lc * CPB) / GROUP;
        const uint8_t* vc_lane = vc_row + within * 16;

        // every global read this thread needs before the value loop is issued up front
        float lgr[TPT][NR];
        uint32_t meta[TPT][M];
#pragma unroll
        for (int tt = 0; tt < TPT; ++tt) {
            const int i = tid + tt * kThreads;
            const bool valid = i < n;
#pragma unroll
            for (int r = 0; r < NR; ++r)
                lgr[tt][r] = valid ? A.logits[((size_t)row * NR + r) * A.logit_stride + c0 + i] : -INFINITY;
            if constexpr (M == 4) {
                const uint4 t4 = valid ? *reinterpret_cast<const uint4*>(vm_row + (size_t)(c0 + i) * 4) : make_uint4(0, 0, 0, 0);
                meta[tt][0] = t4.x; meta[tt][1] = t4.y; meta[tt][2] = t4.z; meta[tt][3] = t4.w;
            } else if constexpr (M == 2) {
                const uint2 t2 = valid ? *reinterpret_cast<const uint2*>(vm_row + (size_t)(c0 + i) * 2) : make_uint2(0, 0);
                meta[tt][0] = t2.x; meta[tt][1] = t2.y;
            } else {
                meta[tt][0] = valid ? vm_row[c0 + i] : 0u;
            }
        }
        // the first value codes of this thread, needed only after the softmax phase
        uint4 w4_first = make_uint4(0, 0, 0, 0);
        if (tid < units) w4_first = *reinterpret_cast<const uint4*>(vc_lane + (size_t)(tid / LPB) * code_block_bytes(BITS));
        // prefetched positions of this chunk, as a bitmap (the first entries of the index list
        // are requested with the other loads)
        constexpr int kIdxUpfront = 2;
        int sidx[kIdxUpfront];
#pragma unroll
        for (int u = 0; u < kIdxUpfront; ++u) {
            const int j = tid + u * kThreads;
            sidx[u] = (A.slot_idx && j < L.topk) ? A.slot_idx[(size_t)row * L.topk + j] : -1;
        }
        if (tid < CH / 32) maskbits[tid] = 0u;
        __syncthreads();
        if (A.slot_idx) {
#pragma unroll
            for (int u = 0; u < kIdxUpfront; ++u) {
                const int t = sidx[u] - c0;
                if (sidx[u] >= 0 && t >= 0 && t < n) atomicOr(&maskbits[t >> 5], 1u << (t & 31));
            }
            for (int j = tid + kIdxUpfront * kThreads; j < L.topk; j += kThreads) {
                const int t = A.slot_idx[(size_t)row * L.topk + j] - c0;
                if (t >= 0 && t < n) atomicOr(&maskbits[t >> 5], 1u << (t & 31));
            }
        }
        __syncthreads();

        float mloc[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) mloc[r] = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < TPT; ++tt) {
            const int i = tid + tt * kThreads;
            const bool masked = i < n && ((maskbits[i >> 5] >> (i & 31)) & 1u);
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                if (masked) lgr[tt][r] = -INFINITY;
                mloc[r] = fmaxf(mloc[r], lgr[tt][r]);
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const float v = wave_max(mloc[r]);
            if (lane == 0) red[wave * NR + r] = v;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            float v = red[r];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) v = fmaxf(v, red[w * NR + r]);
            m_row[r] = v;
        }

        // p = exp(l - m); p * s per (token, value group); the zero-point term sum_i p_i z[i][m] and
        // the row sums sum_i p_i.  With up to four query rows every thread adds up its own tokens
        // and the waves reduce those sums.  With more rows a thread has one token and NR * (M + 1)
        // sums, too many wave reductions: p and z go to LDS instead (in the area the merged
        // outputs use later) and the lanes re-read them as (row, slice of this wave's tokens), so
        // that only the slices of a row are left to add up.
        float* pl = smem;                        // [CH][kPl]
        float* zl = pl + CH * kPl;               // [CH][M]
        float* sl = zl + CH * M;                 // [CH][M]
        float zacc[NR][M], sloc[NR];
        float sc_max = 0.0f;     // largest value scale of this thread's tokens (MFMA path: operand scaling)
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            sloc[r] = 0.0f;
#pragma unroll
            for (int m = 0; m < M; ++m) zacc[r][m] = 0.0f;
        }
#pragma unroll
        for (int tt = 0; tt < TPT; ++tt) {
            const int i = tid + tt * kThreads;
            if (i < n) {
                float p[NR];
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    const float ms = m_row[r] == -INFINITY ? 0.0f : m_row[r];
                    p[r] = __expf(lgr[tt][r] - ms);
                    if constexpr (kSplit) pl[i * kPl + r] = p[r];
                    else sloc[r] += p[r];
                }
                float scv[M], zv[M];
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    float sc, z;
                    derive_scale_zero<BITS>(widen16<BF16>(meta[tt][m] & 0xFFFFu), widen16<BF16>(meta[tt][m] >> 16), L.one_bit_plain, sc, z);
                    scv[m] = sc;
                    zv[m] = z;
                    if constexpr (kSplit) {
                        sc_max = fmaxf(sc_max, sc);
                    } else {
#pragma unroll
                        for (int r = 0; r < NR; ++r) {
                            ps[((i >> 4) * M + m) * kCell + (i & 15) * NR + r] = p[r] * sc;
                            zacc[r][m] = __builtin_fmaf(p[r], z, zacc[r][m]);
                        }
                    }
                }
                if constexpr (kSplit) {   // one vector store per plane and token
                    if constexpr (M == 4) {
                        *reinterpret_cast<float4*>(&zl[i * M]) = make_float4(zv[0], zv[1], zv[2], zv[3]);
                        *reinterpret_cast<float4*>(&sl[i * M]) = make_float4(scv[0], scv[1], scv[2], scv[3]);
                    } else if constexpr (M == 2) {
                        *reinterpret_cast<float2*>(&zl[i * M]) = make_float2(zv[0], zv[1]);
                        *reinterpret_cast<float2*>(&sl[i * M]) = make_float2(scv[0], scv[1]);
                    } else {
                        zl[i] = zv[0];
                        sl[i] = scv[0];
                    }
                }
            }
        }
        if constexpr (kSplit) {
            {
                const float v = wave_max(sc_max);
                if (lane == 0) red_scale[wave] = v;
            }
            __syncthreads();
            constexpr int S = 64 / NR;                    // slices per row inside a wave
            constexpr int T = (CH / kWaves) / S;          // tokens per lane
            static_assert(S == 8 || S == 4, "slice reduction below covers 4 or 8 adjacent lanes");
            const int r = lane / S, slice = lane % S;
            float sa = 0.0f, za[M];
#pragma unroll
            for (int m = 0; m < M; ++m) za[m] = 0.0f;
#pragma unroll
            for (int j = 0; j < T; ++j) {
                const int i = wave * (CH / kWaves) + j * S + slice;   // slices interleaved: one read's lanes in distinct banks
                if (i < n) {
                    const float pr = pl[i * kPl + r];
                    sa += pr;
#pragma unroll
                    for (int m = 0; m < M; ++m) za[m] = __builtin_fmaf(pr, zl[i * M + m], za[m]);
                }
            }
            sa += dpp_move<kDppXor1>(sa);
            sa += dpp_move<kDppXor2>(sa);
            if constexpr (S == 8) sa += dpp_move<kDppHalfMirror>(sa);
#pragma unroll
            for (int m = 0; m < M; ++m) {
                za[m] += dpp_move<kDppXor1>(za[m]);
                za[m] += dpp_move<kDppXor2>(za[m]);
                if constexpr (S == 8) za[m] += dpp_move<kDppHalfMirror>(za[m]);
            }
            if (slice == 0) {
                red_sum[wave * NR + r] = sa;
#pragma unroll
                for (int m = 0; m < M; ++m) red_z[(wave * NR + r) * M + m] = za[m];
            }
        } else {
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const float v = wave_sum(sloc[r]);
                if (lane == 0) red_sum[wave * NR + r] = v;
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    const float zv = wave_sum(zacc[r][m]);
                    if (lane == 0) red_z[(wave * NR + r) * M + m] = zv;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            float v = red_sum[r];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) v += red_sum[w * NR + r];
            l_row[r] = v;
        }

        if constexpr (kSplit) {
            // ---- value side on the matrix cores (8 or 16 query rows per KV head) ----
            // o[r][c] = sum_i code[i][c] * ps[i][m(c)][r] per 32-token block is a 16 x 32 x 16 product:
            // A = codes (rows: 16 channels of one value group, columns: 32 tokens), read from the
            // packed bytes as f16 subnormals (code << (8 - BITS), i.e. code * 2^(8 - BITS - 24), exact);
            // B = ps = p * s (from the planes), scaled by a power of two near the top of the f16
            // range and split into hi + lo f16 (columns: (row r, hi | lo)), C accumulates in fp32.  Wave w owns the 32
            // channels 32 w .. 32 w + 31 (two tiles, one value group), so no sums cross waves.
            constexpr int NT = NR / 8;                      // column tiles of 8 query rows x (hi, lo)
            constexpr int JT = CPB / 2;                     // codes of one byte that go to one tile
            constexpr int LW = 32 / CPB;                    // code lanes (bytes per token) of this wave's channels
            const int ic = lane & 15, kq = lane >> 4;
            const int Lrow = wave * LW + ic % LW;           // code lane of this A row; row's bit = BITS * (JT t + ic / LW)
            const int mw = (32 * wave) / GROUP;             // value group of this wave's channels
            float smax = red_scale[0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) smax = fmaxf(smax, red_scale[w]);
            // 2^(14 - exponent(smax)): the largest p * s (p <= 1) lands in [2^14, 2^15)
            uint32_t eb = (__float_as_uint(smax) >> 23) & 0xFFu;
            eb = eb < 15u ? 15u : (eb > 240u ? 240u : eb);
            const float bscale = __uint_as_float((268u - eb) << 23);
            float4v acc[2][NT];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[t][nt] = float4v{0.f, 0.f, 0.f, 0.f};
            // every code is lifted to the top bits of its byte before it is widened: the matrix
            // cores do not normalise subnormal inputs before they align the products of a dot
            // product, so a code left in the low bits (two significant bits under eight leading
            // zeros) loses the low end of its small products (measured: 3e-5 of the sum for codes
            // at bit 0, 2e-7 at bit 6)
            uint32_t amask[2], ashift[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int j = JT * t + ic / LW;
                amask[t] = MASK << (BITS * j);
                ashift[t] = (8 - BITS) - BITS * j;
            }
            const int nblk = n / kBlockTokens;
            // 8 tokens of code lane Lrow: half block kq / 2, bytes 8 (kq % 2) .. + 7
            const uint8_t* a_lane = vc_row + ((size_t)(kq >> 1) * (16 * BITS) + Lrow) * 16 + 8 * (kq & 1);
            uint2 aw = make_uint2(0, 0);
            if (nblk > 0) aw = *reinterpret_cast<const uint2*>(a_lane);
            for (int b = 0; b < nblk; ++b) {
                uint2 awn = make_uint2(0, 0);
                if (b + 1 < nblk) awn = *reinterpret_cast<const uint2*>(a_lane + (size_t)(b + 1) * code_block_bytes(BITS));
                // B: column (r, hi | lo) = lane % 16, tokens 32 b + 8 kq .. + 7
                const int i0 = b * kBlockTokens + 8 * kq;
                // the two lanes of a column share the work: the hi lane splits tokens 0..3, the lo
                // lane tokens 4..7, then each hands the other the halves of the other's kind
                const int hl = ic & 1, ih = i0 + 4 * hl;
                float sv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) sv[e] = sl[(ih + e) * M + mw] * bscale;
                uint4v bop[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int r = 8 * nt + (ic >> 1);
                    float x[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = pl[(ih + e) * kPl + r] * sv[e];
                    uint32_t keep[2], send[2];
#pragma unroll
                    for (int e2 = 0; e2 < 2; ++e2) {
                        // hi by truncation, lo = x - hi rounded: hi + lo is x to 2^-21
                        const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(x[2 * e2], x[2 * e2 + 1]));
                        const float h0 = widen16<false>(hi & 0xFFFFu), h1 = widen16<false>(hi >> 16);
                        const uint32_t lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(x[2 * e2] - h0, x[2 * e2 + 1] - h1));
                        keep[e2] = hl ? lo : hi;
                        send[e2] = hl ? hi : lo;
                    }
                    const uint32_t r0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send[0], kDppXor1, 0xf, 0xf, true);
                    const uint32_t r1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send[1], kDppXor1, 0xf, 0xf, true);
                    bop[nt] = hl ? uint4v{r0, r1, keep[0], keep[1]} : uint4v{keep[0], keep[1], r0, r1};
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const uint32_t m0 = (aw.x & amask[t]) << ashift[t], m1 = (aw.y & amask[t]) << ashift[t];
                    const uint4v aop{bytes_to_halves<0>(m0), bytes_to_halves<1>(m0), bytes_to_halves<0>(m1), bytes_to_halves<1>(m1)};
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, aop), __builtin_bit_cast(half8, bop[nt]),
                                                                             acc[t][nt], 0, 0, 0);
                }
                aw = awn;
            }
            // C rows 4 kq + v of tile t are A rows (channels), C column = (r, hi | lo): add the lo
            // column to its hi neighbour, undo the two scalings, add the zero-point term, store
            const float unscale = __uint_as_float((127u + 24u + eb - 141u) << 23);   // 2^24 / bscale
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int r = 8 * nt + (ic >> 1);
                    float zsum = 0.0f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) zsum += red_z[(w * NR + r) * M + mw];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float val = acc[t][nt][v];
                        val += dpp_move<kDppXor1>(val);
                        const int row16 = 4 * kq + v;                    // A row inside the tile
                        const int j = JT * t + row16 / LW;               // code index inside its byte
                        const int c = (wave * LW + row16 % LW) * CPB + j;
                        val = val * (unscale * __uint_as_float((uint32_t)(127 - (8 - BITS)) << 23)) + zsum;
                        if ((ic & 1) == 0) po[r * kD + c] = val;
                    }
                }
        } else {
            // sum_i (p_i s_i) code[i][c] for this lane's CPB channels, all (at most four) query rows
            for (int r0 = 0; r0 < NR; r0 += RH) {
                float acc[CPB][RH];
    #pragma unroll
                for (int j = 0; j < CPB; ++j)
    #pragma unroll
                    for (int r = 0; r < RH; ++r) acc[j][r] = 0.0f;
                uint4 w4 = w4_first;
                if (r0 > 0 && tid < units) w4 = *reinterpret_cast<const uint4*>(vc_lane + (size_t)(tid / LPB) * code_block_bytes(BITS));
                for (int u = tid; u < units; u += kThreads) {
                    const int blk = u / LPB;
                    uint4 w4n = make_uint4(0, 0, 0, 0);   // next iteration's codes, in flight during this one's arithmetic
                    if (u + kThreads < units)
                        w4n = *reinterpret_cast<const uint4*>(vc_lane + (size_t)((u + kThreads) / LPB) * code_block_bytes(BITS));
                    const int hb = blk * 2 + within / (16 * BITS);   // 16-token half block inside the chunk
                    const float* psb = ps + (hb * M + mgrp) * kCell + r0;
    #pragma unroll
                    for (int dq = 0; dq < 4; ++dq) {
                        const uint32_t w = comp(w4, dq);
                        float pv[4][RH];
    #pragma unroll
                        for (int b = 0; b < 4; ++b)
    #pragma unroll
                            for (int r = 0; r < RH; ++r) pv[b][r] = psb[(dq * 4 + b) * NR + r];
    #pragma unroll
                        for (int j = 0; j < CPB; ++j) {
                            const uint32_t mk = w & (MASK << (BITS * j));
                            const float f0 = cvt_ubyte<0>(mk), f1 = cvt_ubyte<1>(mk), f2 = cvt_ubyte<2>(mk), f3 = cvt_ubyte<3>(mk);
    #pragma unroll
                            for (int r = 0; r < RH; ++r) {
                                acc[j][r] = __builtin_fmaf(f0, pv[0][r], acc[j][r]);
                                acc[j][r] = __builtin_fmaf(f1, pv[1][r], acc[j][r]);
                                acc[j][r] = __builtin_fmaf(f2, pv[2][r], acc[j][r]);
                                acc[j][r] = __builtin_fmaf(f3, pv[3][r], acc[j][r]);
                            }
                        }
                    }
                    w4 = w4n;
                }
                // codes arrived scaled by 2^(BITS*j); lanes with equal Lc hold the same channels
    #pragma unroll
                for (int j = 0; j < CPB; ++j)
    #pragma unroll
                    for (int r = 0; r < RH; ++r) {
                        float v = acc[j][r] * __uint_as_float((uint32_t)(127 - BITS * j) << 23);
    #pragma unroll
                        for (int mask = 32; mask >= 16 * BITS; mask >>= 1) v += __shfl_xor(v, mask, 64);
                        acc[j][r] = v;
                    }
                __syncthreads();   // o_lds shares the region with ps: everyone is done with ps
                if (lane < 16 * BITS) {
    #pragma unroll
                    for (int j = 0; j < CPB; ++j)
    #pragma unroll
                        for (int r = 0; r < RH; ++r) o_lds[((size_t)wave * NR + r0 + r) * kD + Lc * CPB + j] = acc[j][r];
                }
            }
            __syncthreads();
            for (int e = tid; e < NR * kD; e += kThreads) {
                const int r = e / kD, c = e % kD;
                float v = 0.0f;
    #pragma unroll
                for (int w = 0; w < kWaves; ++w) v += o_lds[((size_t)w * NR + r) * kD + c] + red_z[(w * NR + r) * M + c / GROUP];
                po[e] = v;
            }
        }
    } else {
        attend_extra_chunk<NR, NROWS, BF16>(L, A, row, chunk, smem, red, m_row, l_row, po);
    }
    if (tid < NR) {
        float mv = 0.f, lv = 0.f;
#pragma unroll
        for (int r = 0; r < NR; ++r)
            if (r == tid) { mv = m_row[r]; lv = l_row[r]; }
        pml[2 * tid] = mv;
        pml[2 * tid + 1] = lv;
    }
}

// Merge the chunk partials of one (KV head, query row): o = sum_c o_c e^(m_c - m) / sum_c l_c e^(m_c - m).
// 1024 threads = 16 slices of the chunk list x 64 channel pairs; the chunk weights are
// computed once into LDS so that the partial-output loads are independent of each other.
// (Folding this into the partial kernel behind a "last workgroup" counter needs a
// device-scope fence in every workgroup, which writes back and invalidates the L2 of
// its XCD; measured, that made the kernel eight times slower than this extra launch.)
constexpr int kCombineMaxChunks = 1280;
constexpr int kCombineThreads = 1024, kCombineSlices = kCombineThreads / 64;
__global__ __launch_bounds__(kCombineThreads) void attend_combine_kernel(const float* __restrict__ part_o,
                                                                         const float* __restrict__ part_ml,
                                                                         int max_chunks, int n_chunks, int NR,
                                                                         float* __restrict__ out) {
    __shared__ float wgt[kCombineMaxChunks];
    __shared__ float red[2 * kCombineSlices];
    __shared__ float2 osum[kCombineSlices][64];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int row = blockIdx.x / NR, r = blockIdx.x % NR;
    const float* ml = part_ml + ((size_t)row * max_chunks * NR + r) * 2;
    const size_t ml_stride = (size_t)NR * 2;
    // the first batch of partial outputs is requested before anything depends on the maxima
    const int cp = lane, slice = wave;
    const float2* po = reinterpret_cast<const float2*>(part_o + ((size_t)row * max_chunks * NR + r) * kD) + cp;
    const size_t po_stride = (size_t)NR * kD / 2;
    float2 v0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int ch = slice + kCombineSlices * u;
        v0[u] = ch < n_chunks ? po[ch * po_stride] : make_float2(0.f, 0.f);
    }
    // (max, sum) of this thread's chunks: one 8-byte load each, all requested at once
    constexpr int kMlPerThread = (kCombineMaxChunks + kCombineThreads - 1) / kCombineThreads;
    float2 mlv[kMlPerThread];
#pragma unroll
    for (int u = 0; u < kMlPerThread; ++u) {
        const int ch = tid + u * kCombineThreads;
        mlv[u] = ch < n_chunks ? *reinterpret_cast<const float2*>(ml + ch * ml_stride) : make_float2(-INFINITY, 0.0f);
    }
    float mloc = -INFINITY;
#pragma unroll
    for (int u = 0; u < kMlPerThread; ++u) mloc = fmaxf(mloc, mlv[u].x);
    mloc = wave_max(mloc);
    if (lane == 0) red[wave] = mloc;
    __syncthreads();
    float mmax = red[0];
#pragma unroll
    for (int w = 1; w < kCombineSlices; ++w) mmax = fmaxf(mmax, red[w]);
    float dloc = 0.0f;
#pragma unroll
    for (int u = 0; u < kMlPerThread; ++u) {
        const int ch = tid + u * kCombineThreads;
        if (ch < n_chunks) {
            const float w = mlv[u].x == -INFINITY ? 0.0f : __expf(mlv[u].x - mmax);
            wgt[ch] = w;
            dloc = __builtin_fmaf(mlv[u].y, w, dloc);
        }
    }
    dloc = wave_sum(dloc);
    if (lane == 0) red[kCombineSlices + wave] = dloc;
    __syncthreads();
    float den = 0.0f;
#pragma unroll
    for (int w = 0; w < kCombineSlices; ++w) den += red[kCombineSlices + w];
    float2 o = make_float2(0.f, 0.f);
    for (int c0 = slice; c0 < n_chunks; c0 += kCombineSlices * 8) {
        float2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int ch = c0 + kCombineSlices * u;
            if (c0 == slice) v[u] = v0[u];
            else v[u] = ch < n_chunks ? po[ch * po_stride] : make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int ch = c0 + kCombineSlices * u;
            const float w = ch < n_chunks ? wgt[ch] : 0.0f;
            if (w != 0.0f) {   // a chunk without candidates may hold anything
                o.x = __builtin_fmaf(v[u].x, w, o.x);
                o.y = __builtin_fmaf(v[u].y, w, o.y);
            }
        }
    }
    osum[slice][cp] = o;
    __syncthreads();
    if (tid < 64) {
        float2 res = make_float2(0.f, 0.f);
#pragma unroll
        for (int w = 0; w < kCombineSlices; ++w) {
            res.x += osum[w][tid].x;
            res.y += osum[w][tid].y;
        }
        res.x /= den;
        res.y /= den;
        reinterpret_cast<float2*>(out + ((size_t)row * NR + r) * kD)[tid] = res;
    }
}

template <int BITS, int GROUP, int G, int NROWS>
hipError_t launch3(const LayerView& L, const AttendArgs& A, int n_extra, float* out, int phases, hipStream_t stream) {
    constexpr int NR = G * NROWS;
    if (A.n_main + n_extra > kCombineMaxChunks) return hipErrorInvalidValue;
    if (phases & kAttendPartial) {
        const dim3 grid((A.n_main + n_extra) * L.rows), block(kThreads);
        if (L.bf16)
            SPC_LAUNCH((attend_partial_kernel<BITS, GROUP, G, NROWS, true>), grid, block, stream, L, A);
        else
            SPC_LAUNCH((attend_partial_kernel<BITS, GROUP, G, NROWS, false>), grid, block, stream, L, A);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (phases & kAttendCombine)
        SPC_LAUNCH(attend_combine_kernel, dim3(L.rows * NR), dim3(kCombineThreads), stream, A.part_o, A.part_ml,
                   A.max_chunks, A.n_main + n_extra, NR, out);
    return hipGetLastError();
}

template <int BITS, int GROUP>
hipError_t launch2(const LayerView& L, AttendArgs& A, int n_rows, int n_ex, float* out, int phases, hipStream_t stream) {
#define SPC_CASE(g_, n_)                                                        \
    if (L.G == g_ && n_rows == n_) {                                            \
        A.n_main = (A.Nq + main_chunk(g_ * n_) - 1) / main_chunk(g_ * n_);      \
        const int n_extra = (n_ex + kExtraChunk - 1) / kExtraChunk;             \
        A.n_chunks = A.n_main + n_extra;                                        \
        if (A.n_main + n_extra > A.max_chunks) return hipErrorInvalidValue;     \
        return launch3<BITS, GROUP, g_, n_>(L, A, n_extra, out, phases, stream); \
    }
    SPC_CASE(1, 1) SPC_CASE(1, 2) SPC_CASE(2, 1) SPC_CASE(2, 2) SPC_CASE(4, 1) SPC_CASE(4, 2) SPC_CASE(8, 1)
    SPC_CASE(8, 2)
#undef SPC_CASE
    return hipErrorInvalidValue;
}

}  // namespace

int attend_main_chunk_tokens(int NR) { return main_chunk(NR); }
int attend_chunks(int NR, int Nq, int n_16bit) {
    return (Nq + main_chunk(NR) - 1) / main_chunk(NR) + (n_16bit + kExtraChunk - 1) / kExtraChunk;
}
int attend_extra_chunk_tokens() { return kExtraChunk; }
int attend_max_chunks() { return kCombineMaxChunks; }

hipError_t launch_attend(const LayerView& L, const void* q, int n_rows, int N, int Nq, float sm_scale,
                         const float* logits, size_t logit_stride, const uint16_t* slot, const int32_t* slot_idx,
                         const void* k_spec, const void* v_spec, const AttendScratch& scratch, float* out,
                         int phases, hipStream_t stream) {
    AttendArgs A;
    A.q = (const uint16_t*)q;
    A.logits = logits;
    A.logits_out = nullptr;
    A.logit_stride = logit_stride;
    A.slot = slot;
    A.slot_idx = slot_idx;
    A.k_spec = (const uint16_t*)k_spec;
    A.v_spec = (const uint16_t*)v_spec;
    A.part_o = scratch.part_o;
    A.part_ml = scratch.part_ml;
    A.max_chunks = scratch.max_chunks;
    A.n_main = 0;
    A.n_chunks = 0;
    A.N = N;
    A.Nq = Nq;
    A.sm_scale = sm_scale;
    const int n_ex = (slot_idx ? L.topk : 0) + (N - Nq) + (k_spec ? 1 : 0);
    if (L.bits == 4) {
        // 4-bit codes: a plain partial pass of their own, the merge kernel of the other widths
        const int NR = L.G * n_rows;
        if (phases & kAttendPartial) {
            const AttendArgs4 a4{q, logits, logit_stride, slot, slot_idx, k_spec, v_spec, scratch.part_o, scratch.part_ml,
                                 scratch.max_chunks, N, Nq, sm_scale};
            hipError_t e = launch_attend4_partial(L, a4, n_rows, stream);
            if (e != hipSuccess) return e;
        }
        if (phases & kAttendCombine) {
            const int n_chunks = attend_chunks(NR, Nq, n_ex);
            if (n_chunks > kCombineMaxChunks || n_chunks > scratch.max_chunks) return hipErrorInvalidValue;
            SPC_LAUNCH(attend_combine_kernel, dim3(L.rows * NR), dim3(kCombineThreads), stream, scratch.part_o, scratch.part_ml,
                       scratch.max_chunks, n_chunks, NR, out);
        }
        return hipGetLastError();
    }
    // one query head per KV head, two rows, 2-bit values: the partial pass with the value side on the
    // integer matrix cores (same chunking, same partial-result format, same merge kernel)
    if ((phases & kAttendPartial) && attend_uses_int8_matrix_cores(L, n_rows) && !(kernel_choice() & kChoiceAttendValu)) {
        hipError_t e = launch_attend_i8_partial(L, q, N, Nq, sm_scale, logits, logit_stride, slot, slot_idx, k_spec, v_spec,
                                                scratch, nullptr, 0, nullptr, stream);
        if (e != hipSuccess) return e;
        phases &= ~kAttendPartial;
        if (!phases) return hipSuccess;
    }
    if (L.bits == 2 && L.group == 32) return launch2<2, 32>(L, A, n_rows, n_ex, out, phases, stream);
    if (L.bits == 2 && L.group == 64) return launch2<2, 64>(L, A, n_rows, n_ex, out, phases, stream);
    if (L.bits == 1 && L.group == 32) return launch2<1, 32>(L, A, n_rows, n_ex, out, phases, stream);
    if (L.bits == 1 && L.group == 64) return launch2<1, 64>(L, A, n_rows, n_ex, out, phases, stream);
    if (L.bits == 2 && L.group == 128) return launch2<2, 128>(L, A, n_rows, n_ex, out, phases, stream);
    if (L.bits == 1 && L.group == 128) return launch2<1, 128>(L, A, n_rows, n_ex, out, phases, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
