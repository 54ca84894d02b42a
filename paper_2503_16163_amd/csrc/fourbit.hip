// 4-bit codes (Eq. 2 with B = 4; the KIVI axes and the residual policy as for the other widths): quantise and
// pack, export, low-bit scoring and the low-bit part of the mixed attention of Eq. 1.
//
// These kernels are plain vector-ALU code on a plain layout: a token's 128 codes of K (or V) are 64
// consecutive bytes, channel c in the low (even c) or high (odd c) half of byte c / 2.  The metadata arrays are
// those of the other widths (K: per token group 128 words min | max << 16 at k_meta_index(c); V: per token
// 128 / g words).  The paper's runs use 2 and 1 bits; 4 bits are carried for completeness (the cache is then
// 0.31 of its 16-bit size at g = 32), and nothing here is tuned the way the 1- and 2-bit kernels are.
#include <type_traits>

#include "attend_common.h"

namespace specache {
namespace {

constexpr int kTokBytes = 64;   // packed codes of one token's K or V

// ---- quantise + pack ------------------------------------------------------------------------------------
// One workgroup per group of G tokens of a (batch, KV head).  Threads 0..63: keys, a channel pair each, over the
// G tokens (per-channel groups).  Threads 64..191: values, a (token, channel group) each, over its G channels.
template <int G, bool BF16>
__global__ __launch_bounds__(256) void flush4_kernel(LayerView L, const uint16_t* __restrict__ k_new,
                                                     const uint16_t* __restrict__ v_new, int n_new, int N0, int Nq0) {
    constexpr int M = kD / G;
    const int tid = threadIdx.x, row = blockIdx.y;
    const int t0 = Nq0 + blockIdx.x * G;
    auto src_of = [&](int t, bool value) {
        if (t < N0) return (const uint16_t*)(L.ring + ((size_t)row * L.R + (t % L.R)) * 256 + (value ? kD : 0));
        return (value ? v_new : k_new) + ((size_t)row * n_new + (t - N0)) * kD;
    };
    if (tid < 64) {
        const int c0 = 2 * tid;
        float mn[2] = {INFINITY, INFINITY}, mx[2] = {-INFINITY, -INFINITY};
        for (int i = 0; i < G; ++i) {
            const uint32_t w = *reinterpret_cast<const uint32_t*>(src_of(t0 + i, false) + c0);
            const float a = widen16<BF16>(w & 0xFFFFu), b = widen16<BF16>(w >> 16);
            mn[0] = fminf(mn[0], a); mx[0] = fmaxf(mx[0], a);
            mn[1] = fminf(mn[1], b); mx[1] = fmaxf(mx[1], b);
        }
        float s[2], z[2];
        uint32_t* km = L.km + (size_t)row * L.km_stride + (size_t)(t0 / G) * kD;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            derive_scale_zero<4>(mn[e], mx[e], false, s[e], z[e]);
            const uint32_t lo = BF16 ? __float_as_uint(mn[e]) >> 16 : (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)mn[e]);
            const uint32_t hi = BF16 ? __float_as_uint(mx[e]) >> 16 : (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)mx[e]);
            km[k_meta_index(c0 + e)] = lo | (hi << 16);
        }
        uint8_t* kc = L.kc + (size_t)row * L.kc_stride;
        for (int i = 0; i < G; ++i) {
            const uint32_t w = *reinterpret_cast<const uint32_t*>(src_of(t0 + i, false) + c0);
            const uint32_t q0 = quantize_one<4>(widen16<BF16>(w & 0xFFFFu), s[0], z[0]);
            const uint32_t q1 = quantize_one<4>(widen16<BF16>(w >> 16), s[1], z[1]);
            kc[(size_t)(t0 + i) * kTokBytes + tid] = (uint8_t)(q0 | (q1 << 4));
        }
    } else if (tid < 64 + G * M) {   // G * M = 128
        const int wi = tid - 64, e = wi / M, m = wi % M;
        const uint16_t* src = src_of(t0 + e, true) + m * G;
        float mn = INFINITY, mx = -INFINITY;
        for (int c = 0; c < G; c += 2) {
            const uint32_t w = *reinterpret_cast<const uint32_t*>(src + c);
            const float a = widen16<BF16>(w & 0xFFFFu), b = widen16<BF16>(w >> 16);
            mn = fminf(mn, fminf(a, b));
            mx = fmaxf(mx, fmaxf(a, b));
        }
        float s, z;
        derive_scale_zero<4>(mn, mx, false, s, z);
        const uint32_t lo = BF16 ? __float_as_uint(mn) >> 16 : (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)mn);
        const uint32_t hi = BF16 ? __float_as_uint(mx) >> 16 : (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)mx);
        L.vm[(size_t)row * L.vm_stride + (size_t)(t0 + e) * M + m] = lo | (hi << 16);
        uint8_t* vc = L.vc + (size_t)row * L.vc_stride + (size_t)(t0 + e) * kTokBytes + m * (G / 2);
        for (int c = 0; c < G; c += 2) {
            const uint32_t w = *reinterpret_cast<const uint32_t*>(src + c);
            const uint32_t q0 = quantize_one<4>(widen16<BF16>(w & 0xFFFFu), s, z);
            const uint32_t q1 = quantize_one<4>(widen16<BF16>(w >> 16), s, z);
            vc[c / 2] = (uint8_t)(q0 | (q1 << 4));
        }
    }
}

// Canonical view: one thread per (token, channel).
template <int G, bool BF16>
__global__ __launch_bounds__(128) void export4_kernel(LayerView L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx, float* k_sz,
                                                      uint8_t* v_codes, uint16_t* v_mnmx, float* v_sz) {
    constexpr int M = kD / G;
    const int c = threadIdx.x, t = blockIdx.x, row = blockIdx.y;
    const size_t o = ((size_t)row * Nq + t) * kD + c;
    if (k_codes) k_codes[o] = (L.kc[(size_t)row * L.kc_stride + (size_t)t * kTokBytes + c / 2] >> (4 * (c & 1))) & 15u;
    if (v_codes) v_codes[o] = (L.vc[(size_t)row * L.vc_stride + (size_t)t * kTokBytes + c / 2] >> (4 * (c & 1))) & 15u;
    if (t % G == 0) {
        const size_t gi = ((size_t)row * (Nq / G) + t / G) * kD + c;
        const uint32_t m = L.km[(size_t)row * L.km_stride + (size_t)(t / G) * kD + k_meta_index(c)];
        if (k_mnmx) { k_mnmx[2 * gi] = (uint16_t)(m & 0xFFFFu); k_mnmx[2 * gi + 1] = (uint16_t)(m >> 16); }
        if (k_sz) {
            float s, z;
            derive_scale_zero<4>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), false, s, z);
            k_sz[2 * gi] = s;
            k_sz[2 * gi + 1] = z;
        }
    }
    if (c < M) {
        const size_t gi = ((size_t)row * Nq + t) * M + c;
        const uint32_t m = L.vm[(size_t)row * L.vm_stride + (size_t)t * M + c];
        if (v_mnmx) { v_mnmx[2 * gi] = (uint16_t)(m & 0xFFFFu); v_mnmx[2 * gi + 1] = (uint16_t)(m >> 16); }
        if (v_sz) {
            float s, z;
            derive_scale_zero<4>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), false, s, z);
            v_sz[2 * gi] = s;
            v_sz[2 * gi + 1] = z;
        }
    }
}

// ---- low-bit scoring (Appendix A "Decoding": A = Q K^T on C') -----------------------------------------------
// One workgroup per token group of G tokens of a row: the folded multipliers sm q[r][c] s[c] and the constants
// sum_c sm q[r][c] z[c] are shared by the group's tokens and sit in LDS; 256 / G threads share a token, each
// with G / 2 channels, and add their partial sums up with lane exchanges.
template <int G, int NR, int NROWS, bool BF16>
__global__ __launch_bounds__(256) void score4_kernel(LayerView L, const uint16_t* __restrict__ q, float sm_scale,
                                                     float* __restrict__ logits, size_t logit_stride,
                                                     uint32_t* __restrict__ keys, size_t key_stride) {
    constexpr int TPT = 256 / G;          // threads per token: 8, 4, 2
    constexpr int CPT = kD / TPT;         // channels per thread: 16, 32, 64
    __shared__ float qs[NR][kD];
    __shared__ float qz_part[NR][4];
    __shared__ float qz[NR];
    const int tid = threadIdx.x, row = blockIdx.y, grp = blockIdx.x;
    const uint32_t* km = L.km + (size_t)row * L.km_stride + (size_t)grp * kD;
    // thread (r0 = tid / 128, c = tid % 128) folds rows r0, r0 + 2, ...
    {
        const int c = tid & 127;
        const uint32_t m = km[k_meta_index(c)];
        float s, z;
        derive_scale_zero<4>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), false, s, z);
        for (int r = tid >> 7; r < NR; r += 2) {
            const float qv = widen16<BF16>(q[((size_t)row * NR + r) * kD + c]) * sm_scale;
            qs[r][c] = qv * s;
            float zz = qv * z;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) zz += __shfl_xor(zz, o, 64);
            if ((tid & 63) == 0) qz_part[r][(tid >> 6) & 1] = zz;
        }
    }
    __syncthreads();
    if (tid < NR) qz[tid] = qz_part[tid][0] + qz_part[tid][1];
    __syncthreads();
    const int tok = tid / TPT, sub = tid % TPT;
    const size_t t = (size_t)grp * G + tok;
    const uint8_t* kc = L.kc + (size_t)row * L.kc_stride + t * kTokBytes + sub * (CPT / 2);
    float acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.0f;
#pragma unroll
    for (int b4 = 0; b4 < CPT / 8; ++b4) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(kc + 4 * b4);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float code = (float)((w >> (4 * e)) & 15u);
            const int c = sub * CPT + 8 * b4 + e;
#pragma unroll
            for (int r = 0; r < NR; ++r) acc[r] = __builtin_fmaf(code, qs[r][c], acc[r]);
        }
    }
    float best = -INFINITY;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        float v = acc[r];
#pragma unroll
        for (int o = TPT / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        v += qz[r];
        if (sub == 0) logits[((size_t)row * NR + r) * logit_stride + t] = v;
        if (r % NROWS == NROWS - 1) best = fmaxf(best, v);
    }
    if (sub == 0) keys[(size_t)row * key_stride + t] = float_to_key(best);
}

// ---- mixed attention, partial pass over a chunk (Eq. 1) --------------------------------------------------------
// Main chunks: CH quantised positions (the chunking of the other widths, so that the merge kernel and the
// scratch sizes are shared): softmax numerators from the kept logits with the staged positions masked out,
// (s, z) per (token, value group) in LDS, then thread (code byte = channel pair, quarter of the chunk's tokens)
// accumulates sum_i p[r][i] (code s + z).  Extra chunks: the 16-bit candidates, attend_extra_chunk.
template <int GQ, int NROWS, bool BF16>
__global__ __launch_bounds__(kThreads) void attend4_partial_kernel(LayerView L, AttendArgs A, int CH) {
    constexpr int NR = GQ * NROWS;
    constexpr int kMaxCh = NR <= 8 ? 512 : 256;
    constexpr int kMain = NR * kMaxCh + kMaxCh * 4 * 2;
    constexpr int kRegion = kMain > extra_chunk_floats(NR) ? kMain : extra_chunk_floats(NR);
    __shared__ __attribute__((aligned(16))) float smem[kRegion];
    __shared__ float red[kWaves * NR];
    __shared__ uint32_t maskbits[kMaxCh / 32];
    const int tid = threadIdx.x;
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
    if (chunk >= A.n_main) {
        attend_extra_chunk<NR, NROWS, BF16>(L, A, row, chunk, smem, red, m_row, l_row, po);
    } else {
        const int M = kD / L.group;
        float (*lg)[kMaxCh] = reinterpret_cast<float (*)[kMaxCh]>(smem);
        float2* sz = reinterpret_cast<float2*>(smem + NR * kMaxCh);     // [token][M]
        const int c0 = chunk * CH;
        const int n = (A.Nq - c0) < CH ? (A.Nq - c0) : CH;
        if (tid < kMaxCh / 32) maskbits[tid] = 0u;
        __syncthreads();
        if (A.slot_idx)
            for (int j = tid; j < L.topk; j += kThreads) {
                const int t = A.slot_idx[(size_t)row * L.topk + j] - c0;
                if (t >= 0 && t < n) atomicOr(&maskbits[t >> 5], 1u << (t & 31));
            }
        __syncthreads();
        for (int i = tid; i < n; i += kThreads) {
            const bool masked = (maskbits[i >> 5] >> (i & 31)) & 1u;
#pragma unroll
            for (int r = 0; r < NR; ++r)
                lg[r][i] = masked ? -INFINITY : A.logits[((size_t)row * NR + r) * A.logit_stride + c0 + i];
            for (int m = 0; m < M; ++m) {
                const uint32_t w = L.vm[(size_t)row * L.vm_stride + (size_t)(c0 + i) * M + m];
                float s, z;
                derive_scale_zero<4>(widen16<BF16>(w & 0xFFFFu), widen16<BF16>(w >> 16), false, s, z);
                sz[i * M + m] = make_float2(s, z);
            }
        }
        __syncthreads();
        chunk_softmax<NR, kMaxCh>(lg, n, red, m_row, l_row);
        // thread = (byte b of a token's 64: channels 2b and 2b + 1, quarter of the chunk's tokens); four tokens'
        // bytes are requested at a time
        const int bpos = tid & 63, quarter = tid >> 6, m = (2 * bpos) / L.group;
        const uint8_t* vc = L.vc + (size_t)row * L.vc_stride + (size_t)c0 * kTokBytes + bpos;
        float acc[2][NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[0][r] = acc[1][r] = 0.0f;
        const int per = n / 4, lo = quarter * per, hi = lo + per;   // n is a multiple of 32
        for (int i = lo; i < hi; i += 4) {
            uint32_t by[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) by[u] = vc[(size_t)(i + u) * kTokBytes];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float2 szv = sz[(i + u) * M + m];
                const float v0 = __builtin_fmaf((float)(by[u] & 15u), szv.x, szv.y);
                const float v1 = __builtin_fmaf((float)(by[u] >> 4), szv.x, szv.y);
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    const float p = lg[r][i + u];
                    acc[0][r] = __builtin_fmaf(p, v0, acc[0][r]);
                    acc[1][r] = __builtin_fmaf(p, v1, acc[1][r]);
                }
            }
        }
        // the four quarters' sums through LDS, one query row at a time (the region holds lg and sz until then)
        float* o_lds = smem;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            o_lds[quarter * kD + 2 * bpos] = acc[0][r];
            o_lds[quarter * kD + 2 * bpos + 1] = acc[1][r];
            __syncthreads();
            if (tid < kD) po[r * kD + tid] = (o_lds[tid] + o_lds[kD + tid]) + (o_lds[2 * kD + tid] + o_lds[3 * kD + tid]);
            __syncthreads();
        }
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

template <typename F>
hipError_t by_group(int group, F&& f) {
    if (group == 32) return f(std::integral_constant<int, 32>());
    if (group == 64) return f(std::integral_constant<int, 64>());
    if (group == 128) return f(std::integral_constant<int, 128>());
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_flush4(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0, int Nq0, int n_flush,
                         hipStream_t stream) {
    const dim3 grid(n_flush, L.rows), block(256);
    return by_group(L.group, [&](auto g) {
        constexpr int G = decltype(g)::value;
        if (L.bf16) hipLaunchKernelGGL((flush4_kernel<G, true>), grid, block, 0, stream, L, (const uint16_t*)k_new, (const uint16_t*)v_new, n_new, N0, Nq0);
        else hipLaunchKernelGGL((flush4_kernel<G, false>), grid, block, 0, stream, L, (const uint16_t*)k_new, (const uint16_t*)v_new, n_new, N0, Nq0);
        return hipGetLastError();
    });
}

hipError_t launch_export4(const LayerView& L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx, float* k_sz, uint8_t* v_codes,
                          uint16_t* v_mnmx, float* v_sz, hipStream_t stream) {
    const dim3 grid(Nq, L.rows), block(128);
    return by_group(L.group, [&](auto g) {
        constexpr int G = decltype(g)::value;
        if (L.bf16) hipLaunchKernelGGL((export4_kernel<G, true>), grid, block, 0, stream, L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz);
        else hipLaunchKernelGGL((export4_kernel<G, false>), grid, block, 0, stream, L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz);
        return hipGetLastError();
    });
}

hipError_t launch_score4(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits, size_t logit_stride,
                         uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (Nq % L.group) return hipErrorInvalidValue;
    const dim3 grid(Nq / L.group, L.rows), block(256);
    return by_group(L.group, [&](auto g) {
        constexpr int G = decltype(g)::value;
#define SPC_S4(g_, n_)                                                                                                       \
    if (L.G == g_ && n_rows == n_) {                                                                                         \
        if (L.bf16) SPC_LAUNCH((score4_kernel<G, g_ * n_, n_, true>), grid, block, stream, L, (const uint16_t*)q, sm_scale, logits, logit_stride, keys, key_stride); \
        else SPC_LAUNCH((score4_kernel<G, g_ * n_, n_, false>), grid, block, stream, L, (const uint16_t*)q, sm_scale, logits, logit_stride, keys, key_stride);      \
        return hipGetLastError();                                                                                            \
    }
        SPC_S4(1, 1) SPC_S4(1, 2) SPC_S4(2, 1) SPC_S4(2, 2) SPC_S4(4, 1) SPC_S4(4, 2) SPC_S4(8, 1) SPC_S4(8, 2)
#undef SPC_S4
        return hipErrorInvalidValue;
    });
}

hipError_t launch_attend4_partial(const LayerView& L, const AttendArgs4& a, int n_rows, hipStream_t stream) {
    AttendArgs A;
    A.q = (const uint16_t*)a.q;
    A.logits = a.logits;
    A.logits_out = nullptr;
    A.logit_stride = a.logit_stride;
    A.slot = a.slot;
    A.slot_idx = a.slot_idx;
    A.k_spec = (const uint16_t*)a.k_spec;
    A.v_spec = (const uint16_t*)a.v_spec;
    A.part_o = a.part_o;
    A.part_ml = a.part_ml;
    A.max_chunks = a.max_chunks;
    A.N = a.N;
    A.Nq = a.Nq;
    A.sm_scale = a.sm_scale;
    const int NR = L.G * n_rows, CH = attend_main_chunk_tokens(NR);
    const int n_ex = (a.slot_idx ? L.topk : 0) + (a.N - a.Nq) + (a.k_spec ? 1 : 0);
    A.n_main = (a.Nq + CH - 1) / CH;
    A.n_chunks = A.n_main + (n_ex + kExtraChunk - 1) / kExtraChunk;
    if (A.n_chunks > A.max_chunks || A.n_chunks < 1) return hipErrorInvalidValue;
    const dim3 grid(A.n_chunks * L.rows), block(kThreads);
#define SPC_A4(g_, n_)                                                                                      \
    if (L.G == g_ && n_rows == n_) {                                                                        \
        if (L.bf16) SPC_LAUNCH((attend4_partial_kernel<g_, n_, true>), grid, block, stream, L, A, CH);      \
        else SPC_LAUNCH((attend4_partial_kernel<g_, n_, false>), grid, block, stream, L, A, CH);            \
        return hipGetLastError();                                                                           \
    }
    SPC_A4(1, 1) SPC_A4(1, 2) SPC_A4(2, 1) SPC_A4(2, 2) SPC_A4(4, 1) SPC_A4(4, 2) SPC_A4(8, 1) SPC_A4(8, 2)
#undef SPC_A4
    return hipErrorInvalidValue;
}

}  // namespace specache
