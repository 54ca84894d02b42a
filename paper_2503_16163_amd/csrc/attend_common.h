// Pieces of the mixed attention of Eq. 1 (Section 3.3) shared by the attention kernels: launch
// arguments, wave reductions, and the pass over a chunk of 16-bit candidates (the pairs staged by
// the prefetch, the residual, the speculative token's transient pair).
#pragma once
#include "kernels.h"
#include "layout.h"
#include "wave_ops.h"

namespace specache {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kExtraChunk = 128;


template <int B>
__device__ __forceinline__ float cvt_ubyte(uint32_t w) {
    float f;
    if constexpr (B == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(f) : "v"(w));
    if constexpr (B == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(f) : "v"(w));
    if constexpr (B == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(f) : "v"(w));
    if constexpr (B == 3) asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(f) : "v"(w));
    return f;
}

__device__ __forceinline__ uint32_t comp(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// Operands of v_mfma_f32_16x16x32_f16: lane l holds A[l % 16][8 (l / 16) .. + 7] and
// B[8 (l / 16) .. + 7][l % 16] as eight f16, and C[4 (l / 16) .. + 3][l % 16] as four floats.
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

// two bytes of w, each widened to 16 bits: a small integer n read as f16 is the subnormal n * 2^-24
template <int HI>
__device__ __forceinline__ uint32_t bytes_to_halves(uint32_t w) {
    return __builtin_amdgcn_perm(0u, w, HI ? 0x0c030c02u : 0x0c010c00u);
}

// Wave-wide reductions on the VALU: four DPP steps leave every lane with its 16-lane row's
// result, the four row results are then read as scalars.  (A butterfly of ds_bpermute
// shuffles costs an LDS round trip per step.)
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_move<kDppMirror>(v));
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

struct AttendArgs {
    const uint16_t* q;         // [rows*NR][128]
    const float* logits;       // [rows*NR][logit_stride]
    float* logits_out;         // only the kernel that scores and attends in one pass: where to leave the logits, or null
    size_t logit_stride;
    const uint16_t* slot;      // [rows][k][256] or null
    const int32_t* slot_idx;   // [rows][k] or null
    const uint16_t* k_spec;    // [rows][128] or null
    const uint16_t* v_spec;
    float* part_o;             // [rows][max_chunks][NR][128]
    float* part_ml;            // [rows][max_chunks][NR][2]
    int max_chunks, n_main, n_chunks, N, Nq;
    float sm_scale;
};

// Softmax numerators of one chunk held in lg[NR][CH]: on return lg holds
// p = exp(l - m); m_out/l_out hold the chunk max and sum of every row.
template <int NR, int CH>
__device__ __forceinline__ void chunk_softmax(float (*lg)[CH], int n, float* red, float* m_out, float* l_out) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float mloc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) mloc[r] = -INFINITY;
    for (int i = tid; i < n; i += kThreads)
#pragma unroll
        for (int r = 0; r < NR; ++r) mloc[r] = fmaxf(mloc[r], lg[r][i]);
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const float v = wave_max(mloc[r]);
        if (lane == 0) red[wave * NR + r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        float v = red[r];
        for (int w = 1; w < kWaves; ++w) v = fmaxf(v, red[w * NR + r]);
        m_out[r] = v;
    }
    __syncthreads();
    float sloc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) sloc[r] = 0.0f;
    for (int i = tid; i < n; i += kThreads)
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const float ms = m_out[r] == -INFINITY ? 0.0f : m_out[r];
            const float p = __expf(lg[r][i] - ms);
            lg[r][i] = p;
            sloc[r] += p;
        }
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const float v = wave_sum(sloc[r]);
        if (lane == 0) red[wave * NR + r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        float v = red[r];
        for (int w = 1; w < kWaves; ++w) v += red[w * NR + r];
        l_out[r] = v;
    }
    __syncthreads();
}

// LDS floats attend_extra_chunk needs: lg[NR][128], the query rows [NR][128], two pointer tables
// and a flag table of 128 entries; at the end the same area holds o_lds[4][NR][128].
__host__ __device__ constexpr int extra_chunk_floats(int NR) {
    return (NR * 2 * kExtraChunk + 4 * kExtraChunk + kExtraChunk / 4) > 4 * NR * kD ? (NR * 2 * kExtraChunk + 4 * kExtraChunk + kExtraChunk / 4)
                                                                                  : 4 * NR * kD;
}

// One chunk of up to 128 16-bit candidates of a (batch, KV head) row: logits from the 16-bit keys,
// softmax numerators, weighted sum of the 16-bit values.  Writes the chunk's un-normalised output
// to po[NR][128] and its (max, sum) per query row to m_row / l_row.  Workgroup of 256 threads;
// smem: extra_chunk_floats(NR) floats, 16-byte aligned; red: 4 * NR floats.
template <int NR, int NROWS, bool BF16>
__device__ __forceinline__ void attend_extra_chunk(const LayerView& L, const AttendArgs& A, int row, int chunk, float* smem,
                                                   float* red, float* m_row, float* l_row, float* po) {
    constexpr int CHX = kExtraChunk;
    float (*lg)[CHX] = reinterpret_cast<float (*)[CHX]>(smem);
    float* o_lds = smem;                     // [4][NR][128]
    float (*qf)[kD] = reinterpret_cast<float (*)[kD]>(smem + NR * CHX);
    const uint16_t** src_k = reinterpret_cast<const uint16_t**>(smem + NR * CHX + NR * kD);
    const uint16_t** src_v = src_k + kExtraChunk;
    bool* src_spec = reinterpret_cast<bool*>(smem + NR * CHX + NR * kD + 4 * kExtraChunk);
    const int tid = threadIdx.x;
    const int ks = A.slot_idx ? L.topk : 0;
    const int n_res = A.N - A.Nq;
    const int n_ex = ks + n_res + (A.k_spec ? 1 : 0);
    const int x0 = (chunk - A.n_main) * kExtraChunk;
    const int n = (n_ex - x0) < kExtraChunk ? (n_ex - x0) : kExtraChunk;
    // requested together with the query rows: the position of this thread's staged candidate
    const int t_staged = (tid < n && x0 + tid < ks) ? A.slot_idx[(size_t)row * L.topk + x0 + tid] : -1;
    for (int e = tid; e < NR * kD; e += kThreads)
        qf[e / kD][e % kD] = widen16<BF16>(A.q[((size_t)row * NR) * kD + e]) * A.sm_scale;
    __syncthreads();

    // where each candidate's (K,V) pair lives; null = not a candidate (unused staging entry)
    if (tid < n) {
        const int x = x0 + tid;
        const uint16_t* kp = nullptr;
        bool spec = false, fresh = false;
        if (x < ks) {
            const int t = t_staged;
            if (t >= 0 && t < A.Nq) kp = A.slot + ((size_t)row * L.topk + x) * 256;
        } else if (x < ks + n_res) {
            const int t = A.Nq + (x - ks);
            kp = L.ring + ((size_t)row * L.R + (t % L.R)) * 256;
            // a token that this very launch appends (its copy into the ring may not have landed yet) is read
            // from the caller's buffers
            fresh = L.tail_k != nullptr && t == L.tail_N0;
        } else {
            spec = true;
        }
        src_k[tid] = spec ? A.k_spec + (size_t)row * kD : fresh ? L.tail_k + (size_t)row * kD : kp;
        src_v[tid] = spec ? A.v_spec + (size_t)row * kD : fresh ? L.tail_v + (size_t)row * kD : (kp ? kp + kD : nullptr);
        src_spec[tid] = spec;
    }
    __syncthreads();

    // logits: 16 lanes per candidate, 8 channels per lane; all key loads of a thread issued first
    constexpr int kPass = kExtraChunk / (kThreads / 16);
    const int sub = tid % 16, grp = tid / 16;
    uint4 kb[kPass];
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
        const int xl = grp + p * (kThreads / 16);
        const uint16_t* kp = xl < n ? src_k[xl] : nullptr;
        kb[p] = kp ? *reinterpret_cast<const uint4*>(kp + sub * 8) : make_uint4(0, 0, 0, 0);
    }
    float qreg[NR][8];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int d = 0; d < 8; ++d) qreg[r][d] = qf[r][sub * 8 + d];
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
        const int xl = grp + p * (kThreads / 16);
        float part[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) part[r] = 0.0f;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t w = comp(kb[p], d);
            const float k0 = widen16<BF16>(w & 0xFFFFu), k1 = widen16<BF16>(w >> 16);
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                part[r] = __builtin_fmaf(qreg[r][2 * d], k0, part[r]);
                part[r] = __builtin_fmaf(qreg[r][2 * d + 1], k1, part[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            float v = part[r];
#pragma unroll
            for (int mask = 8; mask >= 1; mask >>= 1) v += __shfl_xor(v, mask, 64);
            if (sub == 0 && xl < n) {
                const bool sees = src_k[xl] != nullptr && (!src_spec[xl] || (r % NROWS == NROWS - 1));
                lg[r][xl] = sees ? v : -INFINITY;
            }
        }
    }
    // sum_x p_x V[x][c]: thread = (channel pair, quarter of the candidates), loads in batches of 8,
    // the first batch requested before the softmax (every candidate with a pair, whatever
    // its weight turns out to be)
    const int cp = tid % 64, quarter = tid / 64;
    constexpr int kPerQuarter = kExtraChunk / 4;
    uint32_t vw0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int xl = quarter * kPerQuarter + u;
        const uint16_t* vp = xl < n ? src_v[xl] : nullptr;
        vw0[u] = vp ? *reinterpret_cast<const uint32_t*>(vp + 2 * cp) : 0u;
    }
    __syncthreads();
    chunk_softmax<NR, CHX>(lg, n, red, m_row, l_row);

    float acc[NR][2];
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r][0] = acc[r][1] = 0.0f;
#pragma unroll
    for (int b0 = 0; b0 < kPerQuarter; b0 += 8) {
        uint32_t vw[8];
        bool use[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int xl = quarter * kPerQuarter + b0 + u;
            bool any = false;
            if (xl < n) {
#pragma unroll
                for (int r = 0; r < NR; ++r) any = any || lg[r][xl] != 0.0f;
            }
            use[u] = any;
            // weight 0 (also every unused staging entry): its memory is never read after the first batch
            if (b0 == 0) vw[u] = vw0[u];
            else vw[u] = any ? *reinterpret_cast<const uint32_t*>(src_v[xl] + 2 * cp) : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int xl = quarter * kPerQuarter + b0 + u;
            if (xl < n && use[u]) {
                const float v0 = widen16<BF16>(vw[u] & 0xFFFFu), v1 = widen16<BF16>(vw[u] >> 16);
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    const float p = lg[r][xl];
                    acc[r][0] = __builtin_fmaf(p, v0, acc[r][0]);
                    acc[r][1] = __builtin_fmaf(p, v1, acc[r][1]);
                }
            }
        }
    }
    __syncthreads();   // done reading lg before the region is reused
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        o_lds[((size_t)quarter * NR + r) * kD + 2 * cp] = acc[r][0];
        o_lds[((size_t)quarter * NR + r) * kD + 2 * cp + 1] = acc[r][1];
    }
    __syncthreads();
    for (int e = tid; e < NR * kD; e += kThreads) {
        const int r = e / kD, cc = e % kD;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) v += o_lds[((size_t)w * NR + r) * kD + cc];
        po[e] = v;
    }
}

}  // namespace
}  // namespace specache
