// Quant and Offload of new KV pairs (Appendix A "Decoding"; quantiser of Eq. 2 / Eq. 3,
// Section 3.4; KIVI's axes and residual, Section 2.1 / 4.1), plus the export hook that
// unpacks the device layout into the canonical one-code-per-byte view.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

template <bool BF16>
__device__ __forceinline__ uint32_t narrow16(float f) {
    // exact: f is one of the 16-bit inputs
    if constexpr (BF16) {
        return __float_as_uint(f) >> 16;
    } else {
        _Float16 h = (_Float16)f;
        uint16_t u;
        __builtin_memcpy(&u, &h, 2);
        return u;
    }
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
// lane exchange patterns inside a row of 16 lanes: neighbours 1 and 2 apart, then the
// mirrored halves of 8 and of 16 lanes
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

constexpr int kFlushThreads = 256;

// Reciprocal of a group's scale for quantize_near(); NaN sends every value of the group
// down the exact path (zero, subnormal or non-finite scales).
__device__ __forceinline__ float safe_rcp(float s) {
    return (s >= 1e-30f && s <= 1e30f) ? __builtin_amdgcn_rcpf(s) : __builtin_nanf("");
}

// Candidate for the code of quantize_one(), which takes the rounding decision of Eq. 2 on the
// correctly rounded quotient.  (x - z) * rs + 0.5 is within 1.2e-6 of that rounded sum (1 ulp
// of the reciprocal, the roundings of both forms, quotient <= 2^BITS), so its integer part is
// the same code unless it lies within 1e-5 of a boundary between two codes: `unsafe` is set
// for those, and for groups without a usable reciprocal, and the caller then repeats its
// values with the IEEE division.  Clamping to [0.5, 2^BITS - 0.5] first keeps values beyond
// the outer codes (the group's own minimum in the 1-bit form) away from that test.
template <int BITS>
__device__ __forceinline__ uint32_t quantize_near(float x, float z, float rs, bool& unsafe) {
    float f = __builtin_fmaf(__fsub_rn(x, z), rs, 0.5f);
    f = __builtin_amdgcn_fmed3f(f, 0.5f, (float)(1 << BITS) - 0.5f);
    unsafe |= fabsf(__builtin_amdgcn_fractf(f) - 0.5f) > 0.5f - 1e-5f;
    return (uint32_t)(int)f;
}

// One workgroup (4 waves) quantises one group of G tokens of one (batch, KV head): 128 key
// groups (one per channel, over the G tokens) and G * 128/G value groups (per token, over
// G channels).  A lane owns 4 adjacent channels (one 8-byte load) of G/8 tokens: the two
// halves of a wave take the even and the odd token of a pair, wave w the pairs w, w+4, ...
// Keys reduce over tokens (registers, then the 8 partial results per channel through LDS),
// values over the G/4 lanes of a channel group (DPP).  Codes are assembled into the device
// layout's 16-byte pieces in LDS and leave as coalesced 16-byte stores.
template <int BITS, int G, bool BF16>
__global__ __launch_bounds__(kFlushThreads) void flush_kernel(LayerView L, const uint16_t* __restrict__ k_new,
                                                              const uint16_t* __restrict__ v_new, int n_new,
                                                              int N0, int Nq0) {
    constexpr int M = kD / G;        // value groups per token
    constexpr int NT = G / 8;        // tokens per thread
    constexpr int NW = 4 * BITS;     // K code dwords per token
    constexpr int KL = 32 / BITS / 4;  // lanes that share one K code dword
    constexpr int VL = G / 4;        // lanes of one value group
    constexpr int kExactUnroll = NT > 8 ? NT : 1;   // see the exact-division path of the keys
    __shared__ float kmn[8][kD];
    __shared__ float kmx[8][kD];
    __shared__ __align__(16) uint32_t kd[NW][G];
    __shared__ __align__(16) uint8_t vb[16 * BITS][G];

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int hf = lane / 32, j = lane % 32;
    const int row = blockIdx.y;
    const int t0 = Nq0 + blockIdx.x * G;

    uint2 kraw[NT], vraw[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const int t = t0 + (i * 4 + wave) * 2 + hf;
        const uint16_t* src_k;
        const uint16_t* src_v;
        if (t < N0) {
            const uint16_t* r = L.ring + ((size_t)row * L.R + (t % L.R)) * 256;
            src_k = r;
            src_v = r + kD;
        } else {
            const size_t o = ((size_t)row * n_new + (t - N0)) * kD;
            src_k = k_new + o;
            src_v = v_new + o;
        }
        kraw[i] = reinterpret_cast<const uint2*>(src_k)[j];
        vraw[i] = reinterpret_cast<const uint2*>(src_v)[j];
    }

    // ---- keys: channels 4j..4j+3 over this thread's tokens, then over the workgroup ----
    float kx[NT][4];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        kx[i][0] = widen16<BF16>(kraw[i].x & 0xFFFFu);
        kx[i][1] = widen16<BF16>(kraw[i].x >> 16);
        kx[i][2] = widen16<BF16>(kraw[i].y & 0xFFFFu);
        kx[i][3] = widen16<BF16>(kraw[i].y >> 16);
    }
    {
        float mn[4], mx[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            mn[b] = mx[b] = kx[0][b];
#pragma unroll
            for (int i = 1; i < NT; ++i) {
                mn[b] = fminf(mn[b], kx[i][b]);
                mx[b] = fmaxf(mx[b], kx[i][b]);
            }
        }
        *reinterpret_cast<float4*>(&kmn[wave * 2 + hf][4 * j]) = make_float4(mn[0], mn[1], mn[2], mn[3]);
        *reinterpret_cast<float4*>(&kmx[wave * 2 + hf][4 * j]) = make_float4(mx[0], mx[1], mx[2], mx[3]);
    }
    __syncthreads();
    float kmin[4], kmax[4];
    {
        float4 a = *reinterpret_cast<const float4*>(&kmn[0][4 * j]);
        float4 c = *reinterpret_cast<const float4*>(&kmx[0][4 * j]);
#pragma unroll
        for (int p = 1; p < 8; ++p) {
            const float4 a2 = *reinterpret_cast<const float4*>(&kmn[p][4 * j]);
            const float4 c2 = *reinterpret_cast<const float4*>(&kmx[p][4 * j]);
            a.x = fminf(a.x, a2.x); a.y = fminf(a.y, a2.y); a.z = fminf(a.z, a2.z); a.w = fminf(a.w, a2.w);
            c.x = fmaxf(c.x, c2.x); c.y = fmaxf(c.y, c2.y); c.z = fmaxf(c.z, c2.z); c.w = fmaxf(c.w, c2.w);
        }
        kmin[0] = a.x; kmin[1] = a.y; kmin[2] = a.z; kmin[3] = a.w;
        kmax[0] = c.x; kmax[1] = c.y; kmax[2] = c.z; kmax[3] = c.w;
    }
    if (tid < 32) {
        uint32_t* km = L.km + (size_t)row * L.km_stride + (size_t)(t0 / G) * kD;
#pragma unroll
        for (int b = 0; b < 4; ++b)  // k_meta_index(4j + b) == 32 b + j
            km[32 * b + j] = narrow16<BF16>(kmin[b]) | (narrow16<BF16>(kmax[b]) << 16);
    }
    {
        float ks[4], kz[4], krs[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            derive_scale_zero<BITS>(kmin[b], kmax[b], L.one_bit_plain, ks[b], kz[b]);
            krs[b] = safe_rcp(ks[b]);
        }
        uint32_t kw[NT];
        bool unsafe = !(krs[0] == krs[0] && krs[1] == krs[1] && krs[2] == krs[2] && krs[3] == krs[3]);
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            kw[i] = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) kw[i] |= quantize_near<BITS>(kx[i][b], kz[b], krs[b], unsafe) << (8 * b);
        }
        if (unsafe) {
            // rolled where the token array still fits the registers that can be indexed at run time;
            // beyond that a rolled loop would move the array to scratch memory for the fast path too
#pragma unroll kExactUnroll
            for (int i = 0; i < NT; ++i) {
                kw[i] = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) kw[i] |= quantize_one<BITS>(kx[i][b], ks[b], kz[b]) << (8 * b);
            }
        }
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            uint32_t w = kw[i];
            // channel 4j+b is code w' = 4 (j % KL) + b of dword j / KL: bit 8 b + BITS (j % KL)
            w <<= BITS * (j % KL);
            w |= dpp_u32<kDppXor1>(w);
            w |= dpp_u32<kDppXor2>(w);
            if constexpr (KL == 8) w |= dpp_u32<kDppHalfMirror>(w);
            if (j % KL == 0) kd[j / KL][(i * 4 + wave) * 2 + hf] = w;
        }
    }

    // ---- values: per token, groups of G channels = VL adjacent lanes ----
    uint32_t* vm = L.vm + (size_t)row * L.vm_stride + (size_t)t0 * M;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const int e = (i * 4 + wave) * 2 + hf;
        float x[4];
        x[0] = widen16<BF16>(vraw[i].x & 0xFFFFu);
        x[1] = widen16<BF16>(vraw[i].x >> 16);
        x[2] = widen16<BF16>(vraw[i].y & 0xFFFFu);
        x[3] = widen16<BF16>(vraw[i].y >> 16);
        float mn = fminf(fminf(x[0], x[1]), fminf(x[2], x[3]));
        float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
        mn = fminf(mn, dpp_f32<kDppXor1>(mn));
        mx = fmaxf(mx, dpp_f32<kDppXor1>(mx));
        mn = fminf(mn, dpp_f32<kDppXor2>(mn));
        mx = fmaxf(mx, dpp_f32<kDppXor2>(mx));
        mn = fminf(mn, dpp_f32<kDppHalfMirror>(mn));
        mx = fmaxf(mx, dpp_f32<kDppHalfMirror>(mx));
        if constexpr (VL >= 16) {
            mn = fminf(mn, dpp_f32<kDppMirror>(mn));
            mx = fmaxf(mx, dpp_f32<kDppMirror>(mx));
        }
        if constexpr (VL == 32) {   // the two rows of 16 lanes of this half of the wave
            mn = fminf(mn, __shfl_xor(mn, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
        }
        if (j % VL == 0) vm[e * M + j / VL] = narrow16<BF16>(mn) | (narrow16<BF16>(mx) << 16);
        float vs, vz;
        derive_scale_zero<BITS>(mn, mx, L.one_bit_plain, vs, vz);
        const float vrs = safe_rcp(vs);
        bool unsafe = !(vrs == vrs);
        uint32_t byte = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) byte |= quantize_near<BITS>(x[b], vz, vrs, unsafe) << (BITS * b);
        if (unsafe) {
            byte = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) byte |= quantize_one<BITS>(x[b], vs, vz) << (BITS * b);
        }
        if constexpr (BITS == 1) {
            // a byte holds 8 channels = two lanes
            byte <<= 4 * (j % 2);
            byte |= dpp_u32<kDppXor1>(byte);
            if (j % 2 == 0) vb[j / 2][e] = (uint8_t)byte;
        } else {
            vb[j][e] = (uint8_t)byte;
        }
    }
    __syncthreads();

    // ---- 16-byte pieces of the device layout ----
    constexpr int kPieces = G * BITS;  // per operand; <= 256
    auto k_piece = [&](int id) {
        // K: [32-token sub-block][dword W][half of the lane's 8 tokens][quad lane]
        const int kl = id % 4, h2 = (id / 4) % 2, W = (id / 8) % NW, sb = id / (8 * NW);
        const int e = sb * 32 + kl * 8 + h2 * 4;
        const uint4 v = *reinterpret_cast<const uint4*>(&kd[W][e]);
        *reinterpret_cast<uint4*>(L.kc + (size_t)row * L.kc_stride + k_dword_offset<BITS>(t0 + e, W)) = v;
    };
    auto v_piece = [&](int id) {
        // V: [32-token block][half of 16 tokens][byte lane]
        const int Lb = id % (16 * BITS), half = (id / (16 * BITS)) % 2, sb = id / (32 * BITS);
        const int e = sb * 32 + half * 16;
        const uint4 v = *reinterpret_cast<const uint4*>(&vb[Lb][e]);
        *reinterpret_cast<uint4*>(L.vc + (size_t)row * L.vc_stride + v_byte_offset<BITS>(t0 + e, Lb)) = v;
    };
    if constexpr (kPieces <= 128) {
        if (tid < kPieces) k_piece(tid);
        else if (tid >= 128 && tid < 128 + kPieces) v_piece(tid - 128);
    } else {
        static_assert(kPieces == kFlushThreads, "one K piece and one V piece per thread");
        k_piece(tid);
        v_piece(tid);
    }
}

// Offload: every new token goes to the pinned host copy C; tokens that stay
// unquantised after this call also go to the VRAM residual ring.
// 32 lanes x 16 B move one 512-byte (K,V) pair.
__global__ __launch_bounds__(256) void append_copy_kernel(LayerView L, const uint4* __restrict__ k_new,
                                                          const uint4* __restrict__ v_new, int n_new, int N0,
                                                          int ring_from) {
    const int row = blockIdx.y;
    const int tn = blockIdx.x * 8 + threadIdx.x / 32;
    if (tn >= n_new) return;
    const int part = threadIdx.x % 32;
    const size_t src = ((size_t)row * n_new + tn) * 16 + (part % 16);
    const uint4 v = part < 16 ? k_new[src] : v_new[src];
    const int t = N0 + tn;
    reinterpret_cast<uint4*>(L.host)[((size_t)row * L.max_seq + t) * 32 + part] = v;
    if (t >= ring_from) reinterpret_cast<uint4*>(L.ring)[((size_t)row * L.R + (t % L.R)) * 32 + part] = v;
}

// Canonical view: one thread per (token, channel).
template <int BITS, int G, bool BF16>
__global__ __launch_bounds__(128) void export_kernel(LayerView L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx,
                                                     float* k_sz, uint8_t* v_codes, uint16_t* v_mnmx,
                                                     float* v_sz) {
    constexpr int M = kD / G;
    const int c = threadIdx.x, t = blockIdx.x, row = blockIdx.y;
    const uint8_t* kc_row = L.kc + (size_t)row * L.kc_stride;
    const uint8_t* vc_row = L.vc + (size_t)row * L.vc_stride;
    const size_t o = ((size_t)row * Nq + t) * kD + c;
    if (k_codes) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(kc_row + k_dword_offset<BITS>(t, k_dword_of_channel<BITS>(c)));
        k_codes[o] = (uint8_t)((w >> k_bit_of_channel<BITS>(c)) & ((1u << BITS) - 1));
    }
    if (v_codes) {
        const uint8_t b = vc_row[v_byte_offset<BITS>(t, v_lane_of_channel<BITS>(c))];
        v_codes[o] = (uint8_t)((b >> v_bit_of_channel<BITS>(c)) & ((1u << BITS) - 1));
    }
    if (t % G == 0) {
        const size_t gi = ((size_t)row * (Nq / G) + t / G) * kD + c;
        const uint32_t m = L.km[(size_t)row * L.km_stride + (size_t)(t / G) * kD + k_meta_index(c)];
        if (k_mnmx) { k_mnmx[2 * gi] = (uint16_t)(m & 0xFFFFu); k_mnmx[2 * gi + 1] = (uint16_t)(m >> 16); }
        if (k_sz) {
            float s, z;
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), L.one_bit_plain, s, z);
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
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), L.one_bit_plain, s, z);
            v_sz[2 * gi] = s;
            v_sz[2 * gi + 1] = z;
        }
    }
}

template <int BITS, int G>
hipError_t flush_dispatch(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0, int Nq0,
                          int n_flush, hipStream_t stream) {
    const dim3 grid(n_flush, L.rows), block(kFlushThreads);
    if (L.bf16)
        hipLaunchKernelGGL((flush_kernel<BITS, G, true>), grid, block, 0, stream, L, (const uint16_t*)k_new,
                           (const uint16_t*)v_new, n_new, N0, Nq0);
    else
        hipLaunchKernelGGL((flush_kernel<BITS, G, false>), grid, block, 0, stream, L, (const uint16_t*)k_new,
                           (const uint16_t*)v_new, n_new, N0, Nq0);
    return hipGetLastError();
}

template <int BITS, int G>
hipError_t export_dispatch(const LayerView& L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx, float* k_sz,
                           uint8_t* v_codes, uint16_t* v_mnmx, float* v_sz, hipStream_t stream) {
    const dim3 grid(Nq, L.rows), block(128);
    if (L.bf16)
        hipLaunchKernelGGL((export_kernel<BITS, G, true>), grid, block, 0, stream, L, Nq, k_codes, k_mnmx, k_sz,
                           v_codes, v_mnmx, v_sz);
    else
        hipLaunchKernelGGL((export_kernel<BITS, G, false>), grid, block, 0, stream, L, Nq, k_codes, k_mnmx, k_sz,
                           v_codes, v_mnmx, v_sz);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_flush(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0, int Nq0,
                        int n_flush, hipStream_t stream) {
    if (n_flush <= 0) return hipSuccess;
    if (L.bits == 4) return launch_flush4(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 2 && L.group == 32) return flush_dispatch<2, 32>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 2 && L.group == 64) return flush_dispatch<2, 64>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 1 && L.group == 32) return flush_dispatch<1, 32>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 2 && L.group == 128) return flush_dispatch<2, 128>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 1 && L.group == 128) return flush_dispatch<1, 128>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 1 && L.group == 64) return flush_dispatch<1, 64>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    return hipErrorInvalidValue;
}

hipError_t launch_append_copy(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0,
                              int ring_from, hipStream_t stream) {
    if (n_new <= 0) return hipSuccess;
    const dim3 grid((n_new + 7) / 8, L.rows), block(256);
    hipLaunchKernelGGL(append_copy_kernel, grid, block, 0, stream, L, (const uint4*)k_new, (const uint4*)v_new,
                       n_new, N0, ring_from);
    return hipGetLastError();
}

hipError_t launch_export(const LayerView& L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx, float* k_sz,
                         uint8_t* v_codes, uint16_t* v_mnmx, float* v_sz, hipStream_t stream) {
    if (Nq <= 0) return hipSuccess;
    if (L.bits == 4) return launch_export4(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 2 && L.group == 32) return export_dispatch<2, 32>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 2 && L.group == 64) return export_dispatch<2, 64>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 1 && L.group == 32) return export_dispatch<1, 32>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 2 && L.group == 128) return export_dispatch<2, 128>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 1 && L.group == 128) return export_dispatch<1, 128>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 1 && L.group == 64) return export_dispatch<1, 64>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
