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

// One workgroup (128 threads, thread = channel) quantises one group of G tokens of
// one (batch, KV head): D key groups (one per channel, over the G tokens) and
// G * 128/G value groups (per token, over G channels).
template <int BITS, int G, bool BF16>
__global__ __launch_bounds__(128) void flush_kernel(LayerView L, const uint16_t* __restrict__ k_new,
                                                    const uint16_t* __restrict__ v_new, int n_new, int N0,
                                                    int Nq0) {
    constexpr int M = kD / G;  // value groups per token
    __shared__ float vt[G][kD + 1];
    __shared__ uint8_t kcode[G][kD];
    __shared__ uint8_t vcode[G][kD];

    const int c = threadIdx.x;
    const int row = blockIdx.y;
    const int t0 = Nq0 + blockIdx.x * G;

    float kx[G];
#pragma unroll
    for (int e = 0; e < G; ++e) {
        const int t = t0 + e;
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
        kx[e] = widen16<BF16>(src_k[c]);
        vt[e][c] = widen16<BF16>(src_v[c]);
    }

    // keys: this thread's channel over the G tokens
    float mn = kx[0], mx = kx[0];
#pragma unroll
    for (int e = 1; e < G; ++e) {
        mn = kx[e] < mn ? kx[e] : mn;
        mx = kx[e] > mx ? kx[e] : mx;
    }
    float s, z;
    derive_scale_zero<BITS>(mn, mx, s, z);
#pragma unroll
    for (int e = 0; e < G; ++e) kcode[e][c] = (uint8_t)quantize_one<BITS>(kx[e], s, z);
    L.km[(size_t)row * L.km_stride + (size_t)(t0 / G) * kD + k_meta_index(c)] = narrow16<BF16>(mn) | (narrow16<BF16>(mx) << 16);
    __syncthreads();

    // values: G tokens x M groups = 128 (token, group) pairs, one per thread
    {
        const int e = c % G, m = c / G;
        float vmn = vt[e][m * G], vmx = vmn;
        for (int i = 1; i < G; ++i) {
            const float x = vt[e][m * G + i];
            vmn = x < vmn ? x : vmn;
            vmx = x > vmx ? x : vmx;
        }
        float vs, vz;
        derive_scale_zero<BITS>(vmn, vmx, vs, vz);
        for (int i = 0; i < G; ++i) vcode[e][m * G + i] = (uint8_t)quantize_one<BITS>(vt[e][m * G + i], vs, vz);
        L.vm[(size_t)row * L.vm_stride + (size_t)(t0 + e) * M + m] =
            narrow16<BF16>(vmn) | (narrow16<BF16>(vmx) << 16);
    }
    __syncthreads();

    // pack: G tokens x 4*BITS dwords for K, the same count for V
    constexpr int kDwords = G * 4 * BITS;
    uint8_t* kc_row = L.kc + (size_t)row * L.kc_stride;
    uint8_t* vc_row = L.vc + (size_t)row * L.vc_stride;
    for (int id = c; id < kDwords; id += 128) {
        {
            const int e = id / (4 * BITS), W = id % (4 * BITS);
            uint32_t w = 0;
#pragma unroll
            for (int j = 0; j < 32 / BITS; ++j) {
                const int ch = W * (32 / BITS) + j;
                w |= (uint32_t)kcode[e][ch] << k_bit_of_channel<BITS>(ch);
            }
            *reinterpret_cast<uint32_t*>(kc_row + k_dword_offset<BITS>(t0 + e, W)) = w;
        }
        {
            // V block layout: [half][lane][4 dwords of 4 tokens]
            const int blk = id / (128 * BITS), rem = id % (128 * BITS);
            const int half = rem / (64 * BITS), lane = (rem / 4) % (16 * BITS), dq = rem % 4;
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int e = blk * 32 + half * 16 + dq * 4 + b;
                uint32_t byte = 0;
#pragma unroll
                for (int j = 0; j < 8 / BITS; ++j) {
                    const int ch = lane * (8 / BITS) + j;
                    byte |= (uint32_t)vcode[e][ch] << v_bit_of_channel<BITS>(ch);
                }
                w |= byte << (8 * b);
            }
            const int t_first = t0 + blk * 32 + half * 16 + dq * 4;
            *reinterpret_cast<uint32_t*>(vc_row + v_byte_offset<BITS>(t_first, lane)) = w;
        }
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
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), s, z);
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
            derive_scale_zero<BITS>(widen16<BF16>(m & 0xFFFFu), widen16<BF16>(m >> 16), s, z);
            v_sz[2 * gi] = s;
            v_sz[2 * gi + 1] = z;
        }
    }
}

template <int BITS, int G>
hipError_t flush_dispatch(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0, int Nq0,
                          int n_flush, hipStream_t stream) {
    const dim3 grid(n_flush, L.rows), block(128);
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
    if (L.bits == 2 && L.group == 32) return flush_dispatch<2, 32>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 2 && L.group == 64) return flush_dispatch<2, 64>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
    if (L.bits == 1 && L.group == 32) return flush_dispatch<1, 32>(L, k_new, v_new, n_new, N0, Nq0, n_flush, stream);
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
    if (L.bits == 2 && L.group == 32) return export_dispatch<2, 32>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 2 && L.group == 64) return export_dispatch<2, 64>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 1 && L.group == 32) return export_dispatch<1, 32>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    if (L.bits == 1 && L.group == 64) return export_dispatch<1, 64>(L, Nq, k_codes, k_mnmx, k_sz, v_codes, v_mnmx, v_sz, stream);
    return hipErrorInvalidValue;
}

}  // namespace specache
