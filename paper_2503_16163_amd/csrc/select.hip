// Selection score shared by the query heads of a KV head, second form: the maximum over the
// heads of the head's log-probability over the low-bit positions (Appendix A "Decoding" applies
// ArgTopK to the softmax output A; the paper does not say how several query heads share one
// index set).  score = max_h (logit_h[i] - log sum_{j < Nq} exp(logit_h[j])) on the speculative
// row.  Two small kernels after the scoring pass: the first reduces every (row, head)'s logits,
// which the scoring kernel left behind, to (max, sum of exponentials) per slice of 8192
// positions; the second merges the slices into the head's log-sum-exp and rewrites the
// selection keys from the shifted logits.  With one query head per KV head the shift does not
// change the order and the pass is skipped.  Measured on MI355X: 13 us per layer-step on top of
// the scoring kernel, at 32 (row, head) pairs x 131072 positions as at 128 x 32768.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

constexpr int kSliceKeys = 8192;      // positions per workgroup of the first kernel
constexpr int kSliceThreads = 256;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// logits: [rows * G * n_rows][logit_stride]; the speculative row of head h of KV row `row` is row
// (row * G + h) * n_rows + n_rows - 1.  Nq is a multiple of 32.  Workgroup (slice, row * G + h)
// leaves (max, sum of exp(logit - max)) of its slice in part[(row * G + h) * n_slices + slice].
__global__ __launch_bounds__(kSliceThreads) void lse_slices_kernel(const float* __restrict__ logits, size_t logit_stride,
                                                                   int n_rows, int Nq, float2* __restrict__ part) {
    __shared__ float red[kSliceThreads / 64];
    const float* l = logits + ((size_t)blockIdx.y * n_rows + n_rows - 1) * logit_stride;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int lo = blockIdx.x * kSliceKeys, hi = lo + kSliceKeys < Nq ? lo + kSliceKeys : Nq;
    float m = -INFINITY;
    for (int i = lo + threadIdx.x * 4; i < hi; i += kSliceThreads * 4) {
        const float4 v = *reinterpret_cast<const float4*>(l + i);
        m = fmaxf(fmaxf(m, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
    m = wave_max(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.0f;
    for (int i = lo + threadIdx.x * 4; i < hi; i += kSliceThreads * 4) {      // the slice is in cache now
        const float4 v = *reinterpret_cast<const float4*>(l + i);
        s += (expf(v.x - m) + expf(v.y - m)) + (expf(v.z - m) + expf(v.w - m));
    }
    s = wave_sum(s);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = make_float2(m, (red[0] + red[1]) + (red[2] + red[3]));
}

// keys[row][i] = order-preserving key of max_h (logit_h[i] - lse_h); every workgroup first merges the
// slices' (max, sum) pairs of its row's heads into lse_h (a wave per head, at most 8 heads)
__global__ __launch_bounds__(256) void logprob_keys_kernel(const float* __restrict__ logits, size_t logit_stride, int G,
                                                           int n_rows, int Nq, const float2* __restrict__ part,
                                                           int n_slices, uint32_t* __restrict__ keys, size_t key_stride) {
    __shared__ float lse[8];
    const int row = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int h = wave; h < G; h += 4) {
        const float2* p = part + (size_t)(row * G + h) * n_slices;
        float m = -INFINITY;
        for (int s = lane; s < n_slices; s += 64) m = fmaxf(m, p[s].x);
        m = wave_max(m);
        float t = 0.0f;
        for (int s = lane; s < n_slices; s += 64) t += p[s].y * expf(p[s].x - m);
        t = wave_sum(t);
        if (lane == 0) lse[h] = m + logf(t);
    }
    __syncthreads();
    const int i = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= Nq) return;
    float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    for (int h = 0; h < G; ++h) {
        const float4 v = *reinterpret_cast<const float4*>(logits + ((size_t)(row * G + h) * n_rows + n_rows - 1) * logit_stride + i);
        const float c = lse[h];
        best[0] = fmaxf(best[0], v.x - c);
        best[1] = fmaxf(best[1], v.y - c);
        best[2] = fmaxf(best[2], v.z - c);
        best[3] = fmaxf(best[3], v.w - c);
    }
    *reinterpret_cast<uint4*>(keys + (size_t)row * key_stride + i) =
        make_uint4(float_to_key(best[0]), float_to_key(best[1]), float_to_key(best[2]), float_to_key(best[3]));
}

// Selection on the mixed cache (Eq. 1; Appendix A "Decoding" computes one A on C' u C_K and takes
// ArgTopK of its second row): the scoring pass has left pure low-bit logits; for the positions whose
// 16-bit pairs are staged, logits and key are replaced by those of the 16-bit key.  One wave per
// staged pair: lane = two channels, a wave reduction per query row.
template <bool BF16>
__global__ __launch_bounds__(256) void patch_staged_kernel(const uint16_t* __restrict__ q, int NR, int n_rows, float sm_scale,
                                                           const uint16_t* __restrict__ slot, const int32_t* __restrict__ slot_idx,
                                                           int k, int Nq, float* __restrict__ logits, size_t logit_stride,
                                                           uint32_t* __restrict__ keys, size_t key_stride) {
    const int row = blockIdx.y, j = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (j >= k) return;
    const int pos = slot_idx[(size_t)row * k + j];
    if (pos < 0 || pos >= Nq) return;                               // padding of a short selection
    const uint32_t kk = reinterpret_cast<const uint32_t*>(slot + ((size_t)row * k + j) * 256)[lane];
    const float k0 = widen16<BF16>(kk & 0xFFFFu), k1 = widen16<BF16>(kk >> 16);
    float best = -INFINITY;
    for (int r = 0; r < NR; ++r) {
        const uint32_t qq = reinterpret_cast<const uint32_t*>(q + ((size_t)row * NR + r) * kD)[lane];
        float acc = __builtin_fmaf(widen16<BF16>(qq & 0xFFFFu), k0, widen16<BF16>(qq >> 16) * k1);
        acc = wave_sum(acc) * sm_scale;
        if (lane == 0) logits[((size_t)row * NR + r) * logit_stride + pos] = acc;
        if (r % n_rows == n_rows - 1) best = fmaxf(best, acc);
    }
    if (lane == 0) keys[(size_t)row * key_stride + pos] = float_to_key(best);
}

}  // namespace

hipError_t launch_patch_staged(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, const uint16_t* slot,
                               const int32_t* slot_idx, float* logits, size_t logit_stride, uint32_t* keys,
                               size_t key_stride, hipStream_t stream) {
    if (Nq <= 0 || L.topk <= 0) return hipSuccess;
    const dim3 grid((L.topk + 3) / 4, L.rows), block(256);
    if (L.bf16)
        hipLaunchKernelGGL(patch_staged_kernel<true>, grid, block, 0, stream, (const uint16_t*)q, L.G * n_rows, n_rows, sm_scale,
                           slot, slot_idx, L.topk, Nq, logits, logit_stride, keys, key_stride);
    else
        hipLaunchKernelGGL(patch_staged_kernel<false>, grid, block, 0, stream, (const uint16_t*)q, L.G * n_rows, n_rows, sm_scale,
                           slot, slot_idx, L.topk, Nq, logits, logit_stride, keys, key_stride);
    return hipGetLastError();
}

size_t select_logprob_scratch_floats(int rows, int G, int max_seq) {
    return (size_t)rows * G * ((max_seq + kSliceKeys - 1) / kSliceKeys) * 2;
}

hipError_t launch_select_logprob(const LayerView& L, int n_rows, int Nq, const float* logits, size_t logit_stride,
                                 float* scratch, uint32_t* keys, size_t key_stride, hipStream_t stream) {
    if (Nq <= 0) return hipSuccess;
    if (Nq % 4 != 0 || logit_stride % 4 != 0 || key_stride % 4 != 0 || L.G > 8) return hipErrorInvalidValue;
    const int n_slices = (Nq + kSliceKeys - 1) / kSliceKeys;
    hipLaunchKernelGGL(lse_slices_kernel, dim3(n_slices, L.rows * L.G), dim3(kSliceThreads), 0, stream, logits, logit_stride,
                       n_rows, Nq, (float2*)scratch);
    hipLaunchKernelGGL(logprob_keys_kernel, dim3((Nq + 1023) / 1024, L.rows), dim3(256), 0, stream, logits, logit_stride,
                       L.G, n_rows, Nq, (const float2*)scratch, n_slices, keys, key_stride);
    return hipGetLastError();
}

}  // namespace specache
