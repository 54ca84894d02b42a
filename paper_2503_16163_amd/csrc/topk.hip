// ArgTopK of the speculative row (Appendix A "Decoding": K_{t+1} = ArgTopK(A_{1,:});
// "Pre-decoding" for the single-row case).  Softmax is monotone, so the selection
// runs on the logits' order-preserving integer keys.
//
// One workgroup of 1024 threads per (batch, KV head).  Exact radix select on the
// 32-bit keys, most significant digit first (11 + 11 + 10 bits), gives the k-th
// largest key tau and how many keys equal to tau are still needed; a two-pass
// ordered compaction then emits every position with key > tau and the first
// `need` positions with key == tau, in ascending index order (ties go to the
// lower index).  Keys are re-read from memory each pass; a row is at most a few
// hundred KB and stays in L2.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kBins = 2048;

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// exclusive prefix of a 64-bit ballot below this lane
__device__ __forceinline__ int prefix_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(int Nq, int k, const uint32_t* __restrict__ keys,
                                                            size_t key_stride, int32_t* __restrict__ idx_out) {
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_sum[kTopkWaves];
    __shared__ uint32_t sel_digit, sel_need;
    __shared__ uint32_t wave_gt[kTopkWaves], wave_eq[kTopkWaves];

    const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const uint32_t* kr = keys + (size_t)row * key_stride;
    int32_t* out = idx_out + (size_t)row * k;
    const int keff = k < Nq ? k : Nq;

    for (int j = keff + tid; j < k; j += kTopkThreads) out[j] = -1;
    if (keff == 0) return;

    // ---- radix select: find tau and how many keys == tau to take ---------------
    uint32_t prefix = 0, prefix_mask = 0, need = (uint32_t)keff;
    constexpr int shifts[3] = {21, 10, 0};
    constexpr int widths[3] = {11, 11, 10};
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = shifts[pass];
        const uint32_t nb = 1u << widths[pass];
        for (int b = tid; b < kBins; b += kTopkThreads) hist[b] = 0;
        __syncthreads();
        for (int i = tid; i < Nq; i += kTopkThreads) {
            const uint32_t key = kr[i];
            if ((key & prefix_mask) == prefix) atomicAdd(&hist[(key >> shift) & (nb - 1)], 1u);
        }
        __syncthreads();
        // thread t owns bins 2t, 2t+1; "greater" count of a bin = total - inclusive prefix
        const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
        uint32_t incl = h0 + h1;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        uint32_t base = 0, total = 0;
        for (int w = 0; w < kTopkWaves; ++w) {
            const uint32_t s = wave_sum[w];
            if (w < wave) base += s;
            total += s;
        }
        incl += base;                                  // keys in bins <= 2t+1
        const uint32_t gt1 = total - incl;             // keys in bins > 2t+1
        const uint32_t gt0 = gt1 + h1;                 // keys in bins > 2t
        if (gt1 < need && need <= gt1 + h1) { sel_digit = 2 * tid + 1; sel_need = need - gt1; }
        if (gt0 < need && need <= gt0 + h0) { sel_digit = 2 * tid; sel_need = need - gt0; }
        __syncthreads();
        prefix |= sel_digit << shift;
        prefix_mask |= (nb - 1) << shift;
        need = sel_need;
        __syncthreads();
    }
    const uint32_t tau = prefix;

    // ---- ordered compaction -------------------------------------------------------
    // wave w owns the contiguous index range [w*seg, (w+1)*seg), seg a multiple of 64
    const int seg = ((Nq + kTopkWaves * 64 - 1) / (kTopkWaves * 64)) * 64;
    const int lo = wave * seg, hi = (lo + seg < Nq) ? lo + seg : Nq;
    uint32_t cnt_gt = 0, cnt_eq = 0;
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? kr[i] : 0u;
        const bool gt = i < hi && key > tau, eq = i < hi && key == tau;
        cnt_gt += __popcll(__ballot(gt));
        cnt_eq += __popcll(__ballot(eq));
    }
    if (lane == 0) { wave_gt[wave] = cnt_gt; wave_eq[wave] = cnt_eq; }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? kr[i] : 0u;
        const bool gt = i < hi && key > tau, eq = i < hi && key == tau;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        const uint32_t my_eq_rank = eq_before + prefix_below(me);
        const bool take = gt || (eq && my_eq_rank < need);
        if (take) {
            const uint32_t eq_taken_before = my_eq_rank < need ? my_eq_rank : need;
            out[gt_before + prefix_below(mg) + eq_taken_before] = i;
        }
        gt_before += __popcll(mg);
        eq_before += __popcll(me);
    }
}

}  // namespace

hipError_t launch_topk(int rows, int Nq, int k, const uint32_t* keys, size_t key_stride, int32_t* idx_out,
                       hipStream_t stream) {
    hipLaunchKernelGGL(topk_kernel, dim3(rows), dim3(kTopkThreads), 0, stream, Nq, k, keys, key_stride, idx_out);
    return hipGetLastError();
}

}  // namespace specache
