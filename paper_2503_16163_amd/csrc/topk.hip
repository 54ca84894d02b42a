// ArgTopK of the speculative row (Appendix A "Decoding": K_{t+1} = ArgTopK(A_{1,:});
// "Pre-decoding" for the single-row case).  Softmax is monotone, so the selection
// runs on the logits' order-preserving integer keys.
//
// One workgroup of 1024 threads per (batch, KV head).  Exact radix select on the
// 32-bit keys above a cheap lower bound, most significant digit first (11 + 11 + 10
// bits), gives the k-th
// largest key tau and how many keys equal to tau are still needed; a two-pass
// ordered compaction then emits every position with key > tau and the first
// `need` positions with key == tau, in ascending index order (ties go to the
// lower index).  Rows of up to 65536 keys are held in registers across all
// passes; longer rows are re-read from L2 in batches of independent loads.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kBins = 2048;
constexpr int kBatch = 8;   // key loads in flight per thread

// exclusive prefix of a 64-bit ballot below this lane
__device__ __forceinline__ int prefix_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Digit selection shared by both kernels: given hist[] of the current digit among the
// keys that match the prefix so far, find the digit holding the need-th largest key.
__device__ __forceinline__ void select_digit(const uint32_t* hist, uint32_t* wave_sum, uint32_t* sel, uint32_t need) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
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
    if (gt1 < need && need <= gt1 + h1) { sel[0] = 2 * tid + 1; sel[1] = need - gt1; }
    if (gt0 < need && need <= gt0 + h0) { sel[0] = 2 * tid; sel[1] = need - gt0; }
    __syncthreads();
}

// KPT > 0: the row fits in registers (KPT keys per lane, wave w owning the contiguous
// index range [w*seg, (w+1)*seg)), read once.  KPT == 0: any length, keys re-read from
// L2 in batches of independent loads on every pass.
template <int KPT>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(int Nq, int k, const uint32_t* __restrict__ keys,
                                                            size_t key_stride, int32_t* __restrict__ idx_out) {
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_sum[kTopkWaves];
    __shared__ uint32_t sel[2];
    __shared__ uint32_t wave_gt[kTopkWaves], wave_eq[kTopkWaves];

    const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const uint32_t* kr = keys + (size_t)row * key_stride;
    int32_t* out = idx_out + (size_t)row * k;
    const int keff = k < Nq ? k : Nq;

    for (int j = keff + tid; j < k; j += kTopkThreads) out[j] = -1;
    if (keff == 0) return;

    const int seg = ((Nq + kTopkWaves * 64 - 1) / (kTopkWaves * 64)) * 64;
    const int lo = wave * seg, hi = (lo + seg < Nq) ? lo + seg : Nq;

    uint32_t key[KPT > 0 ? KPT : 1];
    if constexpr (KPT > 0) {
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            const int i = lo + it * 64 + lane;
            key[it] = i < hi ? kr[i] : 0u;
        }
    }
    // apply f(index, key) to every key slot of this thread (slots with index >= hi are padding)
    auto for_each_key = [&](auto&& f) {
        if constexpr (KPT > 0) {
#pragma unroll
            for (int it = 0; it < KPT; ++it) f(lo + it * 64 + lane, key[it]);
        } else {
            for (int i0 = lo; i0 < hi; i0 += 64 * kBatch) {
                uint32_t kb[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int i = i0 + u * 64 + lane;
                    kb[u] = i < hi ? kr[i] : 0u;
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) f(i0 + u * 64 + lane, kb[u]);
            }
        }
    };
    auto clear_hist = [&]() {
        for (int b = tid; b < kBins; b += kTopkThreads) hist[b] = 0;
        __syncthreads();
    };

    // ---- a lower bound that leaves few candidates ------------------------------------
    // Every thread's largest key is a distinct element of the row, so the keff-th largest
    // key overall is at least the keff-th largest of the thread maxima; their leading
    // 11-bit digit gives a floor below which no key can be selected.  LDS atomics then
    // only see the few keys above the floor instead of the whole row.
    uint32_t floor_key = 0;
    {
        uint32_t tmax = 0;
        bool any = false;
        for_each_key([&](int i, uint32_t kv) {
            if (i < hi) { tmax = kv > tmax ? kv : tmax; any = true; }
        });
        clear_hist();
        if (any) atomicAdd(&hist[tmax >> 21], 1u);
        if (tid == 0) sel[0] = 0xFFFFFFFFu;   // stays if fewer than keff threads hold keys
        __syncthreads();
        select_digit(hist, wave_sum, sel, (uint32_t)keff);
        if (sel[0] != 0xFFFFFFFFu) floor_key = sel[0] << 21;
        __syncthreads();
    }

    // ---- radix select among keys >= floor_key: tau and how many keys == tau to take --
    uint32_t prefix = 0, prefix_mask = 0, need = (uint32_t)keff;
    constexpr int shifts[3] = {21, 10, 0};
    constexpr int widths[3] = {11, 11, 10};
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = shifts[pass];
        const uint32_t nb = 1u << widths[pass];
        clear_hist();
        const uint32_t cand_lo = prefix > floor_key ? prefix : floor_key;   // no key below this can match
        for_each_key([&](int i, uint32_t kv) {
            const bool cand = i < hi && kv >= cand_lo;
            if (__ballot(cand) == 0) return;   // wave-uniform: most key slots hold no candidate
            if (cand && (kv & prefix_mask) == prefix) atomicAdd(&hist[(kv >> shift) & (nb - 1)], 1u);
        });
        __syncthreads();
        select_digit(hist, wave_sum, sel, need);
        prefix |= sel[0] << shift;
        prefix_mask |= (nb - 1) << shift;
        need = sel[1];
        __syncthreads();
    }
    const uint32_t tau = prefix;

    // ---- ordered compaction: count per wave, then emit in index order ---------------
    uint32_t cnt_gt = 0, cnt_eq = 0;
    for_each_key([&](int i, uint32_t kv) {
        const unsigned long long mge = __ballot(i < hi && kv >= tau);
        if (mge == 0) return;              // wave-uniform skip
        const unsigned long long me = __ballot(i < hi && kv == tau);
        cnt_gt += __popcll(mge & ~me);
        cnt_eq += __popcll(me);
    });
    if (lane == 0) { wave_gt[wave] = cnt_gt; wave_eq[wave] = cnt_eq; }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
    for_each_key([&](int i, uint32_t kv) {
        if (__ballot(i < hi && kv >= tau) == 0) return;   // wave-uniform skip
        const bool gt = i < hi && kv > tau, eq = i < hi && kv == tau;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        const uint32_t my_eq_rank = eq_before + prefix_below(me);
        if (gt || (eq && my_eq_rank < need)) {
            const uint32_t eq_taken_before = my_eq_rank < need ? my_eq_rank : need;
            out[gt_before + prefix_below(mg) + eq_taken_before] = i;
        }
        gt_before += __popcll(mg);
        eq_before += __popcll(me);
    });
}

}  // namespace

hipError_t launch_topk(int rows, int Nq, int k, const uint32_t* keys, size_t key_stride, int32_t* idx_out,
                       hipStream_t stream) {
    const int per_lane = (Nq + kTopkThreads - 1) / kTopkThreads;   // keys per lane if the row sits in registers
    if (per_lane <= 8)
        hipLaunchKernelGGL(topk_kernel<8>, dim3(rows), dim3(kTopkThreads), 0, stream, Nq, k, keys, key_stride, idx_out);
    else if (per_lane <= 32)
        hipLaunchKernelGGL(topk_kernel<32>, dim3(rows), dim3(kTopkThreads), 0, stream, Nq, k, keys, key_stride, idx_out);
    else if (per_lane <= 64)
        hipLaunchKernelGGL(topk_kernel<64>, dim3(rows), dim3(kTopkThreads), 0, stream, Nq, k, keys, key_stride, idx_out);
    else
        hipLaunchKernelGGL(topk_kernel<0>, dim3(rows), dim3(kTopkThreads), 0, stream, Nq, k, keys, key_stride, idx_out);
    return hipGetLastError();
}

}  // namespace specache
