// Pre-fetch(C_K): sparse gather of the selected 16-bit (K,V) pairs from the pinned
// host copy C into a VRAM staging slot (Section 3.3: prefetching runs in parallel
// with later computation; Section 3.2 on sparse CPU->GPU transfers).
//
// The kernel reads host memory directly over the host link: one 512-byte pair is
// a single contiguous read by 32 lanes x 16 B, so each index costs one fat
// request instead of many small copies.  It is launched on the caller's side
// stream.
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

constexpr int kPairsPerBlock = 8;  // 256 threads

__global__ __launch_bounds__(256) void gather_kernel(const uint4* __restrict__ host, int max_seq, int k,
                                                     const int32_t* __restrict__ idx, uint4* __restrict__ slot,
                                                     int32_t* __restrict__ slot_idx) {
    const int row = blockIdx.y;
    const int j = blockIdx.x * kPairsPerBlock + threadIdx.x / 32;
    if (j >= k) return;
    const int part = threadIdx.x % 32;
    int i = idx[(size_t)row * k + j];
    if (i >= max_seq) i = -1;  // never read outside the store
    if (part == 0) slot_idx[(size_t)row * k + j] = i;
    if (i < 0) return;
    slot[((size_t)row * k + j) * 32 + part] = host[((size_t)row * max_seq + i) * 32 + part];
}

}  // namespace

hipError_t launch_gather(const LayerView& L, const int32_t* idx, uint16_t* slot, int32_t* slot_idx,
                         hipStream_t stream) {
    const dim3 grid((L.topk + kPairsPerBlock - 1) / kPairsPerBlock, L.rows), block(256);
    hipLaunchKernelGGL(gather_kernel, grid, block, 0, stream, (const uint4*)L.host, L.max_seq, L.topk, idx,
                       (uint4*)slot, slot_idx);
    return hipGetLastError();
}

}  // namespace specache
