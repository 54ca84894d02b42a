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

// A workgroup moves 8 * kInFlight pairs per trip: 8 groups of 32 lanes, each group kInFlight
// pairs, and every lane issues its kInFlight host reads before the first store.  The grid is kept small and
// loops over the index list: the number of host reads in flight is what matters for the
// link, and a bounded number of them leaves the memory system's request queues to the
// attention kernels that run beside the gather.
template <int kInFlight>
__global__ __launch_bounds__(256) void gather_kernel(const uint4* __restrict__ host, int max_seq, int k, int total,
                                                     const int32_t* __restrict__ idx, uint4* __restrict__ slot,
                                                     int32_t* __restrict__ slot_idx) {
    constexpr int kPairsPerTrip = 8 * kInFlight;
    __builtin_amdgcn_s_setprio(3);   // a wave's issue priority inside its SIMD, not a stream priority
    const int part = threadIdx.x % 32, grp = threadIdx.x / 32;
    for (int base = blockIdx.x * kPairsPerTrip; base < total; base += gridDim.x * kPairsPerTrip) {
        int src[kInFlight];
        size_t row_base[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int e = base + grp + u * 8;           // flat (row, j) entry
            int i = e < total ? idx[e] : -1;
            if (i >= max_seq) i = -1;                    // never read outside the store
            src[u] = i;
            row_base[u] = (size_t)(e / k) * max_seq;
            if (part == 0 && e < total) slot_idx[e] = i;
        }
        uint4 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u)
            v[u] = src[u] >= 0 ? host[(row_base[u] + src[u]) * 32 + part] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u)
            if (src[u] >= 0) slot[(size_t)(base + grp + u * 8) * 32 + part] = v[u];
    }
}

}  // namespace

hipError_t launch_gather(const LayerView& L, int Nq, const int32_t* idx, uint16_t* slot, int32_t* slot_idx,
                         bool link_shared, hipStream_t stream) {
    const int total = L.rows * L.topk;
    // 16 workgroups x 4 reads per lane = 256 KB of host reads in flight, issued at raised wave
    // priority.  Measured on MI355X at 32 heads x 256 pairs per layer: beside the other kernels
    // of the step the link delivers 40-46 GB/s (alone: 49 GB/s with 8 reads per lane, the rate
    // for 512-byte rows), while every further read in flight slows the attention kernel that
    // runs beside the gather (29 us alone, 38 us with 3 per lane, 43 with 4, 49 with 8, 65 with
    // 32 workgroups), also when the gather's workgroups have their compute units to themselves.
    // The gather's few waves issue almost nothing but their host reads; at the default priority
    // they wait for issue slots behind the scoring waves that share their SIMDs, and the link
    // idles meanwhile: with s_setprio 3 the gather takes 90 us per layer instead of 104 us.
    // The number of reads per lane follows the work of the main stream per fetched pair (scored
    // keys x query heads per pair): the more of it, the more the gather has time to spare and the
    // more a read in flight costs the other kernels.  Whole step, us per layer: 128 keys per pair
    // (7B shape at 32 k): 92.4 with four reads, 94.6 with three; 256 (4 query heads per KV head,
    // 32 k keys, 512 pairs): 176 with four, 173.5 with three; 512 (131 k keys, 1024 pairs): 149
    // with two, 154 with three.
    constexpr int kMaxGrid = 16;
    const double keys_per_pair = (double)L.G * Nq / (L.topk > 0 ? L.topk : 1);
    int in_flight = keys_per_pair >= 384.0 ? 2 : keys_per_pair >= 192.0 ? 3 : 4;
    // The caller spreads its gathers over several streams, so two of them are in flight at a time and
    // each other's launch gaps are covered.  Each then gets one read per lane and up to 32 workgroups
    // (the same 128 KB in flight as 16 workgroups x 2 reads, spread over more compute units): the link
    // carries 53-55 GB/s over the step, more than one gather reaches alone, and the other kernels are
    // disturbed less.  Whole step at the 7B shape at 32 k, us per layer: one stream x 16 workgroups x 4
    // reads 93; two streams x 16 x 2: 82.4; x 20 x 2: 80.5; x 32 x 1: 78.3; x 40 x 1: 77.6 - 81.9;
    // x 48 x 1: 85.6.
    int max_grid = kMaxGrid;
    if (link_shared) {
        in_flight = 1;
        max_grid = 32;
    }
    int grid = (total + 8 * in_flight - 1) / (8 * in_flight);
    if (grid > max_grid) grid = max_grid;
    if (grid < 1) return hipSuccess;
    const auto kernel = in_flight == 1 ? gather_kernel<1> : in_flight == 2 ? gather_kernel<2> : in_flight == 3 ? gather_kernel<3> : gather_kernel<4>;
    SPC_LAUNCH(kernel, dim3(grid), dim3(256), stream, (const uint4*)L.host, L.max_seq, L.topk, total, idx, (uint4*)slot, slot_idx);
    return hipGetLastError();
}

}  // namespace specache
