// Roofline denominators measured on the machine the benchmark runs on (see include/specache.h):
// the rate a plain 128-bit streaming read reaches from HBM, and the rate of the host link for a
// large pinned-to-device copy and for a kernel that reads pinned host memory directly (what the
// gather of Section 3.3's prefetch does, only contiguously).  None of this is on the decode path.
#include "../../include/specache.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

namespace {

// Every workgroup walks a contiguous share of the buffer, eight independent 16-byte loads per thread and
// trip (of the shapes tried on MI355X this one reads fastest: 6.3 TB/s from HBM with 4096 workgroups, against
// 5.3 to 5.7 TB/s for a grid-strided walk); the sums only keep the loads alive (the store never happens
// for the data these calls pass in).
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n_vec, uint32_t* sink) {
    const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = per * blockIdx.x, hi = lo + per < n_vec ? lo + per : n_vec;
    uint32_t acc = 0;
    size_t i = lo + threadIdx.x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < hi; i += 256) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;
}

struct Cleanup {
    void* dev = nullptr;
    void* dev2 = nullptr;
    void* host = nullptr;
    hipEvent_t a = nullptr, b = nullptr;
    ~Cleanup() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
        if (dev) (void)hipFree(dev);
        if (dev2) (void)hipFree(dev2);
        if (host) (void)hipHostFree(host);
    }
};

int status_of(hipError_t e) {
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? SPECACHE_ENOMEM : SPECACHE_EHIP;
}

#define MEAS_HIP(call)                                  \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) return status_of(e_);     \
    } while (0)

double median_of(std::vector<double>& v) {
    std::sort(v.begin(), v.end());
    return v[v.size() / 2];
}

// median rate of `reps` timed launches of the read kernel over `n_vec` 16-byte words at `src`
int time_read_kernel(const uint4* src, size_t n_vec, int grid, int reps, uint32_t* sink, Cleanup& c, double* gbs) {
    std::vector<double> rates;
    for (int r = 0; r < reps + 1; ++r) {   // the first launch warms up and is dropped
        MEAS_HIP(hipEventRecord(c.a, nullptr));
        hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, nullptr, src, n_vec, sink);
        MEAS_HIP(hipGetLastError());
        MEAS_HIP(hipEventRecord(c.b, nullptr));
        MEAS_HIP(hipEventSynchronize(c.b));
        float ms = 0.f;
        MEAS_HIP(hipEventElapsedTime(&ms, c.a, c.b));
        if (r > 0 && ms > 0.f) rates.push_back((double)n_vec * 16.0 / ((double)ms * 1e-3) / 1e9);
    }
    if (rates.empty()) return SPECACHE_EHIP;
    *gbs = median_of(rates);
    return SPECACHE_OK;
}

}  // namespace

extern "C" {

int specache_measure_hbm_read(int64_t bytes, int32_t reps, double* gbs) {
    if (!gbs || bytes < (1 << 20) || reps < 1 || reps > 1000) return SPECACHE_EINVAL;
    Cleanup c;
    const size_t n_vec = (size_t)bytes / 16;
    MEAS_HIP(hipMalloc(&c.dev, n_vec * 16));
    MEAS_HIP(hipMalloc(&c.dev2, 256));
    MEAS_HIP(hipMemset(c.dev, 0x5A, n_vec * 16));
    MEAS_HIP(hipEventCreate(&c.a));
    MEAS_HIP(hipEventCreate(&c.b));
    // 16 workgroups per compute unit of a 256-unit chip: every unit has loads in flight throughout
    return time_read_kernel((const uint4*)c.dev, n_vec, 256 * 16, reps, (uint32_t*)c.dev2, c, gbs);
}

int specache_measure_link(int64_t bytes, int32_t reps, double* memcpy_gbs, double* kernel_gbs) {
    if ((!memcpy_gbs && !kernel_gbs) || bytes < (1 << 20) || reps < 1 || reps > 1000) return SPECACHE_EINVAL;
    Cleanup c;
    const size_t n = (size_t)bytes / 16 * 16;
    MEAS_HIP(hipHostMalloc(&c.host, n, hipHostMallocDefault));
    MEAS_HIP(hipMalloc(&c.dev, n));
    MEAS_HIP(hipMalloc(&c.dev2, 256));
    for (size_t i = 0; i < n / 8; ++i) ((uint64_t*)c.host)[i] = 0x5A5A5A5A5A5A5A5Aull;
    MEAS_HIP(hipEventCreate(&c.a));
    MEAS_HIP(hipEventCreate(&c.b));
    if (memcpy_gbs) {
        std::vector<double> rates;
        for (int r = 0; r < reps + 1; ++r) {
            MEAS_HIP(hipEventRecord(c.a, nullptr));
            MEAS_HIP(hipMemcpyAsync(c.dev, c.host, n, hipMemcpyHostToDevice, nullptr));
            MEAS_HIP(hipEventRecord(c.b, nullptr));
            MEAS_HIP(hipEventSynchronize(c.b));
            float ms = 0.f;
            MEAS_HIP(hipEventElapsedTime(&ms, c.a, c.b));
            if (r > 0 && ms > 0.f) rates.push_back((double)n / ((double)ms * 1e-3) / 1e9);
        }
        if (rates.empty()) return SPECACHE_EHIP;
        *memcpy_gbs = median_of(rates);
    }
    if (kernel_gbs) {
        void* dev_view = nullptr;
        MEAS_HIP(hipHostGetDevicePointer(&dev_view, c.host, 0));
        // few workgroups, many reads in flight each: the link, not the compute units, is the resource
        if (int rc = time_read_kernel((const uint4*)dev_view, n / 16, 64, reps, (uint32_t*)c.dev2, c, kernel_gbs)) return rc;
    }
    return SPECACHE_OK;
}

}  // extern "C"
