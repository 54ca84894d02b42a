// ArgTopK of the speculative row (Appendix A "Decoding": K_{t+1} = ArgTopK(A_{1,:});
// "Pre-decoding" for the single-row case).  Softmax is monotone, so the selection
// runs on the logits' order-preserving integer keys.
//
// One workgroup of 1024 threads per (batch, KV head); rows of up to 65536 keys sit in
// registers, longer rows are re-read from L2 in batches of independent loads.  The
// number of barrier-separated phases, not arithmetic, bounds this kernel, so the exact
// k-th largest key tau is found in three short steps:
//   1. floor: every thread's largest key is a distinct element of the row, so tau is at
//      least the k-th largest thread maximum; one 2048-bin histogram of the maxima's
//      leading bits gives a floor F below which nothing can be selected;
//   2. one 2048-bin histogram of (key - F) >> shift over the keys >= F, with the shift
//      chosen from the row maximum so that the bins are as fine as 2048 bins allow,
//      locates the bin that holds tau and the rank of tau inside it;
//   3. the handful of keys in that bin are collected and ranked by one wave.
// If that bin holds more than 64 keys (many equal or almost equal scores) step 2 is
// repeated inside the bin, which narrows the range by 11 bits each time.
// A two-pass ordered compaction then emits every position with key > tau and the first
// `need` positions with key == tau in ascending index order (ties to the lower index).
#include "kernels.h"
#include "layout.h"

namespace specache {
namespace {

constexpr int kBins = 2048;
constexpr int kBatch = 8;    // key loads in flight per thread (streaming variant)
constexpr int kSmall = 64;   // keys one wave ranks directly

// exclusive prefix of a 64-bit ballot below this lane
__device__ __forceinline__ int prefix_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// hist[] is stored skewed (bin b at b + b / 32) so that a lane walking 32 consecutive bins
// and its neighbours touch different banks.
__device__ __forceinline__ int skew(int b) { return b + (b >> 5); }
constexpr int kHistWords = kBins + kBins / 32;

// Wave 0 only: find the bin holding the need-th largest counted key (bins ordered by
// value, larger bin = larger keys).  Writes sel[0] = bin (or 0xFFFFFFFF if fewer than
// `need` keys were counted) and sel[1] = rank of the wanted key inside that bin (1-based,
// counted from the bin's largest key).
__device__ __forceinline__ void select_bin_wave0(const uint32_t* hist, uint32_t* sel, uint32_t need) {
    const int lane = threadIdx.x & 63;
    // lane l owns bins 32l .. 32l+31, held in registers
    uint32_t h[32];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        h[j] = hist[skew(32 * lane + j)];
        mine += h[j];
    }
    // keys in bins owned by higher lanes
    uint32_t above = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_down(above, d, 64);
        if (lane + d < 64) above += o;
    }
    above -= mine;
    if (lane == 0) sel[0] = 0xFFFFFFFFu;
    // walk this lane's bins from the top; exactly one (lane, bin) pair brackets `need`
    uint32_t gt = above, found_bin = 0xFFFFFFFFu, found_rank = 0;
#pragma unroll
    for (int j = 31; j >= 0; --j) {
        const bool hit = gt < need && need <= gt + h[j];
        found_bin = hit ? (uint32_t)(32 * lane + j) : found_bin;
        found_rank = hit ? need - gt : found_rank;
        gt += h[j];
    }
    if (found_bin != 0xFFFFFFFFu) { sel[0] = found_bin; sel[1] = found_rank; }
}

// A row may be split into `parts` ranges of part_len keys, one workgroup each, that write
// their selections (position in the row, and the key if key_out is set) side by side; a
// second launch then selects among those candidates and translates its positions through
// `map`.  parts == 1, map == key_out == null is the plain single-launch selection.
struct TopkIo {
    int nq_total, parts, part_len;
    const int32_t* map;      // [rows][map_stride] or null
    size_t map_stride;
    uint32_t* key_out;       // [rows * parts][k] or null
};

// THREADS: 1024 for long rows; 256 for rows of up to 8192 keys, so that several rows share a
// compute unit and hide each other's barrier latency.
template <int THREADS, int KPT>
__global__ __launch_bounds__(THREADS) void topk_kernel(TopkIo io, int k, const uint32_t* __restrict__ keys,
                                                       size_t key_stride, int32_t* __restrict__ idx_out) {
    constexpr int kTopkThreads = THREADS;
    constexpr int kTopkWaves = THREADS / 64;
    __shared__ uint32_t hist[kHistWords];
    __shared__ uint32_t wave_red[kTopkWaves];
    __shared__ uint32_t sel[2];
    __shared__ uint32_t small_keys[kSmall];
    __shared__ uint32_t small_n;
    __shared__ uint32_t result[2];     // tau, number of keys == tau to take
    __shared__ uint32_t wave_gt[kTopkWaves], wave_eq[kTopkWaves];

    const int row = blockIdx.x / io.parts, part = blockIdx.x % io.parts;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int base = part * io.part_len;
    const int left = io.nq_total - base;
    const int Nq = left < 0 ? 0 : (left < io.part_len ? left : io.part_len);   // keys of this range
    const uint32_t* kr = keys + (size_t)row * key_stride + base;
    int32_t* out = idx_out + (size_t)blockIdx.x * k;
    uint32_t* kout = io.key_out ? io.key_out + (size_t)blockIdx.x * k : nullptr;
    const int32_t* map = io.map ? io.map + (size_t)row * io.map_stride : nullptr;
    const int keff = k < Nq ? k : Nq;
    // output slot `pos` receives local position i, whose key is kv
    auto emit = [&](uint32_t pos, int i, uint32_t kv) {
        out[pos] = map ? map[i] : base + i;
        if (kout) kout[pos] = kv;
    };

    for (int j = keff + tid; j < k; j += kTopkThreads) {
        out[j] = -1;
        if (kout) kout[j] = 0u;     // below every key: never selected by the second launch
    }
    if (keff == 0) return;
    if (keff == Nq) {   // everything is selected
        for (int j = tid; j < Nq; j += kTopkThreads) emit(j, j, kr[j]);
        return;
    }

    // wave w owns the contiguous index range [w*seg, (w+1)*seg), seg a multiple of 64
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
    // apply f(index, key) to every key slot of this thread.  Slots with index >= hi are padding
    // and hold key 0; every range tested below starts at 1 or above, so padding never matches
    // and no pass needs an index test.  (Key 0 itself is the one NaN pattern 0xFFFFFFFF; it is
    // treated as below every other score.)
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

    // ---- step 1: row maximum and the floor from the thread maxima ---------------------
    uint32_t tmax = 0;
    for_each_key([&](int, uint32_t kv) { tmax = kv > tmax ? kv : tmax; });
    const bool any = lo + lane < hi;   // this thread holds at least one key
    {
        uint32_t wm = tmax;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) { const uint32_t o = __shfl_xor(wm, m, 64); wm = o > wm ? o : wm; }
        if (lane == 0) wave_red[wave] = wm;
    }
    for (int b = tid; b < kHistWords; b += kTopkThreads) hist[b] = 0;
    __syncthreads();
    uint32_t row_max = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) row_max = wave_red[w] > row_max ? wave_red[w] : row_max;
    if (any) atomicAdd(&hist[skew(tmax >> 21)], 1u);
    __syncthreads();
    if (wave == 0) select_bin_wave0(hist, sel, (uint32_t)keff);
    __syncthreads();
    // fewer than keff threads hold keys: no floor
    uint32_t range_lo = sel[0] == 0xFFFFFFFFu ? 1u : (sel[0] << 21);
    range_lo = range_lo < 1u ? 1u : range_lo;
    uint32_t range_hi = row_max;          // inclusive
    uint32_t need = (uint32_t)keff;       // rank of tau among the keys >= range_lo
    __syncthreads();

    // ---- step 2 (repeated while the bin is crowded): histogram inside [range_lo, range_hi] ----
    for (int round = 0; round < 4; ++round) {
        const uint32_t span = range_hi - range_lo;
        const int shift = span < (uint32_t)kBins ? 0 : 32 - __builtin_clz(span) - 11;
        for (int b = tid; b < kHistWords; b += kTopkThreads) hist[b] = 0;
        if (tid == 0) small_n = 0;
        __syncthreads();
        for_each_key([&](int, uint32_t kv) {
            const uint32_t off = kv - range_lo;
            const bool cand = off <= span;       // one unsigned test for range_lo <= kv <= range_hi
            if (__ballot(cand) == 0) return;     // wave-uniform: most key slots hold no candidate
            if (cand) atomicAdd(&hist[skew(off >> shift)], 1u);
        });
        __syncthreads();
        if (wave == 0) select_bin_wave0(hist, sel, need);
        __syncthreads();
        const uint32_t bin = sel[0], rank = sel[1];
        const uint32_t bin_lo = range_lo + (bin << shift);
        const uint32_t bin_hi = shift == 0 ? bin_lo : bin_lo + ((1u << shift) - 1u);
        const uint32_t in_bin = hist[skew(bin)];
        if (shift == 0) {                  // the bin is a single key value
            if (tid == 0) { result[0] = bin_lo; result[1] = rank; }
            __syncthreads();
            break;
        }
        if (in_bin <= (uint32_t)kSmall) {
            // ---- step 3: one wave ranks the bin's keys ----
            for_each_key([&](int, uint32_t kv) {
                const bool cand = kv - bin_lo <= bin_hi - bin_lo;
                if (__ballot(cand) == 0) return;
                if (cand) small_keys[atomicAdd(&small_n, 1u)] = kv;
            });
            __syncthreads();
            if (wave == 0) {
                const uint32_t n = small_n;
                const uint32_t mine = lane < (int)n ? small_keys[lane] : 0u;
                uint32_t greater = 0, equal = 0;
#pragma unroll
                for (int j = 0; j < kSmall; ++j) {
                    const uint32_t kj = __builtin_amdgcn_readlane(mine, j);   // lane j's key, wave-uniform
                    const bool live = (uint32_t)j < n;
                    greater += live && kj > mine;
                    equal += live && kj == mine;
                }
                // tau is the key with greater < rank <= greater + equal
                if (lane < (int)n && greater < rank && rank <= greater + equal) {
                    result[0] = mine;
                    result[1] = rank - greater;
                }
            }
            __syncthreads();
            break;
        }
        range_lo = bin_lo;
        range_hi = bin_hi;
        need = rank;
        __syncthreads();
    }
    const uint32_t tau = result[0];
    need = result[1];

    // ---- ordered compaction: count per wave, then emit in index order ---------------
    uint32_t cnt_gt = 0, cnt_eq = 0;
    for_each_key([&](int, uint32_t kv) {
        const unsigned long long mge = __ballot(kv >= tau);
        if (mge == 0) return;              // wave-uniform skip
        const unsigned long long me = __ballot(kv == tau);
        cnt_gt += __popcll(mge & ~me);
        cnt_eq += __popcll(me);
    });
    if (lane == 0) { wave_gt[wave] = cnt_gt; wave_eq[wave] = cnt_eq; }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
    for_each_key([&](int i, uint32_t kv) {
        if (__ballot(kv >= tau) == 0) return;   // wave-uniform skip
        const bool gt = kv > tau, eq = kv == tau;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        const uint32_t my_eq_rank = eq_before + prefix_below(me);
        if (gt || (eq && my_eq_rank < need)) {
            const uint32_t eq_taken_before = my_eq_rank < need ? my_eq_rank : need;
            emit(gt_before + prefix_below(mg) + eq_taken_before, i, kv);
        }
        gt_before += __popcll(mg);
        eq_before += __popcll(me);
    });
}

// one launch over `rows * io.parts` ranges of at most n keys each
hipError_t launch_ranges(int rows, int n, const TopkIo& io, int k, const uint32_t* keys, size_t key_stride,
                         int32_t* idx_out, hipStream_t stream) {
    const int per_lane_256 = (n + 255) / 256, per_lane = (n + 1023) / 1024;   // keys per lane held in registers
#define SPC_TOPK(T, K) SPC_LAUNCH((topk_kernel<T, K>), dim3(rows * io.parts), dim3(T), stream, io, k, keys, key_stride, idx_out)
    // the floor of step 1 needs more threads than k to bite: small workgroups only for small k
    const bool small_wg = k <= 256;
    if (small_wg && per_lane_256 <= 8) SPC_TOPK(256, 8);
    else if (small_wg && per_lane_256 <= 16) SPC_TOPK(256, 16);
    else if (small_wg && per_lane_256 <= 32) SPC_TOPK(256, 32);
    else if (per_lane <= 16) SPC_TOPK(1024, 16);
    else if (per_lane <= 24) SPC_TOPK(1024, 24);
    else if (per_lane <= 32) SPC_TOPK(1024, 32);
    else if (per_lane <= 40) SPC_TOPK(1024, 40);
    else if (per_lane <= 48) SPC_TOPK(1024, 48);
    else if (per_lane <= 64) SPC_TOPK(1024, 64);
    else SPC_TOPK(1024, 0);
#undef SPC_TOPK
    return hipGetLastError();
}

}  // namespace

// One workgroup's registers hold 65536 keys, but its time grows faster than the row (32 rows, k = 256, alone:
// 17 us for 32768 keys, 34 for 49152, 61 and more for 65536), so rows beyond kTopkSingleLaunchKeys are split
// into ranges of about kTopkPartKeys keys, as many as keep the candidate list of the second launch within
// one workgroup's registers: two launches of 12 to 15 us each.
constexpr int kTopkRegisterKeys = 65536, kTopkPartKeys = 16384, kTopkSingleLaunchKeys = 40960;

int topk_parts(int Nq, int k) {
    if (Nq <= kTopkSingleLaunchKeys || k <= 0) return 1;
    int parts = (Nq + kTopkPartKeys - 1) / kTopkPartKeys;
    const int most = kTopkRegisterKeys / k;
    parts = parts < most ? parts : most;
    return parts < 2 ? 1 : parts;
}

hipError_t launch_topk(int rows, int Nq, int k, const uint32_t* keys, size_t key_stride, int32_t* idx_out,
                       const TopkScratch& scratch, hipStream_t stream) {
    const int parts = topk_parts(Nq, k);
    if (parts > 1 && parts <= scratch.max_parts && scratch.cand_keys && scratch.cand_idx) {
        if (pending_launch_events().stop) pending_launch_events().launches = 2;   // a timing pair spans both launches
        const int part_len = (((Nq + parts - 1) / parts) + 63) / 64 * 64;
        TopkIo first{Nq, parts, part_len, nullptr, 0, scratch.cand_keys};
        hipError_t e = launch_ranges(rows, part_len, first, k, keys, key_stride, scratch.cand_idx, stream);
        if (e != hipSuccess) return e;
        TopkIo second{parts * k, 1, parts * k, scratch.cand_idx, (size_t)parts * k, nullptr};
        return launch_ranges(rows, parts * k, second, k, scratch.cand_keys, (size_t)parts * k, idx_out, stream);
    }
    TopkIo io{Nq, 1, Nq, nullptr, 0, nullptr};
    return launch_ranges(rows, Nq, io, k, keys, key_stride, idx_out, stream);
}

}  // namespace specache
