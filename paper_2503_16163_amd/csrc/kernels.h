// Internal launch interface between the C-ABI host code (specache.hip) and the
// kernel translation units.  Every launcher only enqueues on `stream` and
// returns the hipGetLastError() of its launches.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace specache {

// Geometry and device pointers of one layer, as the kernels see them.
struct LayerView {
    int rows;          // B * Hkv
    int G;             // query heads per KV head
    int bits, group, R, max_seq, topk;
    bool bf16;
    bool one_bit_plain;   // bits == 1: Eq. 2 with B = 1 instead of Eq. 3
    uint8_t* kc;       // K codes   [rows][kc_stride bytes]
    uint32_t* km;      // K meta    [rows][km_stride dwords]  ([group j][128])
    uint8_t* vc;       // V codes   [rows][vc_stride bytes]
    uint32_t* vm;      // V meta    [rows][vm_stride dwords]  ([token][128/g])
    uint16_t* ring;    // residual  [rows][R][256] 16-bit
    uint16_t* host;    // pinned C  [rows][max_seq][256] 16-bit (device-visible address)
    size_t kc_stride, km_stride, vc_stride, vm_stride;
    // Set for one scoring launch only (specache_append_score): the new token's (K, V) pair, which one
    // extra workgroup per row copies to the host store and the residual ring as token tail_N0.
    const uint16_t* tail_k = nullptr;   // [rows][128] 16-bit, null: nothing to append
    const uint16_t* tail_v = nullptr;
    int tail_N0 = 0;
};

// quantize_append: flush `n_flush` groups starting at token Nq0, whose sources are
// the ring (tokens < N0) or k_new/v_new (tokens >= N0, index t - N0 of n_new).
hipError_t launch_flush(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0,
                        int Nq0, int n_flush, hipStream_t stream);
// copy the n_new tokens to the host store (all) and to the ring (tokens >= ring_from)
hipError_t launch_append_copy(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0,
                              int ring_from, hipStream_t stream);

// Per-kernel timing of the scoring pass and of ArgTopK: a pair of events that the next kernel launched through
// SPC_LAUNCH on this thread carries on its own dispatch packet (start and stop of that kernel, as a
// profiler sees them) instead of event records around the launch, which would add the stream's
// marker packets and the launch gap to the figure.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
    int launches = 1;   // kernels the pair spans: the first carries start, the last stop
};
LaunchEvents& pending_launch_events();
#define SPC_LAUNCH(kernel, grid, block, stream, ...)                                                          \
    do {                                                                                                      \
        specache::LaunchEvents& le_ = specache::pending_launch_events();                                      \
        if (le_.stop) {                                                                                       \
            const bool last_ = le_.launches <= 1;                                                             \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, le_.start, last_ ? le_.stop : nullptr, 0,   \
                                  __VA_ARGS__);                                                               \
            if (last_) le_ = specache::LaunchEvents{};                                                        \
            else { le_.start = nullptr; --le_.launches; }                                                     \
        } else {                                                                                              \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                                  \
        }                                                                                                     \
    } while (0)

// score: logits [rows*G*n_rows][logit_stride] fp32 and keys [rows][key_stride] u32 for i < Nq
hipError_t launch_score(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                        size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream);

// the same for 8 or 16 query rows per KV head, on the matrix cores
// selection keys from the heads' log-probabilities (after launch_score); scratch of
// select_logprob_scratch_floats(rows, G, max_seq) floats
size_t select_logprob_scratch_floats(int rows, int G, int max_seq);
hipError_t launch_select_logprob(const LayerView& L, int n_rows, int Nq, const float* logits, size_t logit_stride,
                                 float* scratch, uint32_t* keys, size_t key_stride, hipStream_t stream);
// after launch_score: logits and keys of the staged positions from their 16-bit keys (selection on the mixed cache)
hipError_t launch_patch_staged(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, const uint16_t* slot,
                               const int32_t* slot_idx, float* logits, size_t logit_stride, uint32_t* keys,
                               size_t key_stride, hipStream_t stream);
bool score_uses_matrix_cores(int G, int n_rows);
// one query head per KV head, two rows: integer matrix cores (q must be 16-byte aligned)
bool score_uses_int8_matrix_cores(int G, int n_rows);
hipError_t launch_score_i8(const LayerView& L, const void* q, int Nq, float sm_scale, float* logits,
                           size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream);
hipError_t launch_score_mfma(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits,
                             size_t logit_stride, uint32_t* keys, size_t key_stride, hipStream_t stream);

// top-k over keys[row][0..Nq): idx_out [rows][k], ascending, -1 padded.  Rows too long for one
// workgroup's registers are selected in two launches through the candidate buffers.
struct TopkScratch {
    uint32_t* cand_keys;   // [rows][max_parts][k]
    int32_t* cand_idx;     // [rows][max_parts][k]
    int max_parts;
};
int topk_parts(int Nq, int k);   // ranges a row of Nq keys is split into (1 = single launch)
hipError_t launch_topk(int rows, int Nq, int k, const uint32_t* keys, size_t key_stride, int32_t* idx_out,
                       const TopkScratch& scratch, hipStream_t stream);

// gather rows idx[row][j] of the host store into slot [rows][k][256] and slot_idx [rows][k];
// Nq (quantised positions of the layer) and link_shared (another gather runs beside this one) only pace the transfer
hipError_t launch_gather(const LayerView& L, int Nq, const int32_t* idx, uint16_t* slot, int32_t* slot_idx,
                         bool link_shared, hipStream_t stream);

// attend: partial pass + combine.  slot/slot_idx may be null (nothing prefetched).
struct AttendScratch {
    float* part_o;   // [rows][max_chunks][NR][128]
    float* part_ml;  // [rows][max_chunks][NR][2]  (max, sum)
    int max_chunks;
};
enum { kAttendPartial = 1, kAttendCombine = 2 };   // which of the two launches launch_attend issues
int attend_main_chunk_tokens(int NR);
// chunks the partial pass writes for NR query rows per KV head, Nq quantised and n_16bit 16-bit candidates
int attend_chunks(int NR, int Nq, int n_16bit);
int attend_extra_chunk_tokens();
int attend_max_chunks();   // chunks per row the merge kernel handles
hipError_t launch_attend(const LayerView& L, const void* q, int n_rows, int N, int Nq, float sm_scale,
                         const float* logits, size_t logit_stride, const uint16_t* slot,
                         const int32_t* slot_idx, const void* k_spec, const void* v_spec,
                         const AttendScratch& scratch, float* out, int phases, hipStream_t stream);

// the same partial pass for one query head per KV head, two rows, 2-bit values: value side on the integer matrix cores
bool attend_uses_int8_matrix_cores(const LayerView& L, int n_rows);
// keys != null: the low-bit scoring runs inside the same launch (logits are not read; the speculative row's
// selection keys go to keys, and the logits to logits_out if that is set)
hipError_t launch_attend_i8_partial(const LayerView& L, const void* q, int N, int Nq, float sm_scale, const float* logits,
                                    size_t logit_stride, const uint16_t* slot, const int32_t* slot_idx, const void* k_spec,
                                    const void* v_spec, const AttendScratch& scratch, uint32_t* keys, size_t key_stride,
                                    float* logits_out, hipStream_t stream);

// Process-wide choice of kernels, for A/B measurements of one formulation against the other
// (specache_debug_kernel_choice): bits set here send the shapes that the matrix-core kernels
// would take to the vector-ALU kernels instead.
enum { kChoiceScoreValu = 1, kChoiceAttendValu = 2, kChoiceKeepLogits = 4 };
int& kernel_choice();

// 4-bit codes: plain kernels on a layout of their own (fourbit.hip); the merge kernel, the gather, ArgTopK and
// the append are shared with the other widths
struct AttendArgs4 {
    const void* q;
    const float* logits;
    size_t logit_stride;
    const uint16_t* slot;
    const int32_t* slot_idx;
    const void* k_spec;
    const void* v_spec;
    float* part_o;
    float* part_ml;
    int max_chunks, N, Nq;
    float sm_scale;
};
hipError_t launch_flush4(const LayerView& L, const void* k_new, const void* v_new, int n_new, int N0, int Nq0, int n_flush,
                         hipStream_t stream);
hipError_t launch_export4(const LayerView& L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx, float* k_sz, uint8_t* v_codes,
                          uint16_t* v_mnmx, float* v_sz, hipStream_t stream);
hipError_t launch_score4(const LayerView& L, const void* q, int n_rows, int Nq, float sm_scale, float* logits, size_t logit_stride,
                         uint32_t* keys, size_t key_stride, hipStream_t stream);
hipError_t launch_attend4_partial(const LayerView& L, const AttendArgs4& a, int n_rows, hipStream_t stream);

// export: canonical unpacked view of rows' quantised prefix into device buffers
hipError_t launch_export(const LayerView& L, int Nq, uint8_t* k_codes, uint16_t* k_mnmx, float* k_sz,
                         uint8_t* v_codes, uint16_t* v_mnmx, float* v_sz, hipStream_t stream);

}  // namespace specache
