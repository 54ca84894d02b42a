/*
 * specache.h: C ABI of the MI355X (gfx950) SpeCache decode-step library.
 *
 * One attention layer's per-decode-step hot path of SpeCache (arXiv 2503.16163):
 * quantise and append the new KV pair to the low-bit VRAM copy C' and offload it
 * to the 16-bit CPU copy C; score the low-bit keys against the current and the
 * speculative query in one pass; select the top-k positions of the speculative
 * row; prefetch those 16-bit pairs from pinned host memory on a side stream;
 * attend over C' with the prefetched pairs substituted (Section 3.3 "Decoding",
 * Eq. 1; Section 3.4, Eq. 2-3; Appendix A algorithms "Pre-decoding", "Decoding").
 *
 * General conventions
 *   - Every function returns 0 on success or a negative specache_status.  Nothing
 *     throws, aborts or prints.  specache_last_error() gives a message for the
 *     most recent failure on that context.
 *   - "device" pointers are HIP device memory on the context's GPU, "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes
 *     in; the context owns the caches, the pinned host store, the staging slots,
 *     its scratch memory and its events.
 *   - Streams are hipStream_t values passed as void* (NULL = the null stream).
 *     The four hot calls only enqueue work; create / destroy / export_* /
 *     debug_* synchronise.
 *   - 16-bit tensors (dtype of the config: binary16 or bfloat16) are contiguous
 *     with the head dimension innermost.  head_dim is 128.
 *   - Calls on one context must come from one host thread at a time.
 *   - A context keeps one score scratch: specache_attend(layer) must follow the
 *     specache_score_topk of the same layer with no other layer scored between.
 *   - The append, the scoring call and the attend of a layer are ordered by stream
 *     order only (the residual ring and the score scratch carry no events of their
 *     own): pass all three the same stream.  Only the staging slots, the index
 *     lists and the selection keys are ordered across streams by the library.
 */
#ifndef SPECACHE_H
#define SPECACHE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum specache_status {
    SPECACHE_OK = 0,
    SPECACHE_EINVAL = -1,    /* bad argument or configuration                         */
    SPECACHE_ECAPACITY = -2, /* append would exceed max_seq                           */
    SPECACHE_ENOMEM = -3,    /* device or pinned host allocation failed               */
    SPECACHE_EHIP = -4,      /* a HIP runtime call failed                             */
    SPECACHE_ESTATE = -5     /* call order violated (slot never gathered, layer
                                mismatch between score_topk and attend, empty cache) */
} specache_status;

enum { SPECACHE_FP16 = 0, SPECACHE_BF16 = 1 };
enum { SPECACHE_1BIT_IMPROVED = 0, SPECACHE_1BIT_KIVI = 1 };
enum { SPECACHE_SELECT_MAX_LOGIT = 0, SPECACHE_SELECT_MAX_LOGPROB = 1 };
enum { SPECACHE_SELECT_LOWBIT = 0, SPECACHE_SELECT_MIXED = 1 };

/*
 * Configuration (Section 4.1 "Implementation Details" names the knobs: bit width,
 * group size, residual length, k).  All fields are validated by specache_create.
 */
typedef struct specache_config {
    int32_t n_layers;   /* >= 1                                                        */
    int32_t batch;      /* B >= 1                                                      */
    int32_t n_q_heads;  /* Hq, a multiple of n_kv_heads; Hq / Hkv in {1, 2, 4, 8} (with the
                           two query rows of a decode step: up to 16 rows per KV head) */
    int32_t n_kv_heads; /* Hkv >= 1                                                    */
    int32_t head_dim;   /* must be 128                                                 */
    int32_t bits;       /* 1 (Eq. 3), 2 (Eq. 2; the paper's two widths) or 4 (Eq. 2)    */
    int32_t group;      /* g: 32, 64 (the paper's) or 128; keys grouped per channel over
                           g tokens, values per token over g channels                  */
    int32_t residual;   /* R: multiple of g, g <= R <= 256.  Tokens are appended one at
                           a time; when N - Nq reaches R the oldest g unquantised
                           tokens are quantised.  The paper uses 64.                   */
    int32_t max_seq;    /* capacity in tokens per (batch, KV head), multiple of 64;
                           at most about 650000 (320000 with 8 query heads per KV head) */
    int32_t topk;       /* k: 1 .. 4096                                                */
    int32_t dtype;      /* SPECACHE_FP16 or SPECACHE_BF16: type of K, V, q and C       */
    float sm_scale;     /* logit scale; <= 0 selects 1/sqrt(head_dim)                  */
    int32_t one_bit_form; /* read when bits == 1: SPECACHE_1BIT_IMPROVED (Eq. 3, the paper's
                           choice) or SPECACHE_1BIT_KIVI (Eq. 2 with B = 1, the unmodified
                           quantiser that Section 4.4 / Table 5 compare against)        */
    int32_t select_form; /* how the Hq / Hkv query heads of a KV head share one index set (the
                           paper is silent): SPECACHE_SELECT_MAX_LOGIT, the largest scaled
                           low-bit logit of the speculative row over the heads, or
                           SPECACHE_SELECT_MAX_LOGPROB, the largest log-probability, each
                           head's logits less their log-sum-exp over the low-bit positions
                           (Appendix A applies ArgTopK to the softmax output).  The same
                           order when Hq == Hkv                                         */
    int32_t select_cache; /* which logits ArgTopK ranks: SPECACHE_SELECT_LOWBIT, the pure
                           low-bit logits (the "low-bit copy" of Section 1), or
                           SPECACHE_SELECT_MIXED, those of the mixed cache of Eq. 1: the
                           positions staged by the layer's last specache_gather are scored
                           with their 16-bit keys (Appendix A "Decoding" computes one A)  */
    int32_t async_select; /* 0: specache_score_topk runs entirely on the caller's stream.
                           1: ArgTopK runs on a stream of the library's own, after the
                           scoring pass, so that the caller's stream goes straight on to
                           specache_attend (which does not need the selection) while the
                           positions are ranked beside it.  specache_gather orders itself
                           after the selection either way; on the caller's stream
                           topk_idx_out is complete only after the next
                           specache_score_topk call (of any layer), which waits for it,
                           or after a device synchronise.
                           2 (SPECACHE_SELECT_STREAM_GATHER): ArgTopK runs on the gather's
                           side stream, directly ahead of the gather: the caller uses
                           specache_score + specache_select_gather in place of
                           specache_score_topk + specache_gather.  Every layer then has a
                           key array of its own (4 bytes per cached position and KV head)
                           and a layer-step needs two event records and two event waits
                           between the streams, against three and four with 1; each
                           costs the issuing thread several microseconds                */
} specache_config;

enum { SPECACHE_SELECT_STREAM_CALLER = 0, SPECACHE_SELECT_STREAM_OWN = 1, SPECACHE_SELECT_STREAM_GATHER = 2 };

typedef struct specache_ctx specache_ctx;

/* Allocates every buffer for all layers on the current HIP device (including
 * n_layers * B * Hkv * max_seq * 512 bytes of pinned host memory for C).
 * *out is NULL on failure. */
int specache_create(const specache_config* cfg, specache_ctx** out);

/* Synchronises the device and frees everything.  NULL is allowed. */
int specache_destroy(specache_ctx* ctx);

/* Message of the most recent failed call on ctx (never NULL; "" if none).
 * With ctx == NULL returns the message of the last failed specache_create. */
const char* specache_last_error(const specache_ctx* ctx);

/* Token counts of a layer: N tokens cached, of which the first Nq are quantised
 * (Nq is a multiple of g; N - Nq < R tokens sit 16-bit in the VRAM residual). */
int specache_counts(const specache_ctx* ctx, int32_t layer, int32_t* n_tokens, int32_t* n_quantized);

/* Host-only helper, no GPU work: how many groups of g tokens an append of n_new
 * tokens moves from the residual into C' under the residual policy above, for a
 * layer holding n_tokens of which n_quantized are quantised.
 * Errors: EINVAL (inconsistent counts, null output). */
int specache_plan_append(int32_t residual, int32_t group, int32_t n_tokens, int32_t n_quantized, int32_t n_new,
                         int32_t* n_flush_groups);

/*
 * Quant + Offload of new KV pairs (Appendix A "Decoding": C' = [C', Quant(K_t, V_t)],
 * C = [C, Offload(C_t)]; quantiser of Eq. 2 for 2 bits, Eq. 3 for 1 bit).
 * k_new, v_new: device, 16-bit, [B, Hkv, n_new, 128].  Defined as n_new single-token
 * appends in order (n_new = the prompt length performs the bulk load after
 * prefill).  Every token is written to the pinned host store and to the VRAM
 * residual; full groups leaving the residual are quantised and packed.
 * Errors: EINVAL (null pointer, n_new < 0, bad layer), ECAPACITY (N + n_new >
 * max_seq; nothing is appended).
 */
int specache_quantize_append(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new,
                             int32_t n_new, void* stream);

/*
 * Low-bit scoring and ArgTopK (Appendix A "Decoding": A = Softmax(Q K^T) on the
 * low-bit keys, K_{t+1} = ArgTopK(A_{1,:}); "Pre-decoding" with n_rows = 1).
 * q: device, 16-bit, [B, Hq, n_rows, 128], 16-byte aligned, n_rows in {1, 2}; row 0 is
 * the output token's query, row 1 the speculative token's.  For every quantised position
 * i < Nq and every query head the logit sm_scale * q . K'_i is computed from the
 * packed keys (read once for all rows and heads of a KV head) and kept in the
 * context for the following specache_attend.  The selection score of position i
 * for a KV head is the maximum over its Hq/Hkv query heads of the LAST row's
 * logit.  topk_idx_out: device int32 [B, Hkv, k] (see async_select for when it is
 * complete); receives the min(k, Nq)
 * positions with the largest selection score (ties to the lower index) in
 * ascending index order, the rest -1.
 * Errors: EINVAL (also a q that is not 16-byte aligned), ESTATE (no call order
 * requirement fails here; Nq = 0 is allowed and yields all -1).
 */
int specache_score_topk(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows,
                        int32_t* topk_idx_out, void* stream);

/*
 * Pre-fetch(C_K) (Section 3.3: the selected 16-bit pairs are fetched from CPU
 * memory in parallel with later computation).  idx: device int32 [B, Hkv, k],
 * ascending with -1 padding (the format specache_score_topk writes).  Copies
 * the selected (K, V) rows from the pinned host store into staging slot
 * `slot` (0 or 1) of the layer, together with the index list.  Enqueued on
 * side_stream; the library orders it after the layer's last specache_score_topk
 * and after the last specache_attend that read this slot, and orders later
 * specache_attend calls on this slot after it (stream order where the calls
 * share a stream, events of its own otherwise).  A stream handed to one of the
 * hot calls must stay alive until the context is destroyed: a later call may
 * still record an event on it.
 * Reusing a slot discards what it held (the paper's eviction).
 * Callers that step several layers do well to alternate two side streams by layer:
 * two gathers then share the link and cover each other's launch gaps (the library
 * notices the alternation and paces each gather accordingly).
 * Errors: EINVAL (slot not 0/1, null idx, bad layer).
 */
int specache_gather(specache_ctx* ctx, int32_t layer, const int32_t* idx, int32_t slot, void* side_stream);

/*
 * The same two steps split at the other seam (contexts created with async_select =
 * SPECACHE_SELECT_STREAM_GATHER only; ESTATE otherwise).
 * specache_score: the scoring pass of specache_score_topk alone, on `stream`: the
 * logits for the following specache_attend and the layer's selection keys.
 * specache_select_gather: ArgTopK of those keys (Appendix A "Decoding":
 * K_{t+1} = ArgTopK(A_{1,:})) followed by Pre-fetch(C_K) of the selected pairs into
 * staging slot `slot`, both on side_stream, ordered after the layer's last
 * specache_score and after the last specache_attend that read the slot.
 * topk_idx_out (device int32 [B, Hkv, k], format as in specache_score_topk) is written
 * on side_stream; it is complete when the gather is (a specache_attend on that slot
 * follows both).  slot = -1: the selection alone, nothing is fetched (topk_idx_out is
 * then complete for work enqueued on side_stream after the call, or after a device
 * synchronise).  The next specache_score of the layer orders itself after this
 * selection.  Arguments, ownership and slot semantics as in specache_score_topk and
 * specache_gather.
 * Errors: EINVAL, ESTATE (wrong mode; select_gather without a specache_score before it).
 */
int specache_score(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, void* stream);
int specache_select_gather(specache_ctx* ctx, int32_t layer, int32_t* topk_idx_out, int32_t slot, void* side_stream);

/*
 * specache_quantize_append of ONE token followed by specache_score, as one call (same context
 * mode as specache_score).  k_new, v_new: device, 16-bit, [B, Hkv, 1, 128], as in
 * specache_quantize_append; q, n_rows, stream as in specache_score.  When the token does not
 * complete a group that leaves the residual, the scoring launch itself carries the Offload
 * of the new pair (Appendix A "Decoding") to the CPU copy and to the residual, which saves
 * a kernel launch per layer-step; otherwise the two steps run one after the other.  Results
 * are those of the two calls.
 * Errors: those of the two calls.
 */
int specache_append_score(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                          int32_t n_rows, void* stream);

/*
 * Mixed attention, Eq. 1: O = Attn([T_t, T'_{t+1}], C' u C_K).
 * q as in specache_score_topk (same n_rows).  Candidates of every row: quantised
 * positions i < Nq with the staged 16-bit pair where i is in the slot's index
 * list and the dequantised low-bit pair elsewhere; the 16-bit residual positions
 * Nq <= i < N; and, for the last row only when k_spec/v_spec are non-NULL
 * (device, 16-bit, [B, Hkv, 1, 128]), that transient pair (it is never appended).
 * slot = -1: nothing prefetched (pre-decoding, or the k = 0 baseline).
 * out: device float32 [B, Hq, n_rows, 128].
 * Errors: EINVAL; ESTATE (slot never gathered, layer not the last one scored,
 * n_rows differs from the scoring call, the cache grew since the scoring call,
 * or no candidate at all).
 */
int specache_attend(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                    const void* v_spec, int32_t slot, float* out, void* stream);

/*
 * specache_score followed by specache_attend of the same layer, as one call (contexts created
 * with async_select = SPECACHE_SELECT_STREAM_GATHER; ESTATE otherwise): Appendix A "Decoding",
 * A = Softmax(Q K^T) on the mixed cache and O = A V, with the low-bit logits of both rows computed
 * on the way and the speculative row's selection keys left for the following
 * specache_select_gather (which may be enqueued right after this call: the slot it fills is the
 * other one).  With one query head per KV head, two query rows, 1- or 2-bit codes and selection on the
 * low-bit logits, one pass over a chunk of 512 positions reads its packed keys, keeps the logits
 * on the chip, and reads its packed values: the logits never travel to memory and back, and the
 * layer-step has one launch less.  Every other shape or option runs the two calls one after the
 * other.  Results are those of the two calls (the attention output to the 2e-3 bar: the softmax
 * partials are formed per 128 positions instead of per 512); specache_debug_logits afterwards
 * needs SPECACHE_KEEP_ONE_PASS_LOGITS.  Arguments as in specache_score and specache_attend.
 * Errors: those of the two calls.
 */
int specache_score_attend(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                          const void* v_spec, int32_t slot, float* out, void* stream);

/*
 * specache_quantize_append of ONE token followed by specache_score_attend, as one call: a whole layer-step on
 * the caller's stream but for the selection and the prefetch (Appendix A "Decoding": C' = [C', Quant(K_t, V_t)],
 * C = [C, Offload(C_t)], A, O).  k_new, v_new: device, 16-bit, [B, Hkv, 1, 128].  Where specache_score_attend
 * runs as one launch and the token does not complete a group that leaves the residual, that launch also
 * carries the Offload of the new pair to the CPU copy and to the residual (the attention reads the pair from
 * k_new / v_new, which must stay unchanged until the launch has run): one launch less per layer-step.
 * Otherwise the steps run one after the other.  Results are those of the separate calls.
 * Errors: those of the separate calls.
 */
int specache_append_score_attend(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                                 int32_t n_rows, const void* k_spec, const void* v_spec, int32_t slot, float* out,
                                 void* stream);

/*
 * One layer-step of Appendix A "Decoding" as ONE call, for the two query rows of a decode step:
 * specache_append_score_attend(ctx, layer, k_new, v_new, q, 2, k_spec, v_spec, read_slot, out, stream), then
 * specache_select_gather(ctx, layer, topk_idx_out, fill_slot, side_stream): the new pair is appended, both rows
 * are scored and attend over the mixed cache (the pairs staged in read_slot in place of their low-bit copies),
 * and on the side stream K_{t+1} = ArgTopK of the speculative row is selected and its pairs are fetched into
 * fill_slot for the next step.  Nothing but the two calls: a stepping loop in an interpreted language pays for
 * one call per layer instead of two.  Arguments, results and errors are those of the two calls (the first
 * failure is returned and the second call is then not made).
 */
int specache_decode_step(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                         const void* k_spec, const void* v_spec, int32_t read_slot, float* out, void* stream,
                         int32_t* topk_idx_out, int32_t fill_slot, void* side_stream);

/*
 * specache_attend for callers that must not allocate device memory around the call and want
 * the call's scratch out of the context: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels, same results; the partial
 * results of the split over the sequence (rows x chunks x query rows x 130 floats) go to a
 * 16 MiB array that is part of the library's device image (one copy per GPU, held until the
 * process ends) instead of the context's scratch buffer.  The call allocates and frees nothing.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * contexts) race; calls ordered by one stream do not.  Nothing in the array has to start at
 * zero (the merge reads only what the partial pass of the same call wrote).
 * Errors: those of specache_attend; ECAPACITY when the partial results of this call do not fit
 * the array (nothing is launched; use specache_attend); EHIP when the array's address cannot
 * be obtained on the current device.
 */
int specache_attend_static(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                           const void* v_spec, int32_t slot, float* out, void* stream);

/*
 * Parity hooks (synchronise the device; all output pointers are host memory and
 * may be NULL to skip that array).
 *
 * specache_export_quantized: canonical view of C' of one layer.
 *   k_codes u8 [B,Hkv,Nq,128]      one code per byte
 *   k_minmax u16 [B,Hkv,Nq/g,128,2] stored (min,max) bit patterns per key group
 *   k_scale_zero f32 [B,Hkv,Nq/g,128,2] (s,z) as the kernels derive them on the GPU
 *   v_codes u8 [B,Hkv,Nq,128], v_minmax u16 [B,Hkv,Nq,128/g,2], v_scale_zero f32 [...,2]
 * specache_export_rows: 16-bit rows [first, first+count) of the host store C,
 *   out u16 [B,Hkv,count,2,128] (K row then V row per token).
 * specache_debug_logits: the logits kept by the last specache_score_topk,
 *   out f32 [B,Hq,n_rows,Nq].
 */
int specache_export_quantized(specache_ctx* ctx, int32_t layer, uint8_t* k_codes, uint16_t* k_minmax,
                              float* k_scale_zero, uint8_t* v_codes, uint16_t* v_minmax, float* v_scale_zero);
int specache_export_rows(specache_ctx* ctx, int32_t layer, int32_t first, int32_t count, uint16_t* out);
int specache_debug_logits(specache_ctx* ctx, float* out);

/*
 * Test hook for the two-stream staging protocol: enqueues on `stream` a fill of staging slot
 * `slot` (0 or 1) of the layer with 0xFFFF words, a NaN in binary16 and bfloat16 alike, so that
 * an attend that reads the slot before the next gather has rewritten it returns NaNs.  The
 * slot's index list is left as it is.  The caller orders the fill (put it on the stream of the
 * attend that read the slot last, behind that attend).
 * Errors: EINVAL.
 */
int specache_debug_poison_slot(specache_ctx* ctx, int32_t layer, int32_t slot, void* stream);

/*
 * Test hook, process-wide: the nth allocating call (device memory, pinned host memory, events,
 * streams; counted from 1) of the NEXT specache_create reports out-of-memory without running, so
 * that the way create backs out of a half-built context (everything allocated so far is freed,
 * *out stays NULL, ENOMEM) can be tested at every point without exhausting a machine's memory.
 * 0 switches it off; the setting is consumed by that one create.  Errors: EINVAL (nth < 0).
 */
int specache_debug_fail_alloc(int32_t nth);

/*
 * Measurement hook, process-wide: which formulation of the two streaming kernels runs for one
 * query head per KV head and two query rows.  0 (the default): the integer matrix cores; a flag
 * set: that kernel's vector-ALU formulation instead (same results to the parity bars), so that
 * the two can be timed and profiled against each other.  Takes effect for calls made afterwards.
 * Errors: EINVAL (unknown flag).
 */
enum { SPECACHE_SCORE_ON_VECTOR_ALU = 1, SPECACHE_ATTEND_ON_VECTOR_ALU = 2,
       SPECACHE_KEEP_ONE_PASS_LOGITS = 4 /* specache_score_attend also writes its logits out, for specache_debug_logits */ };
int specache_debug_kernel_choice(int32_t flags);

/*
 * Measurement hook.  While enabled, every hot call brackets each of its kernel
 * phases with a pair of HIP events on the stream the phase is launched on.
 * specache_timing synchronises the device, adds up the elapsed time of all
 * pairs recorded since the previous call into total_us[SPECACHE_K_COUNT] (host,
 * microseconds) and launches[SPECACHE_K_COUNT] (host), forgets them, and then
 * switches recording on (enable != 0) or off.  Either output may be NULL.
 * The scoring, ArgTopK and attention kernels are timed by events that their own dispatch
 * packets carry (start and stop of the kernel as a profiler sees them); the other phases by
 * event records around the launch.
 */
enum {
    SPECACHE_K_FLUSH = 0,       /* quantise + pack of full groups            */
    SPECACHE_K_APPEND_COPY = 1, /* offload to host store + residual update   */
    SPECACHE_K_SCORE = 2,       /* fused dequantise + q.K^T                  */
    SPECACHE_K_TOPK = 3,        /* radix select + ordered compaction         */
    SPECACHE_K_GATHER = 4,      /* host-link gather (side stream)            */
    SPECACHE_K_ATTEND = 5,      /* mixed attention: partial pass over chunks */
    SPECACHE_K_ATTEND_COMBINE = 6, /* mixed attention: merge of the chunks    */
    SPECACHE_K_SCORE_ATTEND = 7, /* scoring and partial pass of specache_score_attend in one launch */
    SPECACHE_K_COUNT = 8
};
int specache_timing(specache_ctx* ctx, int32_t enable, double* total_us, int64_t* launches);

/*
 * Roofline denominators, measured on the current HIP device (no context; each call allocates
 * its buffers, synchronises, and frees them; not part of the decode path).
 * specache_measure_hbm_read: median rate, in GB/s (1e9 bytes/s), of `reps` launches of a plain
 *   kernel that reads `bytes` of device memory once with 16-byte loads (after one untimed launch).
 * specache_measure_link: the same for the host link, over `bytes` of pinned host memory:
 *   *memcpy_gbs for hipMemcpyAsync to device memory, *kernel_gbs for a kernel that reads the
 *   pinned buffer directly (contiguously; the gather of Section 3.3's prefetch reads 512-byte
 *   rows the same way).  Either output may be NULL.
 * bytes >= 1 MiB, 1 <= reps <= 1000.  Errors: EINVAL, ENOMEM, EHIP.
 */
int specache_measure_hbm_read(int64_t bytes, int32_t reps, double* gbs);
int specache_measure_link(int64_t bytes, int32_t reps, double* memcpy_gbs, double* kernel_gbs);

#ifdef __cplusplus
}
#endif
#endif /* SPECACHE_H */
