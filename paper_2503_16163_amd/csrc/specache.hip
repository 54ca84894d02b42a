// C ABI of the SpeCache decode-step library (see include/specache.h): argument
// checks, buffer ownership, the append bookkeeping of the residual policy and the
// stream/event protocol between the main stream and the prefetch side stream.
// All arithmetic of the method lives in the kernels.
#include "../../include/specache.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"
#include "layout.h"
#include <cstdlib>

using namespace specache;

namespace specache {
LaunchEvents& pending_launch_events() {
    static thread_local LaunchEvents le;
    return le;
}
int& kernel_choice() {
    static int choice = 0;
    return choice;
}
}  // namespace specache

namespace {

struct Layer {
    LayerView view{};
    int N = 0, Nq = 0;
    void* host_alloc = nullptr;
    uint16_t* slot[2] = {nullptr, nullptr};
    int32_t* slot_idx[2] = {nullptr, nullptr};
    bool slot_filled[2] = {false, false};
    hipEvent_t gathered[2] = {nullptr, nullptr};
    hipStream_t gather_stream[2] = {nullptr, nullptr};
    // Ordering of a slot's reader (attend) before its next writer (gather).  An event record costs
    // the stream about as much as a small kernel, so attend records `attended` only when the later
    // gather could not be ordered otherwise: an attend enqueued on the stream of the layer's last
    // score_topk precedes, in that stream, the next score_topk's `idx_ready` record, which every
    // gather waits for.  The sequence numbers tell whether that record came after the attend.
    hipEvent_t attended[2] = {nullptr, nullptr};
    bool attended_recorded[2] = {false, false};
    hipStream_t attend_stream[2] = {nullptr, nullptr};
    uint64_t attend_seq[2] = {0, 0};     // 0: no attend has read the slot
    hipEvent_t idx_ready = nullptr;
    bool idx_ready_recorded = false;
    hipStream_t idx_ready_stream = nullptr;       // where idx_ready was recorded
    hipStream_t select_origin_stream = nullptr;   // the stream score_topk was called on (the same, unless ArgTopK runs aside)
    uint64_t idx_ready_seq = 0;
    const int32_t* last_gather_idx = nullptr;
    int last_gather_slot = -1;
    // ArgTopK on the gather's stream (specache_score + specache_select_gather): the layer has a key
    // array of its own, which the selection reads on the side stream while the caller's stream goes
    // on to other layers.  The next scoring pass of the layer waits for the gather that followed
    // that selection; the attend after it then needs no wait of its own for the same slot.
    uint32_t* keys = nullptr;            // [rows][logit_stride]
    bool keys_valid = false;
    int keys_Nq = 0;
    int keys_reader_slot = -1;           // slot of the select_gather that read `keys` last
    bool gathered_waited_set[2] = {false, false};
    hipStream_t gathered_waited[2] = {nullptr, nullptr};   // stream that has already waited for gathered[s]
    hipEvent_t selected = nullptr;       // a selection without a gather behind it (select_gather with slot -1)
    bool selected_pending = false;
    hipStream_t selected_stream = nullptr;
};

thread_local std::string g_create_error;
int g_fail_alloc_at = 0;   // specache_debug_fail_alloc

}  // namespace

struct specache_ctx {
    specache_config cfg{};
    int device = 0;
    float sm_scale = 0.f;
    std::vector<Layer> layers;
    float* logits = nullptr;     // [rows*G*2][logit_stride]
    uint32_t* keys = nullptr;    // [rows][logit_stride]
    float* lse = nullptr;        // (max, sum) per slice of every head's speculative row (log-probability selection)
    size_t logit_stride = 0;
    AttendScratch scratch{};
    TopkScratch topk_scratch{};
    int scored_layer = -1, scored_rows = 0, scored_N = 0, scored_Nq = 0;
    bool logits_kept = false;    // the last scoring pass left its logits in `logits` (the one-pass score + attend need not)
    uint64_t seq = 0;            // counts the calls that order streams (see Layer)
    hipStream_t last_gather_stream = nullptr;   // stream of the previous specache_gather, of any layer
    bool last_gather_stream_set = false;
    // ArgTopK on a stream of the library's own (async_select): the scoring pass stays on the caller's
    // stream, which goes on to the attention kernels while the selection runs beside them
    bool async_select = false;
    hipStream_t select_stream = nullptr;
    hipEvent_t scored = nullptr;            // scoring pass done (recorded on the caller's stream)
    hipEvent_t last_select = nullptr;       // idx_ready of the most recent selection: it has read ctx->keys
    // selections on the gather's stream: those of two side streams may overlap, so the candidate
    // arrays of the two-launch ArgTopK exist twice, each remembering its last user
    bool select_on_gather = false;
    struct SelectScratch { TopkScratch s{}; bool used = false; hipStream_t stream = nullptr; hipEvent_t done = nullptr; };
    SelectScratch select_scratch[2];
    int select_scratch_next = 0;
    std::string err;
    // optional per-kernel timing: (start, stop) event pairs recorded around each launch
    bool timing = false;
    std::vector<hipEvent_t> ev_pool;
    struct Span { int kind; hipEvent_t a, b; };
    std::vector<Span> spans;
};

namespace {

int fail(specache_ctx* ctx, int code, const std::string& msg) {
    if (ctx) ctx->err = msg; else g_create_error = msg;
    return code;
}

int fail_hip(specache_ctx* ctx, hipError_t e, const char* what) {
    (void)hipGetLastError();
    return fail(ctx, e == hipErrorOutOfMemory ? SPECACHE_ENOMEM : SPECACHE_EHIP,
                std::string(what) + ": " + hipGetErrorString(e));
}

#define SPC_HIP(ctx, call)                                     \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return fail_hip(ctx, e_, #call); \
    } while (0)

// Brackets one launcher call with a pair of timing events when timing is on.  on_kernel: the
// events are handed to the launcher's first SPC_LAUNCH instead, which times that kernel alone.
struct TimedLaunch {
    specache_ctx* ctx;
    hipStream_t st;
    int kind;
    bool on_kernel;
    hipEvent_t a = nullptr, b = nullptr;
    static hipEvent_t take(specache_ctx* c) {
        if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        return hipEventCreate(&e) == hipSuccess ? e : nullptr;
    }
    TimedLaunch(specache_ctx* c, hipStream_t s, int k, bool kernel_events = false)
        : ctx(c), st(s), kind(k), on_kernel(kernel_events) {
        if (!c->timing) return;
        a = take(c);
        b = take(c);
        if (!a || !b) return;
        if (on_kernel) pending_launch_events() = LaunchEvents{a, b};
        else (void)hipEventRecord(a, st);
    }
    ~TimedLaunch() {
        if (!a || !b) return;
        if (on_kernel) {
            LaunchEvents& le = pending_launch_events();
            if (le.stop) {   // no kernel took them (nothing was launched): no span
                le = LaunchEvents{};
                ctx->ev_pool.push_back(a);
                ctx->ev_pool.push_back(b);
                return;
            }
        } else {
            (void)hipEventRecord(b, st);
        }
        ctx->spans.push_back({kind, a, b});
    }
};

// An ordering event completed by a kernel's own dispatch packet instead of a record behind it: one call
// into the runtime less per event, and the issuing thread's calls are what bounds a step with little to
// fetch.  Between arm() and landed() exactly one launcher runs; landed() is false when that launcher
// launched nothing or when the launch carries timing events (the caller then records the event itself).
struct CarriedEvent {
    bool armed = false;
    CarriedEvent(specache_ctx* c, hipEvent_t ev) {
        if (c->timing || !ev) return;
        pending_launch_events() = LaunchEvents{nullptr, ev};
        armed = true;
    }
    bool landed() {
        if (!armed) return false;
        armed = false;
        LaunchEvents& le = pending_launch_events();
        const bool taken = le.stop == nullptr;
        le = LaunchEvents{};
        return taken;
    }
    ~CarriedEvent() { if (armed) pending_launch_events() = LaunchEvents{}; }
};

int check_ctx_layer(specache_ctx* ctx, int32_t layer) {
    if (!ctx) return SPECACHE_EINVAL;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, SPECACHE_EINVAL, "layer out of range");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return fail(ctx, SPECACHE_EINVAL, "the context's device is not the current HIP device");
    return SPECACHE_OK;
}

void free_all(specache_ctx* ctx) {
    for (Layer& L : ctx->layers) {
        (void)hipFree(L.view.kc);
        (void)hipFree(L.view.km);
        (void)hipFree(L.view.vc);
        (void)hipFree(L.view.vm);
        (void)hipFree(L.view.ring);
        if (L.host_alloc) (void)hipHostFree(L.host_alloc);
        for (int s = 0; s < 2; ++s) {
            (void)hipFree(L.slot[s]);
            (void)hipFree(L.slot_idx[s]);
            if (L.gathered[s]) (void)hipEventDestroy(L.gathered[s]);
            if (L.attended[s]) (void)hipEventDestroy(L.attended[s]);
        }
        if (L.idx_ready) (void)hipEventDestroy(L.idx_ready);
        if (L.selected) (void)hipEventDestroy(L.selected);
        (void)hipFree(L.keys);
    }
    for (auto& ss : ctx->select_scratch) { (void)hipFree(ss.s.cand_keys); (void)hipFree(ss.s.cand_idx); }
    for (auto& sp : ctx->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
    (void)hipFree(ctx->logits);
    if (ctx->select_stream) (void)hipStreamDestroy(ctx->select_stream);
    if (ctx->scored) (void)hipEventDestroy(ctx->scored);
    (void)hipFree(ctx->keys);
    (void)hipFree(ctx->lse);
    (void)hipFree(ctx->scratch.part_o);
    (void)hipFree(ctx->scratch.part_ml);
    (void)hipFree(ctx->topk_scratch.cand_keys);
    (void)hipFree(ctx->topk_scratch.cand_idx);
}

// The scoring pass of one layer on stream st: low-bit logits of every query row, selection keys of
// the last row, and the optional rewrites of those keys (mixed-cache selection, log-probability form).
// done / done_carried: an event to complete when the keys are final; *done_carried tells whether the scoring
// launch's own dispatch packet does that (only where no rewrite of the keys follows it).
int score_phase(specache_ctx* ctx, Layer& L, const void* q, int n_rows, uint32_t* keys, hipStream_t st,
                const LayerView* fused_view = nullptr, hipEvent_t done = nullptr, bool* done_carried = nullptr) {
    if (L.Nq > 0) {
        TimedLaunch t(ctx, st, SPECACHE_K_SCORE, /*kernel_events=*/true);
        const bool rewrites = (ctx->cfg.select_cache == SPECACHE_SELECT_MIXED && L.last_gather_slot >= 0) ||
                              (ctx->cfg.select_form == SPECACHE_SELECT_MAX_LOGPROB && L.view.G > 1);
        CarriedEvent carried(ctx, rewrites ? nullptr : done);
        SPC_HIP(ctx, launch_score(fused_view ? *fused_view : L.view, q, n_rows, L.Nq, ctx->sm_scale, ctx->logits, ctx->logit_stride, keys,
                                  ctx->logit_stride, st));
        if (done_carried) *done_carried = carried.landed();
        // selection on the mixed cache: the positions staged by the layer's last gather are scored with
        // their 16-bit keys (that slot is the one the coming attend reads; the next gather into it
        // waits for this stream's next selection event, so it cannot overtake the patch)
        if (ctx->cfg.select_cache == SPECACHE_SELECT_MIXED && L.last_gather_slot >= 0) {
            const int sl = L.last_gather_slot;
            if (L.gather_stream[sl] != st) SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[sl], 0));
            SPC_HIP(ctx, launch_patch_staged(L.view, q, n_rows, L.Nq, ctx->sm_scale, L.slot[sl], L.slot_idx[sl], ctx->logits,
                                             ctx->logit_stride, keys, ctx->logit_stride, st));
        }
        // several query heads per KV head and the log-probability form: the keys are rewritten from
        // the logits shifted by every head's log-sum-exp (one head: same order, nothing to do)
        if (ctx->cfg.select_form == SPECACHE_SELECT_MAX_LOGPROB && L.view.G > 1)
            SPC_HIP(ctx, launch_select_logprob(L.view, n_rows, L.Nq, ctx->logits, ctx->logit_stride, ctx->lse, keys,
                                               ctx->logit_stride, st));
    }
    return SPECACHE_OK;
}

// Orders a gather into `slot` on stream st after the attend that read the slot last.
int order_gather_after_attend(specache_ctx* ctx, Layer& L, int slot, hipStream_t st) {
    if (L.attend_seq[slot] != 0 && L.attend_stream[slot] != st) {
        const bool behind_idx_ready = L.idx_ready_recorded && L.attend_stream[slot] == L.select_origin_stream &&
                                      L.attend_seq[slot] < L.idx_ready_seq;
        if (!L.attended_recorded[slot] && !behind_idx_ready) {
            // a second gather into the slot without a new score_topk in between: record now, on the
            // attend's stream, which orders this gather after everything enqueued there so far
            SPC_HIP(ctx, hipEventRecord(L.attended[slot], L.attend_stream[slot]));
            L.attended_recorded[slot] = true;
        }
        if (L.attended_recorded[slot]) SPC_HIP(ctx, hipStreamWaitEvent(st, L.attended[slot], 0));
    }
    return SPECACHE_OK;
}

// Launches the gather of `idx` into `slot` on st and records its completion.
int gather_phase(specache_ctx* ctx, Layer& L, int Nq, const int32_t* idx, int slot, hipStream_t st) {
    // the slot's previous gather, if it ran on another stream that this one has not waited for
    if (L.slot_filled[slot] && L.gather_stream[slot] != st && !(L.gathered_waited_set[slot] && L.gathered_waited[slot] == st))
        SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[slot], 0));
    bool gathered_carried = false;
    {
        TimedLaunch t(ctx, st, SPECACHE_K_GATHER);
        CarriedEvent gathered(ctx, L.gathered[slot]);
        // a caller that alternates side streams has two gathers on the link at a time
        const bool link_shared = ctx->last_gather_stream_set && ctx->last_gather_stream != st;
        SPC_HIP(ctx, launch_gather(L.view, Nq, idx, L.slot[slot], L.slot_idx[slot], link_shared, st));
        gathered_carried = gathered.landed();
        ctx->last_gather_stream = st;
        ctx->last_gather_stream_set = true;
    }
    if (!gathered_carried) SPC_HIP(ctx, hipEventRecord(L.gathered[slot], st));
    L.gather_stream[slot] = st;
    L.gathered_waited_set[slot] = false;
    L.slot_filled[slot] = true;
    L.last_gather_idx = idx;
    L.last_gather_slot = slot;
    return SPECACHE_OK;
}

// ---- scratch memory for callers that cannot allocate (specache_attend_static) ----------------------
// A file-scope device array holds the attention partials of such a call.  Every GPU the library
// runs on carries its own copy at its own address; in host code the array's name is only a handle
// for hipGetSymbolAddress, never an address to hand to a kernel.  The address is looked up once
// per device, with that device current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
float* g_static_scratch[kMaxDevices] = {};

int static_scratch_of_current_device(specache_ctx* ctx, float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(ctx, SPECACHE_EINVAL, "device ordinal beyond the static scratch table");
    if (!g_static_scratch[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail_hip(ctx, e != hipSuccess ? e : hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        g_static_scratch[dev] = (float*)ptr;
    }
    *out = g_static_scratch[dev];
    return SPECACHE_OK;
}

}  // namespace

extern "C" {

int specache_plan_append(int32_t residual, int32_t group, int32_t n_tokens, int32_t n_quantized, int32_t n_new,
                         int32_t* n_flush_groups) {
    if (group <= 0 || residual < group || residual % group || n_tokens < n_quantized || n_quantized < 0 ||
        n_tokens - n_quantized >= residual || n_new < 0 || !n_flush_groups)
        return SPECACHE_EINVAL;
    const long total = (long)(n_tokens - n_quantized) + n_new;
    *n_flush_groups = total >= residual ? (int32_t)((total - residual) / group + 1) : 0;
    return SPECACHE_OK;
}

int specache_create(const specache_config* cfg, specache_ctx** out) {
    if (out) *out = nullptr;
    if (!cfg || !out) return fail(nullptr, SPECACHE_EINVAL, "null config or output pointer");
    const specache_config& c = *cfg;
    if (c.n_layers < 1 || c.batch < 1 || c.n_kv_heads < 1 || c.n_q_heads < 1)
        return fail(nullptr, SPECACHE_EINVAL, "n_layers, batch and head counts must be positive");
    if (c.n_q_heads % c.n_kv_heads) return fail(nullptr, SPECACHE_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    const int G = c.n_q_heads / c.n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return fail(nullptr, SPECACHE_EINVAL, "n_q_heads / n_kv_heads must be 1, 2, 4 or 8");
    if (c.head_dim != kD) return fail(nullptr, SPECACHE_EINVAL, "head_dim must be 128");
    if (c.bits != 1 && c.bits != 2 && c.bits != 4) return fail(nullptr, SPECACHE_EINVAL, "bits must be 1, 2 or 4");
    if (c.one_bit_form != SPECACHE_1BIT_IMPROVED && c.one_bit_form != SPECACHE_1BIT_KIVI)
        return fail(nullptr, SPECACHE_EINVAL, "one_bit_form must be SPECACHE_1BIT_IMPROVED or SPECACHE_1BIT_KIVI");
    if (c.async_select < 0 || c.async_select > 2) return fail(nullptr, SPECACHE_EINVAL, "async_select must be 0, 1 or 2");
    if (c.select_cache != SPECACHE_SELECT_LOWBIT && c.select_cache != SPECACHE_SELECT_MIXED)
        return fail(nullptr, SPECACHE_EINVAL, "select_cache must be SPECACHE_SELECT_LOWBIT or SPECACHE_SELECT_MIXED");
    if (c.select_form != SPECACHE_SELECT_MAX_LOGIT && c.select_form != SPECACHE_SELECT_MAX_LOGPROB)
        return fail(nullptr, SPECACHE_EINVAL, "select_form must be SPECACHE_SELECT_MAX_LOGIT or SPECACHE_SELECT_MAX_LOGPROB");
    if (c.group != 32 && c.group != 64 && c.group != 128)
        return fail(nullptr, SPECACHE_EINVAL, "group must be 32, 64 or 128");
    if (c.residual < c.group || c.residual % c.group || c.residual > 256)
        return fail(nullptr, SPECACHE_EINVAL, "residual must be a multiple of group in [group, 256]");
    if (c.max_seq < 64 || c.max_seq % 64) return fail(nullptr, SPECACHE_EINVAL, "max_seq must be a positive multiple of 64");
    if (c.topk < 1 || c.topk > 4096) return fail(nullptr, SPECACHE_EINVAL, "topk must be in [1, 4096]");
    if (c.dtype != SPECACHE_FP16 && c.dtype != SPECACHE_BF16) return fail(nullptr, SPECACHE_EINVAL, "dtype must be fp16 or bf16");
    {
        // attend splits a row into chunks whose partial results one workgroup merges
        int most = 0;
        for (int n = 1; n <= 2; ++n) {
            const int ch = attend_main_chunk_tokens(G * n), ec = attend_extra_chunk_tokens();
            const int chunks = (c.max_seq + ch - 1) / ch + (c.topk + c.residual + 1 + ec - 1) / ec;
            most = chunks > most ? chunks : most;
        }
        if (most > attend_max_chunks())
            return fail(nullptr, SPECACHE_EINVAL, "max_seq is beyond what attend splits into chunks (about 650000 tokens, "
                                                  "320000 with 8 query heads per KV head)");
    }

    specache_ctx* ctx = new (std::nothrow) specache_ctx();
    if (!ctx) return fail(nullptr, SPECACHE_ENOMEM, "host allocation failed");
    ctx->cfg = c;
    ctx->sm_scale = c.sm_scale > 0.f ? c.sm_scale : 1.0f / std::sqrt((float)kD);
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) { delete ctx; return fail_hip(nullptr, e, "hipGetDevice"); }

    const int rows = c.batch * c.n_kv_heads;
    const size_t cap = (size_t)c.max_seq;
    ctx->layers.resize(c.n_layers);
    auto bail = [&](hipError_t err, const char* what) {
        const int rc = fail_hip(nullptr, err, what);
        free_all(ctx);
        delete ctx;
        return rc;
    };
    // specache_debug_fail_alloc: the n-th allocating call of this create reports hipErrorOutOfMemory instead of running
    int fail_at = g_fail_alloc_at;
    g_fail_alloc_at = 0;
    int alloc_no = 0;
#define SPC_ALLOC(call)                                                             \
    do {                                                                            \
        hipError_t e_ = ++alloc_no == fail_at ? hipErrorOutOfMemory : (call);       \
        if (e_ != hipSuccess) return bail(e_, #call);                               \
    } while (0)

    // The events only order streams of this device among themselves and the host never waits on
    // them, so they need no system-scope fence (measured: 2.3 us per layer-step less).
    const unsigned kOrderEventFlags = hipEventDisableTiming | hipEventDisableSystemFence;
    for (Layer& L : ctx->layers) {
        LayerView& v = L.view;
        v.rows = rows; v.G = G; v.bits = c.bits; v.group = c.group; v.R = c.residual;
        v.one_bit_plain = c.bits == 1 && c.one_bit_form == SPECACHE_1BIT_KIVI;
        v.max_seq = c.max_seq; v.topk = c.topk; v.bf16 = c.dtype == SPECACHE_BF16;
        v.kc_stride = (cap + kTileTokens - 1) / kTileTokens * k_tile_bytes(c.bits);
        v.vc_stride = cap / kBlockTokens * code_block_bytes(c.bits);
        v.km_stride = cap / c.group * kD;
        v.vm_stride = cap * (kD / c.group);
        SPC_ALLOC(hipMalloc((void**)&v.kc, rows * v.kc_stride));
        SPC_ALLOC(hipMalloc((void**)&v.vc, rows * v.vc_stride));
        SPC_ALLOC(hipMalloc((void**)&v.km, rows * v.km_stride * 4));
        SPC_ALLOC(hipMalloc((void**)&v.vm, rows * v.vm_stride * 4));
        SPC_ALLOC(hipMalloc((void**)&v.ring, (size_t)rows * c.residual * kRowBytes));
        SPC_ALLOC(hipHostMalloc(&L.host_alloc, (size_t)rows * cap * kRowBytes, hipHostMallocDefault));
        void* dev_view = nullptr;
        SPC_ALLOC(hipHostGetDevicePointer(&dev_view, L.host_alloc, 0));
        v.host = (uint16_t*)dev_view;
        for (int s = 0; s < 2; ++s) {
            SPC_ALLOC(hipMalloc((void**)&L.slot[s], (size_t)rows * c.topk * kRowBytes));
            SPC_ALLOC(hipMalloc((void**)&L.slot_idx[s], (size_t)rows * c.topk * 4));
            SPC_ALLOC(hipMemset(L.slot_idx[s], 0xFF, (size_t)rows * c.topk * 4));
            SPC_ALLOC(hipEventCreateWithFlags(&L.gathered[s], kOrderEventFlags));
            SPC_ALLOC(hipEventCreateWithFlags(&L.attended[s], kOrderEventFlags));
        }
        SPC_ALLOC(hipEventCreateWithFlags(&L.idx_ready, kOrderEventFlags));
    }
    ctx->async_select = c.async_select == SPECACHE_SELECT_STREAM_OWN;
    ctx->select_on_gather = c.async_select == SPECACHE_SELECT_STREAM_GATHER;
    if (ctx->select_on_gather) {
        for (Layer& L : ctx->layers) {
            SPC_ALLOC(hipMalloc((void**)&L.keys, (size_t)rows * cap * 4));
            SPC_ALLOC(hipEventCreateWithFlags(&L.selected, kOrderEventFlags));
        }
        const int parts = topk_parts((int)cap, c.topk);
        for (auto& ss : ctx->select_scratch) {
            ss.s.max_parts = parts;
            if (parts > 1) {
                SPC_ALLOC(hipMalloc((void**)&ss.s.cand_keys, (size_t)rows * parts * c.topk * 4));
                SPC_ALLOC(hipMalloc((void**)&ss.s.cand_idx, (size_t)rows * parts * c.topk * 4));
            }
        }
    }
    if (ctx->async_select) {
        SPC_ALLOC(hipStreamCreateWithFlags(&ctx->select_stream, hipStreamNonBlocking));
        SPC_ALLOC(hipEventCreateWithFlags(&ctx->scored, kOrderEventFlags));
    }
    ctx->logit_stride = cap;
    SPC_ALLOC(hipMalloc((void**)&ctx->logits, (size_t)rows * G * 2 * cap * 4));
    SPC_ALLOC(hipMalloc((void**)&ctx->keys, (size_t)rows * cap * 4));
    SPC_ALLOC(hipMalloc((void**)&ctx->lse, select_logprob_scratch_floats(rows, G, cap) * 4));
    int max_main = 0;
    for (int n = 1; n <= 2; ++n) {
        const int ch = attend_main_chunk_tokens(G * n);
        const int m = (int)((cap + ch - 1) / ch);
        max_main = m > max_main ? m : max_main;
    }
    const int ec = attend_extra_chunk_tokens();
    ctx->scratch.max_chunks = max_main + (c.topk + c.residual + 1 + ec - 1) / ec;
    SPC_ALLOC(hipMalloc((void**)&ctx->scratch.part_o, (size_t)rows * ctx->scratch.max_chunks * G * 2 * kD * 4));
    SPC_ALLOC(hipMalloc((void**)&ctx->scratch.part_ml, (size_t)rows * ctx->scratch.max_chunks * G * 2 * 2 * 4));
    ctx->topk_scratch.max_parts = topk_parts((int)cap, c.topk);
    if (ctx->topk_scratch.max_parts > 1) {
        const size_t n = (size_t)rows * ctx->topk_scratch.max_parts * c.topk;
        SPC_ALLOC(hipMalloc((void**)&ctx->topk_scratch.cand_keys, n * 4));
        SPC_ALLOC(hipMalloc((void**)&ctx->topk_scratch.cand_idx, n * 4));
    }
    SPC_ALLOC(hipDeviceSynchronize());
#undef SPC_ALLOC
    {
        // the static scratch array's address on this device, for specache_attend_static (a failure
        // here only surfaces when that entry point is called, with its own message)
        float* unused = nullptr;
        (void)static_scratch_of_current_device(nullptr, &unused);
    }
    *out = ctx;
    return SPECACHE_OK;
}

int specache_destroy(specache_ctx* ctx) {
    if (!ctx) return SPECACHE_OK;
    (void)hipDeviceSynchronize();
    free_all(ctx);
    delete ctx;
    return SPECACHE_OK;
}

const char* specache_last_error(const specache_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int specache_counts(const specache_ctx* ctx, int32_t layer, int32_t* n_tokens, int32_t* n_quantized) {
    if (!ctx || layer < 0 || layer >= ctx->cfg.n_layers) return SPECACHE_EINVAL;
    if (n_tokens) *n_tokens = ctx->layers[layer].N;
    if (n_quantized) *n_quantized = ctx->layers[layer].Nq;
    return SPECACHE_OK;
}

int specache_quantize_append(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, int32_t n_new,
                             void* stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (n_new < 0 || (n_new > 0 && (!k_new || !v_new))) return fail(ctx, SPECACHE_EINVAL, "null k_new/v_new or negative n_new");
    if (n_new == 0) return SPECACHE_OK;
    Layer& L = ctx->layers[layer];
    if ((long)L.N + n_new > ctx->cfg.max_seq) return fail(ctx, SPECACHE_ECAPACITY, "append exceeds max_seq");
    int32_t n_flush = 0;
    if (specache_plan_append(ctx->cfg.residual, ctx->cfg.group, L.N, L.Nq, n_new, &n_flush) != SPECACHE_OK)
        return fail(ctx, SPECACHE_ESTATE, "inconsistent token counts");
    const int Nq1 = L.Nq + n_flush * ctx->cfg.group, N1 = L.N + n_new;
    hipStream_t st = (hipStream_t)stream;
    // the flush reads residual tokens from the ring, so it precedes the ring update
    if (n_flush > 0) {
        TimedLaunch t(ctx, st, SPECACHE_K_FLUSH);
        SPC_HIP(ctx, launch_flush(L.view, k_new, v_new, n_new, L.N, L.Nq, n_flush, st));
    }
    {
        TimedLaunch t(ctx, st, SPECACHE_K_APPEND_COPY);
        SPC_HIP(ctx, launch_append_copy(L.view, k_new, v_new, n_new, L.N, Nq1 > L.N ? Nq1 : L.N, st));
    }
    L.N = N1;
    L.Nq = Nq1;
    return SPECACHE_OK;
}

int specache_score_topk(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, int32_t* topk_idx_out,
                        void* stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!q || !topk_idx_out) return fail(ctx, SPECACHE_EINVAL, "null q or topk_idx_out");
    if (n_rows != 1 && n_rows != 2) return fail(ctx, SPECACHE_EINVAL, "n_rows must be 1 or 2");
    if ((uintptr_t)q & 15) return fail(ctx, SPECACHE_EINVAL, "q must be 16-byte aligned");
    Layer& L = ctx->layers[layer];
    hipStream_t st = (hipStream_t)stream;
    hipStream_t tk = ctx->async_select ? ctx->select_stream : st;   // where ArgTopK runs
    // a gather still reading this index buffer must finish before it is overwritten
    if (L.last_gather_idx == topk_idx_out && L.last_gather_slot >= 0)
        SPC_HIP(ctx, hipStreamWaitEvent(tk, L.gathered[L.last_gather_slot], 0));
    // the key array is shared by all layers: the previous selection, running aside, must have read it
    if (ctx->async_select && ctx->last_select) SPC_HIP(ctx, hipStreamWaitEvent(st, ctx->last_select, 0));
    if (int rc = score_phase(ctx, L, q, n_rows, ctx->keys, st)) return rc;
    if (ctx->async_select) {
        SPC_HIP(ctx, hipEventRecord(ctx->scored, st));
        SPC_HIP(ctx, hipStreamWaitEvent(tk, ctx->scored, 0));
    }
    {
        TimedLaunch t(ctx, tk, SPECACHE_K_TOPK, /*kernel_events=*/true);
        SPC_HIP(ctx, launch_topk(L.view.rows, L.Nq, ctx->cfg.topk, ctx->keys, ctx->logit_stride, topk_idx_out,
                                 ctx->topk_scratch, tk));
    }
    SPC_HIP(ctx, hipEventRecord(L.idx_ready, tk));
    ctx->last_select = L.idx_ready;
    L.idx_ready_recorded = true;
    L.idx_ready_stream = tk;
    L.select_origin_stream = st;
    L.idx_ready_seq = ++ctx->seq;
    ctx->scored_layer = layer;
    ctx->scored_rows = n_rows;
    ctx->scored_N = L.N;
    ctx->scored_Nq = L.Nq;
    ctx->logits_kept = true;
    return SPECACHE_OK;
}

// The layer's key array is about to be rewritten on st: the selections that read it come first.
static int wait_for_keys_readers(specache_ctx* ctx, Layer& L, hipStream_t st) {
    // the layer's previous selection read L.keys on the stream of the gather that followed it
    if (L.keys_reader_slot >= 0) {
        const int sl = L.keys_reader_slot;
        if (L.gather_stream[sl] != st && !(L.gathered_waited_set[sl] && L.gathered_waited[sl] == st)) {
            SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[sl], 0));
            L.gathered_waited[sl] = st;
            L.gathered_waited_set[sl] = true;
        }
        L.keys_reader_slot = -1;
    }
    if (L.selected_pending) {
        if (L.selected_stream != st) SPC_HIP(ctx, hipStreamWaitEvent(st, L.selected, 0));
        L.selected_pending = false;
    }
    return SPECACHE_OK;
}

// "scored": what the selection waits for, and what orders a gather after the attends enqueued so far
static int record_scored(specache_ctx* ctx, Layer& L, int32_t layer, int32_t n_rows, hipStream_t st, bool carried = false) {
    if (!carried) SPC_HIP(ctx, hipEventRecord(L.idx_ready, st));
    L.idx_ready_recorded = true;
    L.idx_ready_stream = st;
    L.select_origin_stream = st;
    L.idx_ready_seq = ++ctx->seq;
    L.keys_valid = true;
    L.keys_Nq = L.Nq;
    ctx->scored_layer = layer;
    ctx->scored_rows = n_rows;
    ctx->scored_N = L.N;
    ctx->scored_Nq = L.Nq;
    return SPECACHE_OK;
}

// specache_score, optionally with the copy of one new token carried by the scoring launch
static int score_impl(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, void* stream, const void* k_new,
                      const void* v_new) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!ctx->select_on_gather) return fail(ctx, SPECACHE_ESTATE, "specache_score needs async_select = SPECACHE_SELECT_STREAM_GATHER");
    if (!q) return fail(ctx, SPECACHE_EINVAL, "null q");
    if (n_rows != 1 && n_rows != 2) return fail(ctx, SPECACHE_EINVAL, "n_rows must be 1 or 2");
    if ((uintptr_t)q & 15) return fail(ctx, SPECACHE_EINVAL, "q must be 16-byte aligned");
    Layer& L = ctx->layers[layer];
    hipStream_t st = (hipStream_t)stream;
    if (int rc = wait_for_keys_readers(ctx, L, st)) return rc;
    bool carried = false;
    if (k_new) {
        // the scoring launch appends token N: one more workgroup per row copies the pair
        LayerView fused = L.view;
        fused.tail_k = (const uint16_t*)k_new;
        fused.tail_v = (const uint16_t*)v_new;
        fused.tail_N0 = L.N;
        if (int rc = score_phase(ctx, L, q, n_rows, L.keys, st, &fused, L.idx_ready, &carried)) return rc;
        L.N += 1;   // only once the launch that copies the token is enqueued
    } else if (int rc = score_phase(ctx, L, q, n_rows, L.keys, st, nullptr, L.idx_ready, &carried)) {
        return rc;
    }
    ctx->logits_kept = true;
    return record_scored(ctx, L, layer, n_rows, st, carried);
}

int specache_score(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, void* stream) {
    return score_impl(ctx, layer, q, n_rows, stream, nullptr, nullptr);
}

int specache_append_score(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                          int32_t n_rows, void* stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!ctx->select_on_gather)
        return fail(ctx, SPECACHE_ESTATE, "specache_append_score needs async_select = SPECACHE_SELECT_STREAM_GATHER");
    if (!k_new || !v_new) return fail(ctx, SPECACHE_EINVAL, "null k_new or v_new");
    Layer& L = ctx->layers[layer];
    if ((long)L.N + 1 > ctx->cfg.max_seq) return fail(ctx, SPECACHE_ECAPACITY, "append exceeds max_seq");
    int32_t n_flush = 0;
    if (specache_plan_append(ctx->cfg.residual, ctx->cfg.group, L.N, L.Nq, 1, &n_flush) != SPECACHE_OK)
        return fail(ctx, SPECACHE_ESTATE, "inconsistent token counts");
    // a group leaves the residual with this token, or nothing is quantised yet (no scoring launch): two steps
    // (the 4-bit scoring kernel carries no append)
    if (n_flush > 0 || L.Nq == 0 || ctx->cfg.bits == 4) {
        if (int rc = specache_quantize_append(ctx, layer, k_new, v_new, 1, stream)) return rc;
        return score_impl(ctx, layer, q, n_rows, stream, nullptr, nullptr);
    }
    return score_impl(ctx, layer, q, n_rows, stream, k_new, v_new);
}

int specache_select_gather(specache_ctx* ctx, int32_t layer, int32_t* topk_idx_out, int32_t slot, void* side_stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!ctx->select_on_gather)
        return fail(ctx, SPECACHE_ESTATE, "specache_select_gather needs async_select = SPECACHE_SELECT_STREAM_GATHER");
    if (!topk_idx_out) return fail(ctx, SPECACHE_EINVAL, "null topk_idx_out");
    if (slot < -1 || slot > 1) return fail(ctx, SPECACHE_EINVAL, "slot must be -1, 0 or 1");
    Layer& L = ctx->layers[layer];
    if (!L.keys_valid) return fail(ctx, SPECACHE_ESTATE, "specache_select_gather must follow specache_score of the layer");
    hipStream_t st = (hipStream_t)side_stream;
    if (st != L.idx_ready_stream) SPC_HIP(ctx, hipStreamWaitEvent(st, L.idx_ready, 0));
    // a gather on another stream that still reads this index buffer must finish before it is overwritten
    if (L.last_gather_idx == topk_idx_out && L.last_gather_slot >= 0 && L.gather_stream[L.last_gather_slot] != st)
        SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[L.last_gather_slot], 0));
    if (slot >= 0)
        if (int rc = order_gather_after_attend(ctx, L, slot, st)) return rc;
    // an earlier selection of the same keys on another stream: the next scoring pass waits for the
    // latest selection only, so this one goes behind it
    if (L.keys_reader_slot >= 0 && L.gather_stream[L.keys_reader_slot] != st)
        SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[L.keys_reader_slot], 0));
    if (L.selected_pending && L.selected_stream != st) SPC_HIP(ctx, hipStreamWaitEvent(st, L.selected, 0));
    specache_ctx::SelectScratch* ss = nullptr;
    if (ctx->select_scratch[0].s.max_parts > 1) {
        // the candidate arrays last used on this stream, else the set whose turn it is (after its last user)
        for (auto& c : ctx->select_scratch)
            if (c.used && c.stream == st) ss = &c;
        if (!ss) {
            ss = &ctx->select_scratch[ctx->select_scratch_next];
            ctx->select_scratch_next ^= 1;
            if (ss->used) SPC_HIP(ctx, hipStreamWaitEvent(st, ss->done, 0));
        }
    }
    {
        TimedLaunch t(ctx, st, SPECACHE_K_TOPK, /*kernel_events=*/true);
        SPC_HIP(ctx, launch_topk(L.view.rows, L.keys_Nq, ctx->cfg.topk, L.keys, ctx->logit_stride, topk_idx_out,
                                 ss ? ss->s : ctx->select_scratch[0].s, st));
    }
    if (slot >= 0) {
        if (int rc = gather_phase(ctx, L, L.keys_Nq, topk_idx_out, slot, st)) return rc;
        L.keys_reader_slot = slot;
    } else {
        // selection only: an event of its own tells the layer's next scoring pass that the keys were read
        SPC_HIP(ctx, hipEventRecord(L.selected, st));
        L.selected_pending = true;
        L.selected_stream = st;
    }
    if (ss) {
        ss->used = true;
        ss->stream = st;
        ss->done = slot >= 0 ? L.gathered[slot] : L.selected;   // recorded behind the selection on this stream
    }
    return SPECACHE_OK;
}

int specache_gather(specache_ctx* ctx, int32_t layer, const int32_t* idx, int32_t slot, void* side_stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!idx) return fail(ctx, SPECACHE_EINVAL, "null idx");
    if (slot != 0 && slot != 1) return fail(ctx, SPECACHE_EINVAL, "slot must be 0 or 1");
    Layer& L = ctx->layers[layer];
    hipStream_t st = (hipStream_t)side_stream;
    if (L.idx_ready_recorded && st != L.idx_ready_stream) SPC_HIP(ctx, hipStreamWaitEvent(st, L.idx_ready, 0));
    if (int rc = order_gather_after_attend(ctx, L, slot, st)) return rc;
    if (int rc = gather_phase(ctx, L, L.Nq, idx, slot, st)) return rc;
    return SPECACHE_OK;
}

// the attention kernels that read `slot` are enqueued on st: remember it for the slot's next gather
static int record_attended(specache_ctx* ctx, Layer& L, int slot, hipStream_t st) {
    if (slot >= 0) {
        L.attend_stream[slot] = st;
        L.attend_seq[slot] = ++ctx->seq;
        L.attended_recorded[slot] = false;
        if (!(L.idx_ready_recorded && st == L.select_origin_stream)) {
            SPC_HIP(ctx, hipEventRecord(L.attended[slot], st));
            L.attended_recorded[slot] = true;
        }
    }
    return SPECACHE_OK;
}

// specache_attend with the partial results in `scratch`: the context's own, or the static array
static int attend_impl(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                       const void* v_spec, int32_t slot, float* out, void* stream, const AttendScratch* static_scratch) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!q || !out) return fail(ctx, SPECACHE_EINVAL, "null q or out");
    if (n_rows != 1 && n_rows != 2) return fail(ctx, SPECACHE_EINVAL, "n_rows must be 1 or 2");
    if ((k_spec == nullptr) != (v_spec == nullptr)) return fail(ctx, SPECACHE_EINVAL, "k_spec and v_spec must both be given or both be null");
    if (slot < -1 || slot > 1) return fail(ctx, SPECACHE_EINVAL, "slot must be -1, 0 or 1");
    Layer& L = ctx->layers[layer];
    if (ctx->scored_layer != layer || ctx->scored_rows != n_rows || ctx->scored_N != L.N || ctx->scored_Nq != L.Nq)
        return fail(ctx, SPECACHE_ESTATE, "attend must follow score_topk of the same layer, n_rows and cache state");
    if (!ctx->logits_kept) return fail(ctx, SPECACHE_ESTATE, "the last scoring pass of this layer was specache_score_attend, which keeps no logits");
    if (slot >= 0 && !L.slot_filled[slot]) return fail(ctx, SPECACHE_ESTATE, "slot was never gathered");
    if (L.N == 0 && !k_spec) return fail(ctx, SPECACHE_ESTATE, "no attention candidate");
    AttendScratch scratch = ctx->scratch;
    if (static_scratch) {
        // partial outputs [rows][chunks][NR][128] floats, then the (max, sum) pairs [rows][chunks][NR][2]
        const int NR = L.view.G * n_rows;
        const int chunks = attend_chunks(NR, L.Nq, (slot >= 0 ? ctx->cfg.topk : 0) + (L.N - L.Nq) + (k_spec ? 1 : 0));
        const size_t o_floats = (size_t)L.view.rows * chunks * NR * kD, ml_floats = (size_t)L.view.rows * chunks * NR * 2;
        if ((o_floats + ml_floats) * sizeof(float) > kStaticScratchBytes)
            return fail(ctx, SPECACHE_ECAPACITY, "specache_attend_static: the partial results of this call (rows x chunks x query rows "
                                                 "x 130 floats) exceed the 16 MiB static scratch array; use specache_attend");
        scratch.part_o = static_scratch->part_o;
        scratch.part_ml = static_scratch->part_o + o_floats;
        scratch.max_chunks = chunks;
    }
    hipStream_t st = (hipStream_t)stream;
    if (slot >= 0 && L.gather_stream[slot] != st && !(L.gathered_waited_set[slot] && L.gathered_waited[slot] == st))
        SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[slot], 0));
    for (int phase : {kAttendPartial, kAttendCombine}) {
        TimedLaunch t(ctx, st, phase == kAttendPartial ? SPECACHE_K_ATTEND : SPECACHE_K_ATTEND_COMBINE, /*kernel_events=*/true);
        SPC_HIP(ctx, launch_attend(L.view, q, n_rows, L.N, L.Nq, ctx->sm_scale, ctx->logits, ctx->logit_stride,
                                   slot >= 0 ? L.slot[slot] : nullptr, slot >= 0 ? L.slot_idx[slot] : nullptr, k_spec,
                                   v_spec, scratch, out, phase, st));
    }
    return record_attended(ctx, L, slot, st);
}

int specache_attend(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                    const void* v_spec, int32_t slot, float* out, void* stream) {
    return attend_impl(ctx, layer, q, n_rows, k_spec, v_spec, slot, out, stream, nullptr);
}

// specache_score_attend, optionally with the append of one new token in front (carried by the same launch when
// that launch exists and no group leaves the residual with the token)
static int score_attend_impl(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                             int32_t n_rows, const void* k_spec, const void* v_spec, int32_t slot, float* out, void* stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (!ctx->select_on_gather)
        return fail(ctx, SPECACHE_ESTATE, "specache_score_attend needs async_select = SPECACHE_SELECT_STREAM_GATHER");
    if ((k_new == nullptr) != (v_new == nullptr)) return fail(ctx, SPECACHE_EINVAL, "k_new and v_new must both be given or both be null");
    Layer& L = ctx->layers[layer];
    int32_t n_flush = 0;
    if (k_new) {
        if ((long)L.N + 1 > ctx->cfg.max_seq) return fail(ctx, SPECACHE_ECAPACITY, "append exceeds max_seq");
        if (specache_plan_append(ctx->cfg.residual, ctx->cfg.group, L.N, L.Nq, 1, &n_flush) != SPECACHE_OK)
            return fail(ctx, SPECACHE_ESTATE, "inconsistent token counts");
    }
    const bool one_pass = L.view.G == 1 && n_rows == 2 && attend_uses_int8_matrix_cores(L.view, n_rows) && L.Nq > 0 &&
                          ctx->cfg.select_cache == SPECACHE_SELECT_LOWBIT && q && out && !((uintptr_t)q & 15) &&
                          !(kernel_choice() & (kChoiceScoreValu | kChoiceAttendValu));
    const bool carry = k_new && one_pass && n_flush == 0;
    if (k_new && !carry)
        if (int rc = specache_quantize_append(ctx, layer, k_new, v_new, 1, stream)) return rc;
    if (!one_pass) {
        // other shapes and options: the two passes one after the other, same results
        if (int rc = score_impl(ctx, layer, q, n_rows, stream, nullptr, nullptr)) return rc;
        return attend_impl(ctx, layer, q, n_rows, k_spec, v_spec, slot, out, stream, nullptr);
    }
    if ((k_spec == nullptr) != (v_spec == nullptr)) return fail(ctx, SPECACHE_EINVAL, "k_spec and v_spec must both be given or both be null");
    if (slot < -1 || slot > 1) return fail(ctx, SPECACHE_EINVAL, "slot must be -1, 0 or 1");
    if (slot >= 0 && !L.slot_filled[slot]) return fail(ctx, SPECACHE_ESTATE, "slot was never gathered");
    hipStream_t st = (hipStream_t)stream;
    if (int rc = wait_for_keys_readers(ctx, L, st)) return rc;
    if (slot >= 0 && L.gather_stream[slot] != st && !(L.gathered_waited_set[slot] && L.gathered_waited[slot] == st))
        SPC_HIP(ctx, hipStreamWaitEvent(st, L.gathered[slot], 0));
    const bool keep = (kernel_choice() & kChoiceKeepLogits) != 0;
    LayerView view = L.view;
    if (carry) {
        view.tail_k = (const uint16_t*)k_new;
        view.tail_v = (const uint16_t*)v_new;
        view.tail_N0 = L.N;
    }
    const int N1 = L.N + (carry ? 1 : 0);
    bool scored_carried = false;
    {
        TimedLaunch t(ctx, st, SPECACHE_K_SCORE_ATTEND, /*kernel_events=*/true);
        CarriedEvent scored(ctx, L.idx_ready);
        SPC_HIP(ctx, launch_attend_i8_partial(view, q, N1, L.Nq, ctx->sm_scale, nullptr, ctx->logit_stride,
                                              slot >= 0 ? L.slot[slot] : nullptr, slot >= 0 ? L.slot_idx[slot] : nullptr, k_spec,
                                              v_spec, ctx->scratch, L.keys, ctx->logit_stride, keep ? ctx->logits : nullptr, st));
        scored_carried = scored.landed();
    }
    L.N = N1;   // only once the launch that copies the token is enqueued
    ctx->logits_kept = keep;
    // the keys are complete here: the selection on the side stream can start while the chunks are merged
    if (int rc = record_scored(ctx, L, layer, n_rows, st, scored_carried)) return rc;
    {
        TimedLaunch t(ctx, st, SPECACHE_K_ATTEND_COMBINE, /*kernel_events=*/true);
        SPC_HIP(ctx, launch_attend(L.view, q, n_rows, L.N, L.Nq, ctx->sm_scale, ctx->logits, ctx->logit_stride,
                                   slot >= 0 ? L.slot[slot] : nullptr, slot >= 0 ? L.slot_idx[slot] : nullptr, k_spec, v_spec,
                                   ctx->scratch, out, kAttendCombine, st));
    }
    return record_attended(ctx, L, slot, st);
}

int specache_score_attend(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                          const void* v_spec, int32_t slot, float* out, void* stream) {
    return score_attend_impl(ctx, layer, nullptr, nullptr, q, n_rows, k_spec, v_spec, slot, out, stream);
}

int specache_append_score_attend(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                                 int32_t n_rows, const void* k_spec, const void* v_spec, int32_t slot, float* out,
                                 void* stream) {
    if (ctx && (!k_new || !v_new)) return fail(ctx, SPECACHE_EINVAL, "null k_new or v_new");
    return score_attend_impl(ctx, layer, k_new, v_new, q, n_rows, k_spec, v_spec, slot, out, stream);
}

int specache_decode_step(specache_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, const void* q,
                         const void* k_spec, const void* v_spec, int32_t read_slot, float* out, void* stream,
                         int32_t* topk_idx_out, int32_t fill_slot, void* side_stream) {
    if (int rc = specache_append_score_attend(ctx, layer, k_new, v_new, q, 2, k_spec, v_spec, read_slot, out, stream)) return rc;
    return specache_select_gather(ctx, layer, topk_idx_out, fill_slot, side_stream);
}

int specache_attend_static(specache_ctx* ctx, int32_t layer, const void* q, int32_t n_rows, const void* k_spec,
                           const void* v_spec, int32_t slot, float* out, void* stream) {
    if (!ctx) return SPECACHE_EINVAL;
    float* base = nullptr;
    if (int rc = static_scratch_of_current_device(ctx, &base)) return rc;
    const AttendScratch st{base, nullptr, 0};
    return attend_impl(ctx, layer, q, n_rows, k_spec, v_spec, slot, out, stream, &st);
}

int specache_debug_fail_alloc(int32_t nth) {
    if (nth < 0) return SPECACHE_EINVAL;
    g_fail_alloc_at = nth;
    return SPECACHE_OK;
}

int specache_debug_kernel_choice(int32_t flags) {
    if (flags < 0 || flags > (SPECACHE_SCORE_ON_VECTOR_ALU | SPECACHE_ATTEND_ON_VECTOR_ALU | SPECACHE_KEEP_ONE_PASS_LOGITS))
        return SPECACHE_EINVAL;
    kernel_choice() = (flags & SPECACHE_SCORE_ON_VECTOR_ALU ? kChoiceScoreValu : 0) |
                      (flags & SPECACHE_ATTEND_ON_VECTOR_ALU ? kChoiceAttendValu : 0) |
                      (flags & SPECACHE_KEEP_ONE_PASS_LOGITS ? kChoiceKeepLogits : 0);
    return SPECACHE_OK;
}

int specache_debug_poison_slot(specache_ctx* ctx, int32_t layer, int32_t slot, void* stream) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    if (slot != 0 && slot != 1) return fail(ctx, SPECACHE_EINVAL, "slot must be 0 or 1");
    Layer& L = ctx->layers[layer];
    // every 16-bit word becomes 0xFFFF, a NaN in binary16 and in bfloat16
    SPC_HIP(ctx, hipMemsetAsync(L.slot[slot], 0xFF, (size_t)L.view.rows * ctx->cfg.topk * kRowBytes, (hipStream_t)stream));
    return SPECACHE_OK;
}

int specache_export_quantized(specache_ctx* ctx, int32_t layer, uint8_t* k_codes, uint16_t* k_minmax,
                              float* k_scale_zero, uint8_t* v_codes, uint16_t* v_minmax, float* v_scale_zero) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    Layer& L = ctx->layers[layer];
    SPC_HIP(ctx, hipDeviceSynchronize());
    const size_t rows = L.view.rows, Nq = L.Nq, g = ctx->cfg.group;
    if (Nq == 0) return SPECACHE_OK;
    const size_t n_codes = rows * Nq * kD, n_kg = rows * (Nq / g) * kD, n_vg = rows * Nq * (kD / g);
    struct Buf { void* host; size_t bytes; void* dev; };
    Buf bufs[6] = {{k_codes, n_codes, nullptr},        {k_minmax, n_kg * 4, nullptr}, {k_scale_zero, n_kg * 8, nullptr},
                   {v_codes, n_codes, nullptr},        {v_minmax, n_vg * 4, nullptr}, {v_scale_zero, n_vg * 8, nullptr}};
    int rc = SPECACHE_OK;
    for (Buf& b : bufs)
        if (b.host && rc == SPECACHE_OK) {
            hipError_t e = hipMalloc(&b.dev, b.bytes);
            if (e != hipSuccess) rc = fail_hip(ctx, e, "hipMalloc(export)");
        }
    if (rc == SPECACHE_OK) {
        hipError_t e = launch_export(L.view, L.Nq, (uint8_t*)bufs[0].dev, (uint16_t*)bufs[1].dev, (float*)bufs[2].dev,
                                     (uint8_t*)bufs[3].dev, (uint16_t*)bufs[4].dev, (float*)bufs[5].dev, nullptr);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        for (Buf& b : bufs)
            if (b.dev && e == hipSuccess) e = hipMemcpy(b.host, b.dev, b.bytes, hipMemcpyDeviceToHost);
        if (e != hipSuccess) rc = fail_hip(ctx, e, "export");
    }
    for (Buf& b : bufs) (void)hipFree(b.dev);
    return rc;
}

int specache_export_rows(specache_ctx* ctx, int32_t layer, int32_t first, int32_t count, uint16_t* out) {
    if (int rc = check_ctx_layer(ctx, layer)) return rc;
    Layer& L = ctx->layers[layer];
    if (!out || first < 0 || count < 0 || first + count > L.N) return fail(ctx, SPECACHE_EINVAL, "bad row range or null output");
    SPC_HIP(ctx, hipDeviceSynchronize());
    const uint8_t* src = (const uint8_t*)L.host_alloc;
    for (int r = 0; r < L.view.rows; ++r)
        std::memcpy((uint8_t*)out + (size_t)r * count * kRowBytes,
                    src + ((size_t)r * ctx->cfg.max_seq + first) * kRowBytes, (size_t)count * kRowBytes);
    return SPECACHE_OK;
}

int specache_timing(specache_ctx* ctx, int32_t enable, double* total_us, int64_t* launches) {
    if (!ctx) return SPECACHE_EINVAL;
    SPC_HIP(ctx, hipDeviceSynchronize());
    if (total_us) for (int k = 0; k < SPECACHE_K_COUNT; ++k) total_us[k] = 0.0;
    if (launches) for (int k = 0; k < SPECACHE_K_COUNT; ++k) launches[k] = 0;
    for (auto& sp : ctx->spans) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) {
            if (total_us) total_us[sp.kind] += 1e3 * (double)ms;
            if (launches) launches[sp.kind] += 1;
        }
        ctx->ev_pool.push_back(sp.a);
        ctx->ev_pool.push_back(sp.b);
    }
    ctx->spans.clear();
    ctx->timing = enable != 0;
    return SPECACHE_OK;
}

int specache_debug_logits(specache_ctx* ctx, float* out) {
    if (!ctx || !out) return SPECACHE_EINVAL;
    if (ctx->scored_layer < 0) return fail(ctx, SPECACHE_ESTATE, "nothing scored yet");
    if (!ctx->logits_kept) return fail(ctx, SPECACHE_ESTATE, "specache_score_attend kept no logits (see specache_debug_kernel_choice)");
    SPC_HIP(ctx, hipDeviceSynchronize());
    const size_t n = (size_t)ctx->layers[ctx->scored_layer].view.rows * ctx->layers[ctx->scored_layer].view.G * ctx->scored_rows;
    const size_t Nq = ctx->scored_Nq;
    if (Nq == 0) return SPECACHE_OK;
    SPC_HIP(ctx, hipMemcpy2D(out, Nq * 4, ctx->logits, ctx->logit_stride * 4, Nq * 4, n, hipMemcpyDeviceToHost));
    return SPECACHE_OK;
}

}  // extern "C"
