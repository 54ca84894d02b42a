// Sanitizer driver of the library's host-only code paths (run by tests/test_sanitize.py on the CPU):
// the append planner and the argument checks that return before any GPU work.  Built with the host
// pass of csrc/specache.hip and csrc/measure.hip under -fsanitize=address,undefined.  No kernel runs.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/specache.h"

#define REQUIRE(cond)                                                                          \
    do {                                                                                       \
        if (!(cond)) {                                                                         \
            std::fprintf(stderr, "host_sanitize_driver: %s failed at line %d\n", #cond, __LINE__); \
            std::exit(1);                                                                      \
        }                                                                                      \
    } while (0)

int main() {
    // planner: against the residual policy stepped one token at a time
    for (int g : {32, 64, 128})
        for (int R = g; R <= 256; R += g)
            for (int start = 0; start < R; start += 7)
                for (int n_new : {0, 1, 2, g - 1, g, R, 3 * R + 5, 1000}) {
                    int N = start, Nq = 0, flushed = 0;
                    for (int t = 0; t < n_new; ++t) {
                        N += 1;
                        if (N - Nq == R) { Nq += g; flushed += 1; }
                    }
                    int32_t got = -1;
                    REQUIRE(specache_plan_append(R, g, start, 0, n_new, &got) == SPECACHE_OK);
                    REQUIRE(got == flushed);
                }
    int32_t out = 0;
    REQUIRE(specache_plan_append(64, 32, 10, 0, 1, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_plan_append(48, 32, 10, 0, 1, &out) == SPECACHE_EINVAL);
    REQUIRE(specache_plan_append(64, 32, 5, 32, 1, &out) == SPECACHE_EINVAL);
    REQUIRE(specache_plan_append(64, 32, 100, 0, 1, &out) == SPECACHE_EINVAL);
    REQUIRE(specache_plan_append(64, 32, 10, 0, -1, &out) == SPECACHE_EINVAL);
    REQUIRE(specache_plan_append(64, 0, 10, 0, 1, &out) == SPECACHE_EINVAL);

    // configurations rejected before anything is allocated
    specache_config base;
    std::memset(&base, 0, sizeof base);
    base.n_layers = 1; base.batch = 1; base.n_q_heads = 2; base.n_kv_heads = 2; base.head_dim = 128; base.bits = 2;
    base.group = 32; base.residual = 64; base.max_seq = 256; base.topk = 16; base.dtype = SPECACHE_FP16;
    specache_ctx* ctx = reinterpret_cast<specache_ctx*>(0x1);
    auto rejected = [&](specache_config c) {
        ctx = reinterpret_cast<specache_ctx*>(0x1);
        const int rc = specache_create(&c, &ctx);
        return rc == SPECACHE_EINVAL && ctx == nullptr && std::strlen(specache_last_error(nullptr)) > 0;
    };
    { specache_config c = base; c.bits = 3; REQUIRE(rejected(c)); }
    { specache_config c = base; c.bits = 8; REQUIRE(rejected(c)); }
    { specache_config c = base; c.group = 48; REQUIRE(rejected(c)); }
    { specache_config c = base; c.residual = 48; REQUIRE(rejected(c)); }
    { specache_config c = base; c.residual = 512; REQUIRE(rejected(c)); }
    { specache_config c = base; c.max_seq = 100; REQUIRE(rejected(c)); }
    { specache_config c = base; c.topk = 0; REQUIRE(rejected(c)); }
    { specache_config c = base; c.topk = 5000; REQUIRE(rejected(c)); }
    { specache_config c = base; c.head_dim = 64; REQUIRE(rejected(c)); }
    { specache_config c = base; c.n_q_heads = 3; REQUIRE(rejected(c)); }
    { specache_config c = base; c.n_q_heads = 32; c.n_kv_heads = 2; REQUIRE(rejected(c)); }
    { specache_config c = base; c.n_layers = 0; REQUIRE(rejected(c)); }
    { specache_config c = base; c.dtype = 2; REQUIRE(rejected(c)); }
    { specache_config c = base; c.one_bit_form = 2; REQUIRE(rejected(c)); }
    { specache_config c = base; c.select_form = 2; REQUIRE(rejected(c)); }
    { specache_config c = base; c.select_cache = -1; REQUIRE(rejected(c)); }
    { specache_config c = base; c.async_select = 3; REQUIRE(rejected(c)); }
    { specache_config c = base; c.n_q_heads = 8; c.n_kv_heads = 1; c.max_seq = 64 * 20000; REQUIRE(rejected(c)); }
    REQUIRE(specache_create(nullptr, &ctx) == SPECACHE_EINVAL);
    REQUIRE(specache_create(&base, nullptr) == SPECACHE_EINVAL);

    // calls without a context
    REQUIRE(specache_destroy(nullptr) == SPECACHE_OK);
    REQUIRE(specache_counts(nullptr, 0, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_quantize_append(nullptr, 0, nullptr, nullptr, 1, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_score_topk(nullptr, 0, nullptr, 2, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_score(nullptr, 0, nullptr, 2, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_append_score(nullptr, 0, nullptr, nullptr, nullptr, 2, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_select_gather(nullptr, 0, nullptr, 0, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_decode_step(nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, nullptr, 0, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_debug_fail_alloc(-1) == SPECACHE_EINVAL);
    REQUIRE(specache_debug_fail_alloc(0) == SPECACHE_OK);
    REQUIRE(specache_gather(nullptr, 0, nullptr, 0, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_attend(nullptr, 0, nullptr, 2, nullptr, nullptr, -1, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_score_attend(nullptr, 0, nullptr, 2, nullptr, nullptr, -1, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_append_score_attend(nullptr, 0, nullptr, nullptr, nullptr, 2, nullptr, nullptr, -1, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_attend_static(nullptr, 0, nullptr, 2, nullptr, nullptr, -1, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_debug_poison_slot(nullptr, 0, 0, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_export_quantized(nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_export_rows(nullptr, 0, 0, 0, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_debug_logits(nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_timing(nullptr, 0, nullptr, nullptr) == SPECACHE_EINVAL);
    double x = 0.0;
    REQUIRE(specache_measure_hbm_read(1 << 30, 10, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_measure_hbm_read(100, 10, &x) == SPECACHE_EINVAL);
    REQUIRE(specache_measure_hbm_read(1 << 30, 0, &x) == SPECACHE_EINVAL);
    REQUIRE(specache_measure_link(1 << 28, 5, nullptr, nullptr) == SPECACHE_EINVAL);
    REQUIRE(specache_measure_link(10, 5, &x, &x) == SPECACHE_EINVAL);
    REQUIRE(std::strlen(specache_last_error(nullptr)) > 0);
    std::printf("host_sanitize_driver ok\n");
    return 0;
}
