// Sanitizer driver of the CPU oracle (test infrastructure): built together with specache_oracle.cpp
// under -fsanitize=address,undefined and run by tests/test_sanitize.py.  It walks every exported
// function over the shapes the pin suite's heaviest cases use (streamed appends across many flushes,
// all bit widths, group sizes and both 1-bit forms, scores in every form, ArgTopK with ties and
// k > n, attention with prefetched sets and the transient pair) and over the invalid-argument paths.
// It checks only what needs no second implementation (return codes, counts, ranges): the values are
// the pin suite's business, memory and arithmetic errors are the sanitizers'.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
float orc_widen(uint16_t bits, int dtype);
int orc_quantize_group_form(const float* x, int g, int bits, int one_bit_form, float* mn, float* mx, float* s, float* z,
                            uint8_t* codes);
int orc_derive_scale_zero_form(float mn, float mx, int bits, int one_bit_form, float* s, float* z);
int orc_pack_group(const uint8_t* codes, int g, int bits, uint8_t* packed);
int orc_unpack_group(const uint8_t* packed, int g, int bits, uint8_t* codes);
void* orc_cache_create_form(int D, int bits, int g, int R, int dtype, int one_bit_form);
void orc_cache_destroy(void* h);
int orc_cache_append(void* h, const uint16_t* k_rows, const uint16_t* v_rows, int n);
int orc_cache_counts(void* h, int* N, int* Nq);
int orc_cache_export(void* h, uint8_t* k_codes, float* k_mnmx, float* k_sz, uint8_t* v_codes, float* v_mnmx, float* v_sz);
int orc_cache_dequant(void* h, double* k_deq, double* v_deq);
int orc_cache_history(void* h, double* k, double* v);
int orc_scores_mixed(void* hc, const uint16_t* q, int G, int rows, double sm_scale, int select_form, const int32_t* P,
                     int nP, double* logits, double* sigma);
int orc_topk(const double* sigma, int n, int k, int32_t* idx_out);
int orc_attend(void* hc, const uint16_t* q, int G, int rows, double sm_scale, const int32_t* P, int nP,
               const uint16_t* k_spec, const uint16_t* v_spec, double* out);
int orc_full_attention(void* hc, const uint16_t* q, int G, int rows, double sm_scale, const uint16_t* k_spec,
                       const uint16_t* v_spec, double* out, double* weights);
double orc_hit_rate(const double* weights, int n, const int32_t* idx, int n_idx);
}

static uint64_t g_state = 0x243F6A8885A308D3ull;
static uint32_t next_u32() {
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(g_state >> 33);
}
// a finite 16-bit pattern of moderate magnitude (exponent field kept in the middle of the range)
static uint16_t next_pattern(int dtype) {
    const uint32_t r = next_u32();
    if (dtype == 0) return (uint16_t)(((r & 1u) << 15) | ((10u + (r >> 1) % 8u) << 10) | ((r >> 8) & 0x3FFu));
    return (uint16_t)(((r & 1u) << 15) | ((122u + (r >> 1) % 8u) << 7) | ((r >> 8) & 0x7Fu));
}

#define REQUIRE(cond)                                                         \
    do {                                                                      \
        if (!(cond)) {                                                        \
            std::fprintf(stderr, "sanitize_driver: %s failed at line %d\n", #cond, __LINE__); \
            std::exit(1);                                                     \
        }                                                                     \
    } while (0)

int main() {
    // widening of every pattern, both types
    double acc = 0.0;
    for (int dtype = 0; dtype < 2; ++dtype)
        for (uint32_t b = 0; b < 65536; ++b) {
            const float f = orc_widen((uint16_t)b, dtype);
            if (f == f && f < 1e30f && f > -1e30f) acc += f;
        }
    // groups: random, constant, two-valued
    for (int bits : {1, 2, 4, 8})
        for (int g : {32, 64, 128})
            for (int form = 0; form < 2; ++form)
                for (int kind = 0; kind < 3; ++kind) {
                    std::vector<float> x(g);
                    for (int i = 0; i < g; ++i)
                        x[i] = kind == 0 ? orc_widen(next_pattern(0), 0) : kind == 1 ? 1.5f : (i % 2 ? -2.0f : 3.0f);
                    std::vector<uint8_t> codes(g), packed((size_t)g * bits / 8), back(g);
                    float mn, mx, s, z;
                    REQUIRE(orc_quantize_group_form(x.data(), g, bits, form, &mn, &mx, &s, &z, codes.data()) == 0);
                    for (int i = 0; i < g; ++i) REQUIRE(codes[i] < (1u << bits));
                    REQUIRE(orc_pack_group(codes.data(), g, bits, packed.data()) == 0);
                    REQUIRE(orc_unpack_group(packed.data(), g, bits, back.data()) == 0);
                    for (int i = 0; i < g; ++i) REQUIRE(back[i] == codes[i]);
                    REQUIRE(orc_derive_scale_zero_form(mn, mx, bits, form, &s, &z) == 0);
                }
    REQUIRE(orc_quantize_group_form(nullptr, 32, 2, 0, nullptr, nullptr, nullptr, nullptr, nullptr) < 0);
    REQUIRE(orc_pack_group(nullptr, 32, 2, nullptr) < 0);
    REQUIRE(orc_derive_scale_zero_form(0.f, 1.f, 9, 0, nullptr, nullptr) < 0);
    REQUIRE(orc_cache_create_form(128, 3, 32, 64, 0, 0) == nullptr);
    REQUIRE(orc_cache_create_form(128, 2, 48, 64, 0, 0) == nullptr);
    REQUIRE(orc_cache_create_form(128, 2, 32, 48, 0, 0) == nullptr);
    REQUIRE(orc_cache_append(nullptr, nullptr, nullptr, 1) < 0);
    REQUIRE(orc_cache_counts(nullptr, nullptr, nullptr) < 0);

    const int D = 128;
    struct Cfg { int bits, g, R, dtype, form, G, S; };
    const Cfg cfgs[] = {{2, 32, 64, 0, 0, 1, 700}, {1, 32, 64, 1, 0, 4, 500}, {1, 64, 128, 1, 1, 2, 450},
                        {4, 128, 256, 0, 0, 8, 600}, {2, 64, 64, 1, 0, 2, 330}, {8, 32, 32, 0, 0, 1, 100}};
    for (const Cfg& c : cfgs) {
        void* h = orc_cache_create_form(D, c.bits, c.g, c.R, c.dtype, c.form);
        REQUIRE(h != nullptr);
        std::vector<uint16_t> k((size_t)c.S * D), v((size_t)c.S * D);
        for (auto& e : k) e = next_pattern(c.dtype);
        for (auto& e : v) e = next_pattern(c.dtype);
        // half in one call, the rest token by token (crosses every flush boundary both ways)
        const int half = c.S / 2;
        REQUIRE(orc_cache_append(h, k.data(), v.data(), half) == 0);
        for (int t = half; t < c.S; ++t) REQUIRE(orc_cache_append(h, &k[(size_t)t * D], &v[(size_t)t * D], 1) == 0);
        REQUIRE(orc_cache_append(h, nullptr, nullptr, 0) == 0);
        int N = 0, Nq = 0;
        REQUIRE(orc_cache_counts(h, &N, &Nq) == 0);
        REQUIRE(N == c.S && Nq % c.g == 0 && N - Nq < c.R && N - Nq >= c.R - c.g);
        std::vector<uint8_t> kc((size_t)Nq * D), vc((size_t)Nq * D);
        std::vector<float> kmm((size_t)(Nq / c.g) * D * 2), ksz(kmm.size()), vmm((size_t)Nq * (D / c.g) * 2), vsz(vmm.size());
        REQUIRE(orc_cache_export(h, kc.data(), kmm.data(), ksz.data(), vc.data(), vmm.data(), vsz.data()) == 0);
        REQUIRE(orc_cache_export(h, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == 0);
        std::vector<double> kd((size_t)Nq * D), vd((size_t)Nq * D), kh((size_t)N * D), vh((size_t)N * D);
        REQUIRE(orc_cache_dequant(h, kd.data(), vd.data()) == 0);
        REQUIRE(orc_cache_history(h, kh.data(), vh.data()) == 0);
        for (int rows = 1; rows <= 2; ++rows) {
            std::vector<uint16_t> q((size_t)c.G * rows * D), ks(D), vs(D);
            for (auto& e : q) e = next_pattern(c.dtype);
            for (auto& e : ks) e = next_pattern(c.dtype);
            for (auto& e : vs) e = next_pattern(c.dtype);
            std::vector<double> logits((size_t)c.G * rows * Nq), sigma(Nq), out((size_t)c.G * rows * D), w((size_t)c.G * rows * N);
            const int kk = 48;
            std::vector<int32_t> idx(kk), all(Nq + 5);
            for (int form = 0; form < 2; ++form) {
                REQUIRE(orc_scores_mixed(h, q.data(), c.G, rows, 0.088, form, nullptr, 0, logits.data(), sigma.data()) == 0);
                REQUIRE(orc_topk(sigma.data(), Nq, kk, idx.data()) == 0);
                for (int j = 0; j < kk; ++j) REQUIRE(idx[j] >= -1 && idx[j] < Nq);
                REQUIRE(orc_scores_mixed(h, q.data(), c.G, rows, 0.088, form, idx.data(), kk, logits.data(), sigma.data()) == 0);
            }
            REQUIRE(orc_topk(sigma.data(), Nq, Nq + 5, all.data()) == 0);       // k > n: padded
            REQUIRE(all[Nq] == -1 && all[Nq + 4] == -1);
            REQUIRE(orc_topk(sigma.data(), Nq, 0, nullptr) == 0);
            std::vector<double> ties(64, 1.0);
            REQUIRE(orc_topk(ties.data(), 64, 5, idx.data()) == 0);
            REQUIRE(idx[0] == 0 && idx[4] == 4);
            REQUIRE(orc_attend(h, q.data(), c.G, rows, 0.088, idx.data(), kk, ks.data(), vs.data(), out.data()) == 0);
            REQUIRE(orc_attend(h, q.data(), c.G, rows, 0.088, nullptr, 0, nullptr, nullptr, out.data()) == 0);
            REQUIRE(orc_attend(h, q.data(), c.G, rows, 0.088, all.data(), Nq + 5, ks.data(), vs.data(), out.data()) == 0);
            REQUIRE(orc_full_attention(h, q.data(), c.G, rows, 0.088, ks.data(), vs.data(), out.data(), w.data()) == 0);
            const double hit = orc_hit_rate(w.data(), N, all.data(), Nq + 5);
            REQUIRE(hit >= 0.0 && hit <= 1.0 + 1e-9);
            // rejected arguments leave nothing written
            int32_t bad = Nq;
            REQUIRE(orc_attend(h, q.data(), c.G, rows, 0.088, &bad, 1, nullptr, nullptr, out.data()) < 0);
            REQUIRE(orc_attend(h, q.data(), c.G, rows, 0.088, nullptr, 0, ks.data(), nullptr, out.data()) < 0);
            REQUIRE(orc_scores_mixed(h, q.data(), c.G, rows, 0.088, 2, nullptr, 0, nullptr, nullptr) < 0);
            REQUIRE(orc_scores_mixed(h, q.data(), c.G, rows, 0.088, 0, &bad, 1, nullptr, sigma.data()) < 0);
        }
        orc_cache_destroy(h);
    }
    // an empty cache: no candidate is an error, not a crash
    {
        void* h = orc_cache_create_form(D, 2, 32, 64, 0, 0);
        std::vector<uint16_t> q(2 * D, 0x3C00);
        std::vector<double> out(2 * D);
        REQUIRE(orc_attend(h, q.data(), 1, 2, 0.088, nullptr, 0, nullptr, nullptr, out.data()) < 0);
        REQUIRE(orc_scores_mixed(h, q.data(), 1, 2, 0.088, 0, nullptr, 0, nullptr, nullptr) == 0);
        orc_cache_destroy(h);
    }
    orc_cache_destroy(nullptr);
    std::printf("sanitize_driver ok %g\n", acc);
    return 0;
}
