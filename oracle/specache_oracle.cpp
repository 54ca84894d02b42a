// SpeCache decode-step oracle: TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-threaded CPU statement of what one attention layer's
// SpeCache decode step computes, written from the paper's definitions
// (arXiv 2503.16163: Section 3.3 "Decoding" with Eq. 1, Section 3.4 with
// Eq. 2 and Eq. 3, Section 4.1 "Implementation Details", Appendix A
// algorithms "Pre-decoding" and "Decoding").  It shares no code, header,
// table or constant with the GPU library.  Only tests, the smoke check and
// the benchmark's cpu_baseline leg may load it; the product path never does.
//
// Conventions
//   * 16-bit inputs arrive as raw bit patterns (uint16) plus a dtype flag
//     (0 = IEEE binary16, 1 = bfloat16) and are widened exactly to float.
//   * The quantiser (Eq. 2 / Eq. 3) is evaluated in IEEE binary32 in a fixed
//     operation order, because its result is an integer code that the GPU
//     path must reproduce bit for bit.  Build with -ffp-contract=off.
//   * Every dot product, softmax and weighted sum accumulates in double.
//   * No blocking, fusion or reordering: each function is the definition.
//
// Pins (tests/test_oracle_*.py): Eq. 3 interval statement, Eq. 2 closed form,
// Table 1 cache-size column, half-step bound, streaming == one-shot,
// k = Nq reduces to textbook attention, k = 0 reduces to low-bit attention,
// top-k against a full sort, softmax weights sum to one.
// The paper prints no worked numeric example of the quantiser, the scores or
// the attention output, so against the paper's own numbers these functions
// are "parity unpinned"; the pins above are closed forms, invariants and
// reductions to textbook routines.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>
#include <limits>
#include <new>

namespace {

// ---- exact widening of 16-bit floating-point bit patterns -----------------

float binary16_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h >> 15) & 1u;
    const uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
    const uint32_t frac = (uint32_t)h & 0x3FFu;
    double v;
    if (expo == 0) {
        v = std::ldexp((double)frac, -24);              // subnormal or zero
    } else if (expo == 31) {
        v = frac ? std::numeric_limits<double>::quiet_NaN()
                 : std::numeric_limits<double>::infinity();
    } else {
        v = std::ldexp(1.0 + (double)frac / 1024.0, (int)expo - 15);
    }
    return (float)(sign ? -v : v);                       // exact: fits binary32
}

float bfloat16_to_float(uint16_t h) {
    const uint32_t bits = (uint32_t)h << 16;             // top half of a binary32
    float f;
    std::memcpy(&f, &bits, sizeof f);
    return f;
}

float widen(uint16_t bits, int dtype) {
    return dtype == 0 ? binary16_to_float(bits) : bfloat16_to_float(bits);
}

// ---- Eq. 2 / Eq. 3: one quantisation group ---------------------------------
//
// Given g values X: mn = min X, mx = max X.
//   B >= 2 (Eq. 2):  z = mn,                 s = (mx - mn) * c_B,  c_B = float(1/(2^B-1))
//   B == 1 (Eq. 3):  z = (3*mn + mx) * 0.25, s = (mx - mn) * 0.5
//   B == 1, form 1 (the unmodified 1-bit KIVI of Section 4.4 / Table 5, "original"): Eq. 2 with
//                    B = 1, i.e. z = mn, s = mx - mn: the two levels are the group's extremes
//   code = clamp( floor((x - z)/s + 0.5), 0, 2^B-1 ),  all in binary32;
//   s == 0 (constant group) -> every code 0.
// Rounding is half-up, which matches Eq. 3's closed lower / open upper
// interval ends (the exact midpoint belongs to the upper level).

void derive_scale_zero(float mn, float mx, int bits, int one_bit_form, float* s, float* z) {
    if (bits == 1 && one_bit_form == 0) {
        const float three_mn = 3.0f * mn;
        const float sum = three_mn + mx;
        *z = sum * 0.25f;
        const float range = mx - mn;
        *s = range * 0.5f;
    } else {
        const float cB = (float)(1.0 / (double)((1 << bits) - 1));
        *z = mn;
        const float range = mx - mn;
        *s = range * cB;
    }
}

int quantize_one(float x, float s, float z, int bits) {
    if (s == 0.0f) return 0;
    const float d = x - z;
    const float t = d / s;
    const float u = t + 0.5f;
    const float r = std::floor(u);
    const int top = (1 << bits) - 1;
    int c = (int)r;
    if (c < 0) c = 0;
    if (c > top) c = top;
    return c;
}

void quantize_group(const float* x, int g, int stride, int bits, int one_bit_form,
                    float* mn_out, float* mx_out, uint8_t* codes, int code_stride) {
    float mn = x[0], mx = x[0];
    for (int e = 1; e < g; ++e) {
        const float v = x[(size_t)e * stride];
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    float s, z;
    derive_scale_zero(mn, mx, bits, one_bit_form, &s, &z);
    for (int e = 0; e < g; ++e)
        codes[(size_t)e * code_stride] = (uint8_t)quantize_one(x[(size_t)e * stride], s, z, bits);
    *mn_out = mn;
    *mx_out = mx;
}

// ---- the cache of one (batch, KV head) --------------------------------------
//
// Holds what the method holds: the full-precision history (the paper's CPU
// copy C), and for the quantised prefix [0, Nq) the low-bit copy C' (codes and
// the per-group (min, max) pair kept in the cache's 16-bit type).
// Keys are grouped per channel over g consecutive tokens, values per token
// over g consecutive channels (Section 2.1 / 4.1, following KIVI).
// Residual policy (the paper omits it from its pseudocode): tokens are
// appended one at a time; whenever N - Nq reaches R the oldest g unquantised
// tokens are quantised, so Nq is always a multiple of g.

struct Cache {
    int D, bits, g, R, dtype;
    int one_bit_form = 0;                    // 0: Eq. 3; 1: Eq. 2 with B = 1 (Table 5 "original")
    int N = 0, Nq = 0;
    std::vector<uint16_t> k_raw, v_raw;      // [N][D] 16-bit patterns as given
    std::vector<float> k_full, v_full;       // [N][D] widened
    std::vector<uint8_t> k_code, v_code;     // [Nq][D]
    std::vector<float> k_mn, k_mx;           // [Nq/g][D]
    std::vector<float> v_mn, v_mx;           // [Nq][D/g]
};

void flush_oldest_group(Cache& c) {
    const int D = c.D, g = c.g, t0 = c.Nq;
    c.k_code.resize((size_t)(t0 + g) * D);
    c.v_code.resize((size_t)(t0 + g) * D);
    c.k_mn.resize((size_t)(t0 / g + 1) * D);
    c.k_mx.resize((size_t)(t0 / g + 1) * D);
    c.v_mn.resize((size_t)(t0 + g) * (D / g));
    c.v_mx.resize((size_t)(t0 + g) * (D / g));
    // keys: one group per channel, running over the g tokens
    for (int ch = 0; ch < D; ++ch) {
        quantize_group(&c.k_full[(size_t)t0 * D + ch], g, D, c.bits, c.one_bit_form,
                       &c.k_mn[(size_t)(t0 / g) * D + ch], &c.k_mx[(size_t)(t0 / g) * D + ch],
                       &c.k_code[(size_t)t0 * D + ch], D);
    }
    // values: per token, one group per g consecutive channels
    for (int t = t0; t < t0 + g; ++t) {
        for (int m = 0; m < D / g; ++m) {
            quantize_group(&c.v_full[(size_t)t * D + m * g], g, 1, c.bits, c.one_bit_form,
                           &c.v_mn[(size_t)t * (D / g) + m], &c.v_mx[(size_t)t * (D / g) + m],
                           &c.v_code[(size_t)t * D + m * g], 1);
        }
    }
    c.Nq += g;
}

// dequantised key / value element, in double (x' = code*s + z, Eq. 2)
double deq_k(const Cache& c, int t, int ch) {
    float s, z;
    const size_t gi = (size_t)(t / c.g) * c.D + ch;
    derive_scale_zero(c.k_mn[gi], c.k_mx[gi], c.bits, c.one_bit_form, &s, &z);
    return (double)c.k_code[(size_t)t * c.D + ch] * (double)s + (double)z;
}

double deq_v(const Cache& c, int t, int ch) {
    float s, z;
    const size_t gi = (size_t)t * (c.D / c.g) + ch / c.g;
    derive_scale_zero(c.v_mn[gi], c.v_mx[gi], c.bits, c.one_bit_form, &s, &z);
    return (double)c.v_code[(size_t)t * c.D + ch] * (double)s + (double)z;
}

// softmax-weighted sum over an explicit candidate list
struct Candidate {
    std::vector<double> k, v;   // D each
};

void softmax_attend(const std::vector<double>& logits,
                    const std::vector<const double*>& vrows, int D, double* out,
                    double* weights_out) {
    double mx = -std::numeric_limits<double>::infinity();
    for (double l : logits) mx = std::max(mx, l);
    double denom = 0.0;
    std::vector<double> w(logits.size());
    for (size_t i = 0; i < logits.size(); ++i) { w[i] = std::exp(logits[i] - mx); denom += w[i]; }
    for (int ch = 0; ch < D; ++ch) out[ch] = 0.0;
    for (size_t i = 0; i < logits.size(); ++i) {
        const double p = w[i] / denom;
        if (weights_out) weights_out[i] = p;
        for (int ch = 0; ch < D; ++ch) out[ch] += p * vrows[i][ch];
    }
}

}  // namespace

extern "C" {

// Error codes of this library (negative = failure).
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ESTATE = -2 };

float orc_widen(uint16_t bits, int dtype) { return widen(bits, dtype); }

// Eq. 2 / Eq. 3 on one contiguous group of g floats.
// one_bit_form: 0 = Eq. 3, 1 = Eq. 2 with B = 1 (only read when bits == 1).
int orc_quantize_group_form(const float* x, int g, int bits, int one_bit_form, float* mn, float* mx,
                            float* s, float* z, uint8_t* codes) {
    if (!x || g <= 0 || bits < 1 || bits > 8 || (one_bit_form != 0 && one_bit_form != 1)) return ORC_EINVAL;
    quantize_group(x, g, 1, bits, one_bit_form, mn, mx, codes, 1);
    derive_scale_zero(*mn, *mx, bits, one_bit_form, s, z);
    return ORC_OK;
}

int orc_quantize_group(const float* x, int g, int bits, float* mn, float* mx,
                       float* s, float* z, uint8_t* codes) {
    return orc_quantize_group_form(x, g, bits, 0, mn, mx, s, z, codes);
}

int orc_derive_scale_zero_form(float mn, float mx, int bits, int one_bit_form, float* s, float* z) {
    if (bits < 1 || bits > 8 || (one_bit_form != 0 && one_bit_form != 1)) return ORC_EINVAL;
    derive_scale_zero(mn, mx, bits, one_bit_form, s, z);
    return ORC_OK;
}

int orc_derive_scale_zero(float mn, float mx, int bits, float* s, float* z) {
    return orc_derive_scale_zero_form(mn, mx, bits, 0, s, z);
}

// Canonical bit packing used for the bit-exact comparison of codes: element e
// of a group occupies bits [bits*e, bits*e + bits) of the group's g*bits-bit
// little-endian word.
int orc_pack_group(const uint8_t* codes, int g, int bits, uint8_t* packed) {
    if (!codes || !packed || g <= 0 || bits < 1 || bits > 8 || (g * bits) % 8) return ORC_EINVAL;
    std::memset(packed, 0, (size_t)g * bits / 8);
    for (int e = 0; e < g; ++e)
        for (int b = 0; b < bits; ++b) {
            const int pos = e * bits + b;
            if ((codes[e] >> b) & 1) packed[pos / 8] |= (uint8_t)(1u << (pos % 8));
        }
    return ORC_OK;
}

int orc_unpack_group(const uint8_t* packed, int g, int bits, uint8_t* codes) {
    if (!codes || !packed || g <= 0 || bits < 1 || bits > 8 || (g * bits) % 8) return ORC_EINVAL;
    for (int e = 0; e < g; ++e) {
        int c = 0;
        for (int b = 0; b < bits; ++b) {
            const int pos = e * bits + b;
            if ((packed[pos / 8] >> (pos % 8)) & 1) c |= 1 << b;
        }
        codes[e] = (uint8_t)c;
    }
    return ORC_OK;
}

void* orc_cache_create_form(int D, int bits, int g, int R, int dtype, int one_bit_form) {
    if (D <= 0 || (bits != 1 && bits != 2 && bits != 4 && bits != 8) || g <= 0 || D % g ||
        R < g || R % g || (dtype != 0 && dtype != 1) || (one_bit_form != 0 && one_bit_form != 1))
        return nullptr;
    Cache* c = new (std::nothrow) Cache();
    if (!c) return nullptr;
    c->D = D; c->bits = bits; c->g = g; c->R = R; c->dtype = dtype; c->one_bit_form = one_bit_form;
    return c;
}

void* orc_cache_create(int D, int bits, int g, int R, int dtype) {
    return orc_cache_create_form(D, bits, g, R, dtype, 0);
}

void orc_cache_destroy(void* h) { delete static_cast<Cache*>(h); }

// Append n tokens, one after the other (Appendix A "Decoding": the new pair is
// added to the 16-bit copy C and, through the residual policy, to C').
int orc_cache_append(void* h, const uint16_t* k_rows, const uint16_t* v_rows, int n) {
    Cache* c = static_cast<Cache*>(h);
    if (!c || n < 0 || (n > 0 && (!k_rows || !v_rows))) return ORC_EINVAL;
    for (int t = 0; t < n; ++t) {
        for (int ch = 0; ch < c->D; ++ch) {
            const uint16_t kb = k_rows[(size_t)t * c->D + ch], vb = v_rows[(size_t)t * c->D + ch];
            c->k_raw.push_back(kb);
            c->v_raw.push_back(vb);
            c->k_full.push_back(widen(kb, c->dtype));
            c->v_full.push_back(widen(vb, c->dtype));
        }
        c->N += 1;
        if (c->N - c->Nq == c->R) flush_oldest_group(*c);
    }
    return ORC_OK;
}

int orc_cache_counts(void* h, int* N, int* Nq) {
    Cache* c = static_cast<Cache*>(h);
    if (!c) return ORC_EINVAL;
    if (N) *N = c->N;
    if (Nq) *Nq = c->Nq;
    return ORC_OK;
}

// Canonical view of C': one code per byte, (min,max) as floats (exactly the
// stored 16-bit values) and the derived binary32 (s, z).
//   k_codes [Nq][D], k_mnmx [Nq/g][D][2], k_sz [Nq/g][D][2]
//   v_codes [Nq][D], v_mnmx [Nq][D/g][2], v_sz [Nq][D/g][2]
int orc_cache_export(void* h, uint8_t* k_codes, float* k_mnmx, float* k_sz,
                     uint8_t* v_codes, float* v_mnmx, float* v_sz) {
    Cache* c = static_cast<Cache*>(h);
    if (!c) return ORC_EINVAL;
    const int D = c->D, g = c->g;
    if (k_codes) std::memcpy(k_codes, c->k_code.data(), (size_t)c->Nq * D);
    if (v_codes) std::memcpy(v_codes, c->v_code.data(), (size_t)c->Nq * D);
    for (size_t i = 0; i < (size_t)(c->Nq / g) * D; ++i) {
        float s, z;
        derive_scale_zero(c->k_mn[i], c->k_mx[i], c->bits, c->one_bit_form, &s, &z);
        if (k_mnmx) { k_mnmx[2 * i] = c->k_mn[i]; k_mnmx[2 * i + 1] = c->k_mx[i]; }
        if (k_sz) { k_sz[2 * i] = s; k_sz[2 * i + 1] = z; }
    }
    for (size_t i = 0; i < (size_t)c->Nq * (D / g); ++i) {
        float s, z;
        derive_scale_zero(c->v_mn[i], c->v_mx[i], c->bits, c->one_bit_form, &s, &z);
        if (v_mnmx) { v_mnmx[2 * i] = c->v_mn[i]; v_mnmx[2 * i + 1] = c->v_mx[i]; }
        if (v_sz) { v_sz[2 * i] = s; v_sz[2 * i + 1] = z; }
    }
    return ORC_OK;
}

// Dequantised low-bit copy as doubles: k_deq, v_deq [Nq][D]  (X' of Eq. 2).
int orc_cache_dequant(void* h, double* k_deq, double* v_deq) {
    Cache* c = static_cast<Cache*>(h);
    if (!c) return ORC_EINVAL;
    for (int t = 0; t < c->Nq; ++t)
        for (int ch = 0; ch < c->D; ++ch) {
            if (k_deq) k_deq[(size_t)t * c->D + ch] = deq_k(*c, t, ch);
            if (v_deq) v_deq[(size_t)t * c->D + ch] = deq_v(*c, t, ch);
        }
    return ORC_OK;
}

// Full-precision history as doubles: k, v [N][D].
int orc_cache_history(void* h, double* k, double* v) {
    Cache* c = static_cast<Cache*>(h);
    if (!c) return ORC_EINVAL;
    for (size_t i = 0; i < (size_t)c->N * c->D; ++i) {
        if (k) k[i] = c->k_full[i];
        if (v) v[i] = c->v_full[i];
    }
    return ORC_OK;
}

// Low-bit logits (Appendix A "Decoding": Q K^T on the low-bit copy):
//   logits[h][row][i] = sm_scale * sum_c q[h][row][c] * K'[i][c],  i < Nq
// and the selection score of position i for this KV head (the paper is silent on how the G
// query heads of a KV head share one index set),
//   select_form 0:  sigma[i] = max over the G query heads of logits[h][rows-1][i];
//   select_form 1:  sigma[i] = max over the G query heads of the log-probability
//                   logits[h][rows-1][i] - log sum_{j < Nq} exp(logits[h][rows-1][j]),
//                   i.e. of the head's softmax over the low-bit positions (ArgTopK is applied to
//                   the softmax output A in Appendix A; per head the two orders agree, across
//                   heads this form weighs every head's distribution alike).
// q: [G][rows][D] 16-bit patterns.
// P (may be null): positions whose 16-bit pairs are staged; with it the logits are those of the
// mixed cache C' u C_K of Eq. 1 (Appendix A "Decoding" computes one A on the mixed cache and takes
// ArgTopK of its second row), i.e. position i in P is scored with its 16-bit key.  Without it they
// are the pure low-bit logits.  Entries < 0 are ignored.
int orc_scores_mixed(void* hc, const uint16_t* q, int G, int rows, double sm_scale, int select_form,
                     const int32_t* P, int nP, double* logits, double* sigma) {
    Cache* c = static_cast<Cache*>(hc);
    if (!c || !q || G <= 0 || rows <= 0 || (select_form != 0 && select_form != 1) || nP < 0 || (nP > 0 && !P))
        return ORC_EINVAL;
    const int D = c->D, Nq = c->Nq;
    std::vector<char> in_p(Nq, 0);
    for (int j = 0; j < nP; ++j) {
        if (P[j] < 0) continue;
        if (P[j] >= Nq) return ORC_ESTATE;
        in_p[P[j]] = 1;
    }
    std::vector<double> last((size_t)G * Nq);          // logits of the last row of every head
    for (int i = 0; i < Nq; ++i)
        for (int h = 0; h < G; ++h)
            for (int r = 0; r < rows; ++r) {
                double acc = 0.0;
                for (int ch = 0; ch < D; ++ch)
                    acc += (double)widen(q[((size_t)h * rows + r) * D + ch], c->dtype) *
                           (in_p[i] ? (double)c->k_full[(size_t)i * D + ch] : deq_k(*c, i, ch));
                const double l = sm_scale * acc;
                if (logits) logits[((size_t)h * rows + r) * Nq + i] = l;
                if (r == rows - 1) last[(size_t)h * Nq + i] = l;
            }
    if (!sigma) return ORC_OK;
    std::vector<double> lse(G, 0.0);
    if (select_form == 1)
        for (int h = 0; h < G; ++h) {
            double m = -std::numeric_limits<double>::infinity(), sum = 0.0;
            for (int i = 0; i < Nq; ++i) m = std::max(m, last[(size_t)h * Nq + i]);
            for (int i = 0; i < Nq; ++i) sum += std::exp(last[(size_t)h * Nq + i] - m);
            lse[h] = m + std::log(sum);
        }
    for (int i = 0; i < Nq; ++i) {
        double best = -std::numeric_limits<double>::infinity();
        for (int h = 0; h < G; ++h) best = std::max(best, last[(size_t)h * Nq + i] - lse[h]);
        sigma[i] = best;
    }
    return ORC_OK;
}

int orc_scores_form(void* hc, const uint16_t* q, int G, int rows, double sm_scale, int select_form,
                    double* logits, double* sigma) {
    return orc_scores_mixed(hc, q, G, rows, sm_scale, select_form, nullptr, 0, logits, sigma);
}

int orc_scores(void* hc, const uint16_t* q, int G, int rows, double sm_scale,
               double* logits, double* sigma) {
    return orc_scores_mixed(hc, q, G, rows, sm_scale, 0, nullptr, 0, logits, sigma);
}

// ArgTopK: the min(k, n) positions with the largest score, ties to the lower
// index, returned in ascending index order and padded with -1 up to k.
int orc_topk(const double* sigma, int n, int k, int32_t* idx_out) {
    if (n < 0 || k < 0 || (n > 0 && !sigma) || (k > 0 && !idx_out)) return ORC_EINVAL;
    std::vector<int32_t> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return sigma[a] > sigma[b]; });
    const int keff = std::min(k, n);
    std::vector<int32_t> sel(order.begin(), order.begin() + keff);
    std::sort(sel.begin(), sel.end());
    for (int i = 0; i < k; ++i) idx_out[i] = i < keff ? sel[i] : -1;
    return ORC_OK;
}

// Mixed attention, Eq. 1: Attn([T_t, T'_{t+1}], C' ∪ C_K).
// Candidates of every (head, row):
//   * quantised positions i < Nq: the 16-bit pair if i is in P, otherwise the
//     dequantised low-bit pair;
//   * residual positions Nq <= i < N: 16-bit;
//   * for the last row only, when given, the transient pair (k_spec, v_spec).
// out: [G][rows][D] doubles.  P: nP indices, entries < 0 ignored.
int orc_attend(void* hc, const uint16_t* q, int G, int rows, double sm_scale,
               const int32_t* P, int nP, const uint16_t* k_spec, const uint16_t* v_spec,
               double* out) {
    Cache* c = static_cast<Cache*>(hc);
    if (!c || !q || !out || G <= 0 || rows <= 0 || nP < 0 || (nP > 0 && !P)) return ORC_EINVAL;
    if ((k_spec == nullptr) != (v_spec == nullptr)) return ORC_EINVAL;
    const int D = c->D, N = c->N, Nq = c->Nq;
    std::vector<char> in_p(Nq, 0);
    for (int j = 0; j < nP; ++j) {
        if (P[j] < 0) continue;
        if (P[j] >= Nq) return ORC_ESTATE;
        in_p[P[j]] = 1;
    }
    // build the mixed cache once
    std::vector<double> km((size_t)(N + 1) * D), vm((size_t)(N + 1) * D);
    for (int i = 0; i < N; ++i)
        for (int ch = 0; ch < D; ++ch) {
            const bool full = i >= Nq || in_p[i];
            km[(size_t)i * D + ch] = full ? (double)c->k_full[(size_t)i * D + ch] : deq_k(*c, i, ch);
            vm[(size_t)i * D + ch] = full ? (double)c->v_full[(size_t)i * D + ch] : deq_v(*c, i, ch);
        }
    if (k_spec)
        for (int ch = 0; ch < D; ++ch) {
            km[(size_t)N * D + ch] = widen(k_spec[ch], c->dtype);
            vm[(size_t)N * D + ch] = widen(v_spec[ch], c->dtype);
        }
    for (int h = 0; h < G; ++h)
        for (int r = 0; r < rows; ++r) {
            const int ncand = N + ((k_spec && r == rows - 1) ? 1 : 0);
            if (ncand == 0) return ORC_ESTATE;
            std::vector<double> logits(ncand);
            std::vector<const double*> vrows(ncand);
            for (int i = 0; i < ncand; ++i) {
                double acc = 0.0;
                for (int ch = 0; ch < D; ++ch)
                    acc += (double)widen(q[((size_t)h * rows + r) * D + ch], c->dtype) * km[(size_t)i * D + ch];
                logits[i] = sm_scale * acc;
                vrows[i] = &vm[(size_t)i * D];
            }
            softmax_attend(logits, vrows, D, &out[((size_t)h * rows + r) * D], nullptr);
        }
    return ORC_OK;
}

// Textbook full-precision softmax attention over all N 16-bit tokens (plus the
// transient pair for the last row); also returns the softmax weights of every
// (head,row) over the N cached tokens when `weights` is non-null ([G][rows][N]).
int orc_full_attention(void* hc, const uint16_t* q, int G, int rows, double sm_scale,
                       const uint16_t* k_spec, const uint16_t* v_spec, double* out,
                       double* weights) {
    Cache* c = static_cast<Cache*>(hc);
    if (!c || !q || !out || G <= 0 || rows <= 0) return ORC_EINVAL;
    if ((k_spec == nullptr) != (v_spec == nullptr)) return ORC_EINVAL;
    const int D = c->D, N = c->N;
    std::vector<double> ks(D), vs(D);
    if (k_spec)
        for (int ch = 0; ch < D; ++ch) { ks[ch] = widen(k_spec[ch], c->dtype); vs[ch] = widen(v_spec[ch], c->dtype); }
    std::vector<double> kd((size_t)N * D), vd((size_t)N * D);
    for (size_t i = 0; i < (size_t)N * D; ++i) { kd[i] = c->k_full[i]; vd[i] = c->v_full[i]; }
    for (int h = 0; h < G; ++h)
        for (int r = 0; r < rows; ++r) {
            const bool spec = k_spec && r == rows - 1;
            const int ncand = N + (spec ? 1 : 0);
            if (ncand == 0) return ORC_ESTATE;
            std::vector<double> logits(ncand), w(ncand);
            std::vector<const double*> vrows(ncand);
            for (int i = 0; i < ncand; ++i) {
                const double* kr = i < N ? &kd[(size_t)i * D] : ks.data();
                double acc = 0.0;
                for (int ch = 0; ch < D; ++ch)
                    acc += (double)widen(q[((size_t)h * rows + r) * D + ch], c->dtype) * kr[ch];
                logits[i] = sm_scale * acc;
                vrows[i] = i < N ? &vd[(size_t)i * D] : vs.data();
            }
            softmax_attend(logits, vrows, D, &out[((size_t)h * rows + r) * D], w.data());
            if (weights)
                for (int i = 0; i < N; ++i) weights[((size_t)h * rows + r) * N + i] = w[i];
        }
    return ORC_OK;
}

// Hit rate (Section 3.1): the share of a full-attention weight vector that a
// set of positions captures.
double orc_hit_rate(const double* weights, int n, const int32_t* idx, int n_idx) {
    double hit = 0.0;
    for (int j = 0; j < n_idx; ++j)
        if (idx[j] >= 0 && idx[j] < n) hit += weights[idx[j]];
    return hit;
}

}  // extern "C"
