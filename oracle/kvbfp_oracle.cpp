// CPU oracle for the BFP KV-cache path of "Accurate Block Quantization in LLMs
// with Outliers" (Trukhanov & Soloveychik).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
// definition the GPU library is judged against.  It shares no code with the
// HIP path, is never called by it, and may only be used by the tests, the
// smoke check and the CPU-baseline leg of the benchmark.
//
// Every floating-point step is done in double; inputs arrive as fp32 values
// (fp16/bf16 inputs are widened exactly by the caller, so the arithmetic here
// is defined on the same real numbers the GPU sees).
//
// Readings of the paper where it is silent (all listed again in the design
// notes of the repository):
//   * shared exponent: the finest power-of-two scale for which plain
//     round-to-nearest-even of the block's largest magnitude still fits the
//     symmetric mantissa range (Sec. II-B derives the exponent from the block's
//     largest magnitude; mantissas in [-(2^(p-1)-1), 2^(p-1)-1]);
//   * stored exponent byte E = e + 127 + (p-2), E = 0 reserved for an all-zero
//     block, b = 8 exponent bits (Sec. I: BFP12/BFP16 use an 8-bit exponent);
//   * rounding: to nearest (Sec. IV names no tie rule), ties to even;
//   * mantissa code: sign-magnitude, zero always encoded with sign 0;
//   * permutation: stable ascending argsort of the per-channel statistic
//     (Alg. 1 steps 1-2; Sec. III allows either order, a flag selects
//     descending).
//
// Parity pins for each function are in tests/test_oracle_*.py; none is
// "parity unpinned" except reproduction of Table I, which needs weights and a
// dataset that are not available.

#include <cfenv>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>
#include <algorithm>

namespace {

// ---------------------------------------------------------------------------
// Sec. II-B, Eq. (1): one block of n values -> exponent byte + integer mantissas
// ---------------------------------------------------------------------------

// round half to even of a double that is far below 2^52
inline double rne(double v) {
    // nearbyint honours the current rounding mode; we run in FE_TONEAREST.
    return std::nearbyint(v);
}

// scale exponent e (value = 2^e * M) belonging to stored byte E
inline int scale_exp_of(int E, int p) { return E - 127 - (p - 2); }

// Shared exponent byte of a block with largest magnitude amax (> 0, finite):
// the smallest E in 1..255 with RNE(amax * 2^-e) <= q_max.
int block_exponent_byte(double amax, int p) {
    const double qmax = double((1 << (p - 1)) - 1);
    int k = 0;
    (void)std::frexp(amax, &k);          // amax = f * 2^k, f in [0.5, 1)
    // first guess: scaled value f * 2^(p-1) lies in [2^(p-2), 2^(p-1))
    int E = (k - (p - 1)) + 127 + (p - 2);
    if (E < 1) E = 1;
    // "fits" is monotone in E (a coarser scale only shrinks the scaled value), so
    // walking from the guess in both directions finds the smallest fitting E.
    while (E < 255 && rne(std::ldexp(amax, -scale_exp_of(E, p))) > qmax) ++E;
    while (E > 1 && rne(std::ldexp(amax, -scale_exp_of(E - 1, p))) <= qmax) --E;
    return E;
}

// Quantize one block x[0..n) (already in cache channel order).
// codes_out[i] = sign-magnitude code of element i (p bits), returns E.
int quantize_block(const double* x, int n, int p, int* codes_out) {
    double amax = 0.0;
    for (int i = 0; i < n; ++i) amax = std::max(amax, std::fabs(x[i]));
    if (amax == 0.0) {
        for (int i = 0; i < n; ++i) codes_out[i] = 0;
        return 0;
    }
    const int qmax = (1 << (p - 1)) - 1;
    const int E = block_exponent_byte(amax, p);
    const int e = scale_exp_of(E, p);
    for (int i = 0; i < n; ++i) {
        const double m = rne(std::ldexp(x[i], -e));
        const int mi = (int)std::fabs(m);
        if (mi > qmax) std::abort();      // the exponent rule guarantees the range
        const int sign = (m < 0.0) ? 1 : 0;   // m == -0.0 compares false: zero gets sign 0
        codes_out[i] = mi == 0 ? 0 : ((sign << (p - 1)) | mi);
    }
    return E;
}

inline double decode_code(int code, int E, int p) {
    const int mag = code & ((1 << (p - 1)) - 1);
    const int sign = (code >> (p - 1)) & 1;
    const double v = std::ldexp((double)mag, scale_exp_of(E, p));
    return sign ? -v : v;
}

// packed row layout: p = 8 -> byte j is code j; p = 4 -> byte i holds code 2i in
// its low nibble and code 2i+1 in its high nibble.
inline void store_code(uint8_t* row, int j, int p, int code) {
    if (p == 8) { row[j] = (uint8_t)code; return; }
    uint8_t b = row[j >> 1];
    if (j & 1) b = (uint8_t)((b & 0x0F) | (code << 4));
    else       b = (uint8_t)((b & 0xF0) | code);
    row[j >> 1] = b;
}
inline int load_code(const uint8_t* row, int j, int p) {
    if (p == 8) return row[j];
    const uint8_t b = row[j >> 1];
    return (j & 1) ? (b >> 4) : (b & 0x0F);
}

inline bool bfp_params_ok(int D, int n, int p) {
    if (!(p == 4 || p == 8)) return false;
    if (!(n == 16 || n == 32 || n == 64 || n == 128)) return false;
    if (D <= 0 || D % n != 0) return false;
    return true;
}

struct RoundingGuard {
    int saved;
    RoundingGuard() : saved(std::fegetround()) { std::fesetround(FE_TONEAREST); }
    ~RoundingGuard() { std::fesetround(saved); }
};

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------
// Alg. 1 steps 1-2 (and the calibration-statistic variant): per head, a
// statistic per channel, then a stable argsort.
//   stat 0: max over samples of |x|      (calibration rows)
//   stat 1: Euclidean norm over samples  (rows of W_k; compared through the
//           sum of squares, accumulated in double in sample order)
// x element (s, h, c) is x[s*sample_stride + h*head_stride + c*chan_stride].
// perm_out[h*D + j] = channel that lands at position j.
// ---------------------------------------------------------------------------
int kvo_calibrate_perm(const float* x, int64_t n_samples, int32_t n_heads, int32_t D,
                       int64_t sample_stride, int64_t head_stride, int64_t chan_stride,
                       int32_t stat, int32_t descending, int32_t* perm_out) {
    if (!x || !perm_out || n_samples <= 0 || n_heads <= 0 || D <= 0) return -1;
    if (stat != 0 && stat != 1) return -1;
    std::vector<double> key(D);
    std::vector<int32_t> idx(D);
    for (int h = 0; h < n_heads; ++h) {
        for (int c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int64_t s = 0; s < n_samples; ++s) {
                const double v = (double)x[s * sample_stride + h * head_stride + c * chan_stride];
                if (stat == 0) acc = std::max(acc, std::fabs(v));
                else acc += v * v;
            }
            key[c] = descending ? -acc : acc;
        }
        std::iota(idx.begin(), idx.end(), 0);
        std::stable_sort(idx.begin(), idx.end(),
                         [&](int32_t a, int32_t b) { return key[a] < key[b]; });
        for (int j = 0; j < D; ++j) perm_out[(int64_t)h * D + j] = idx[j];
    }
    return 0;
}

// Alg. 1 steps 3-4: out row (h, j) = in row (h, perm[h / heads_per_perm][j]).
int kvo_permute_weights(const float* w_in, float* w_out, int32_t n_heads, int32_t D,
                        int64_t row_len, int32_t heads_per_perm, const int32_t* perm) {
    if (!w_in || !w_out || !perm || n_heads <= 0 || D <= 0 || row_len <= 0 || heads_per_perm <= 0)
        return -1;
    for (int h = 0; h < n_heads; ++h) {
        const int32_t* pi = perm + (int64_t)(h / heads_per_perm) * D;
        for (int j = 0; j < D; ++j) {
            const float* src = w_in + ((int64_t)h * D + pi[j]) * row_len;
            float* dst = w_out + ((int64_t)h * D + j) * row_len;
            std::memcpy(dst, src, sizeof(float) * (size_t)row_len);
        }
    }
    return 0;
}

// Sec. III, last paragraph: the projection after attention takes the value permutation on its columns:
// out[r][(h, j)] = in[r][(h, perm[h / heads_per_perm][j])].
int kvo_permute_weight_columns(const float* w_in, float* w_out, int64_t n_rows, int32_t n_heads, int32_t D,
                               int32_t heads_per_perm, const int32_t* perm) {
    if (!w_in || !w_out || !perm || n_rows <= 0 || n_heads <= 0 || D <= 0 || heads_per_perm <= 0) return -1;
    for (int64_t r = 0; r < n_rows; ++r)
        for (int h = 0; h < n_heads; ++h)
            for (int j = 0; j < D; ++j)
                w_out[(r * n_heads + h) * D + j] =
                    w_in[(r * n_heads + h) * D + perm[(int64_t)(h / heads_per_perm) * D + j]];
    return 0;
}

// ---------------------------------------------------------------------------
// Cast rows to BFP (Sec. II-B) and place them in the packed cache.
//   x        : [B][n_new][H][D] fp32, contiguous
//   pos      : [B] first token position of each sequence's new rows
//   perm     : [H][D] or NULL; cache position j of a row holds x[perm[j]]
//   mant     : [B][H][S_max][D*p/8]   exp : [B][H][S_max][D/n]
// Bytes outside the written rows are left untouched.
// ---------------------------------------------------------------------------
int kvo_quantize_append(int32_t B, int32_t H, int32_t D, int32_t n, int32_t p, int64_t S_max,
                        const float* x, int32_t n_new, const int64_t* pos, const int32_t* perm,
                        uint8_t* mant, uint8_t* exp) {
    if (!x || !pos || !mant || !exp || B <= 0 || H <= 0 || n_new < 0) return -1;
    if (!bfp_params_ok(D, n, p)) return -1;
    RoundingGuard guard;
    const int NB = D / n;
    const int64_t row_bytes = (int64_t)D * p / 8;
    std::vector<double> row(D);
    std::vector<int> codes(n);
    for (int b = 0; b < B; ++b) {
        if (pos[b] < 0 || pos[b] + n_new > S_max) return -1;
        for (int t = 0; t < n_new; ++t) {
            for (int h = 0; h < H; ++h) {
                const float* src = x + (((int64_t)b * n_new + t) * H + h) * D;
                const int32_t* pi = perm ? perm + (int64_t)h * D : nullptr;
                for (int j = 0; j < D; ++j) row[j] = (double)src[pi ? pi[j] : j];
                const int64_t r = ((int64_t)b * H + h) * S_max + pos[b] + t;
                uint8_t* mrow = mant + r * row_bytes;
                uint8_t* erow = exp + r * NB;
                for (int blk = 0; blk < NB; ++blk) {
                    const int E = quantize_block(row.data() + blk * n, n, p, codes.data());
                    erow[blk] = (uint8_t)E;
                    for (int i = 0; i < n; ++i) store_code(mrow, blk * n + i, p, codes[i]);
                }
            }
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Eq. (1): value = 2^e * M.  out: [B][n_tok][H][D] double.
// perm NULL: out[j] = value at cache position j; else out[perm[j]] = that value.
// ---------------------------------------------------------------------------
int kvo_dequantize(int32_t B, int32_t H, int32_t D, int32_t n, int32_t p, int64_t S_max,
                   const uint8_t* mant, const uint8_t* exp, int64_t t0, int64_t n_tok,
                   const int32_t* perm, double* out) {
    if (!mant || !exp || !out || B <= 0 || H <= 0 || t0 < 0 || n_tok < 0 || t0 + n_tok > S_max)
        return -1;
    if (!bfp_params_ok(D, n, p)) return -1;
    const int NB = D / n;
    const int64_t row_bytes = (int64_t)D * p / 8;
    for (int b = 0; b < B; ++b)
        for (int64_t t = 0; t < n_tok; ++t)
            for (int h = 0; h < H; ++h) {
                const int64_t r = ((int64_t)b * H + h) * S_max + t0 + t;
                const uint8_t* mrow = mant + r * row_bytes;
                const uint8_t* erow = exp + r * NB;
                double* dst = out + (((int64_t)b * n_tok + t) * H + h) * D;
                const int32_t* pi = perm ? perm + (int64_t)h * D : nullptr;
                for (int j = 0; j < D; ++j) {
                    const double v = decode_code(load_code(mrow, j, p), erow[j / n], p);
                    dst[pi ? pi[j] : j] = v;
                }
            }
    return 0;
}

// ---------------------------------------------------------------------------
// Decode attention over the packed cache (Sec. III: keys are read back from the
// cache and multiplied with pi(q); the rest is ordinary softmax attention;
// values are treated the same way with their own permutation).
//   q   : [B][Hq][D] fp32 values, out: [B][Hq][D] double
//   query head h uses KV head h / (Hq / Hkv)
//   seq_len : [B] number of cached tokens to attend to (0 -> zeros)
//   perm_k / perm_v : [Hkv][D] or NULL
//   q_mant_bits : 0 = q used as is; 4 or 8 = q' is first cast to BFP with the
//                 cache's block size (Sec. III / Sec. IV: queries in BFP16)
// ---------------------------------------------------------------------------
int kvo_decode_attention(int32_t B, int32_t Hkv, int32_t Hq, int32_t D, int32_t n, int32_t p,
                         int64_t S_max,
                         const uint8_t* k_mant, const uint8_t* k_exp,
                         const uint8_t* v_mant, const uint8_t* v_exp,
                         const float* q, const int64_t* seq_len, double softmax_scale,
                         const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits,
                         double* out) {
    if (!k_mant || !k_exp || !v_mant || !v_exp || !q || !seq_len || !out) return -1;
    if (B <= 0 || Hkv <= 0 || Hq <= 0 || Hq % Hkv != 0) return -1;
    if (!bfp_params_ok(D, n, p)) return -1;
    if (!(q_mant_bits == 0 || q_mant_bits == 4 || q_mant_bits == 8)) return -1;
    RoundingGuard guard;
    const int G = Hq / Hkv;
    const int NB = D / n;
    const int64_t row_bytes = (int64_t)D * p / 8;
    std::vector<double> qp(D), o(D);
    std::vector<int> codes(n);
    std::vector<double> s;
    for (int b = 0; b < B; ++b) {
        const int64_t L = seq_len[b];
        if (L < 0 || L > S_max) return -1;
        s.assign((size_t)L, 0.0);
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const float* qrow = q + ((int64_t)b * Hq + h) * D;
            double* orow = out + ((int64_t)b * Hq + h) * D;
            const int32_t* pk = perm_k ? perm_k + (int64_t)g * D : nullptr;
            const int32_t* pv = perm_v ? perm_v + (int64_t)g * D : nullptr;
            for (int j = 0; j < D; ++j) qp[j] = (double)qrow[pk ? pk[j] : j];
            if (q_mant_bits) {
                for (int blk = 0; blk < NB; ++blk) {
                    const int E = quantize_block(qp.data() + blk * n, n, q_mant_bits, codes.data());
                    for (int i = 0; i < n; ++i)
                        qp[blk * n + i] = decode_code(codes[i], E, q_mant_bits);
                }
            }
            for (int j = 0; j < D; ++j) orow[j] = 0.0;
            if (L == 0) continue;
            const int64_t base = ((int64_t)b * Hkv + g) * S_max;
            double m = -std::numeric_limits<double>::infinity();
            for (int64_t t = 0; t < L; ++t) {
                const uint8_t* mrow = k_mant + (base + t) * row_bytes;
                const uint8_t* erow = k_exp + (base + t) * NB;
                double acc = 0.0;
                for (int j = 0; j < D; ++j)
                    acc += qp[j] * decode_code(load_code(mrow, j, p), erow[j / n], p);
                s[(size_t)t] = softmax_scale * acc;
                m = std::max(m, s[(size_t)t]);
            }
            double denom = 0.0;
            for (int j = 0; j < D; ++j) o[j] = 0.0;
            for (int64_t t = 0; t < L; ++t) {
                const double w = std::exp(s[(size_t)t] - m);
                denom += w;
                const uint8_t* mrow = v_mant + (base + t) * row_bytes;
                const uint8_t* erow = v_exp + (base + t) * NB;
                for (int j = 0; j < D; ++j)
                    o[j] += w * decode_code(load_code(mrow, j, p), erow[j / n], p);
            }
            for (int j = 0; j < D; ++j) orow[pv ? pv[j] : j] = o[j] / denom;
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Rotary embeddings in the reordered channel order (Sec. II-D, Eq. (RoFreq); Alg. 1 step 5).
//
// In the original channel order the rotation of a row x at token index m is
//     (R x)[c] = x[c] cos(m Theta[c]) + s[c] x[i[c]] sin(m Theta[c]),
// with, for the paper's ordering (pairs of consecutive channels, pair_layout 0)
//     Theta = [th_0, th_0, th_1, th_1, ...],  i = [1, 0, 3, 2, ...],  s = [-1, +1, -1, +1, ...],
// and for the half-split ordering of the open-source Llama code (footnote of Sec. III, pair_layout 1)
//     Theta = [th_0 .. th_{D/2-1}, th_0 .. th_{D/2-1}],  i[c] = (c + D/2) mod D,  s = [-1 x D/2, +1 x D/2].
// Alg. 1 step 5 applies the head's permutation to the three vectors: position j of the reordered row
// holds original channel perm[j], so Theta'[j] = Theta[perm[j]], s'[j] = s[perm[j]], and the partner
// of position j is the position that holds channel i[perm[j]]: i'[j] = perm^{-1}[ i[perm[j]] ].
//   theta      : float [D/2]
//   perm       : int32 [n_heads][D]  (gather convention, as everywhere here)
//   theta_out  : float [n_heads][D];  partner_out : int32 [n_heads][D];  sign_out : float [n_heads][D]
// ---------------------------------------------------------------------------
int kvo_permute_rope(int32_t D, int32_t n_heads, int32_t pair_layout, const float* theta,
                     const int32_t* perm, float* theta_out, int32_t* partner_out, float* sign_out) {
    if (D <= 0 || D % 2 != 0 || n_heads <= 0 || !theta || !perm || !theta_out || !partner_out || !sign_out)
        return -1;
    if (pair_layout != 0 && pair_layout != 1) return -1;
    std::vector<float> Theta(D), sgn(D);
    std::vector<int> partner(D), inv(D);
    for (int c = 0; c < D; ++c) {
        if (pair_layout == 0) {
            Theta[c] = theta[c / 2];
            partner[c] = (c % 2 == 0) ? c + 1 : c - 1;
            sgn[c] = (c % 2 == 0) ? -1.0f : 1.0f;
        } else {
            Theta[c] = theta[c % (D / 2)];
            partner[c] = (c + D / 2) % D;
            sgn[c] = (c < D / 2) ? -1.0f : 1.0f;
        }
    }
    for (int h = 0; h < n_heads; ++h) {
        const int32_t* pi = perm + (int64_t)h * D;
        std::fill(inv.begin(), inv.end(), -1);
        for (int j = 0; j < D; ++j) {
            if (pi[j] < 0 || pi[j] >= D || inv[pi[j]] != -1) return -1;   // not a permutation
            inv[pi[j]] = j;
        }
        for (int j = 0; j < D; ++j) {
            theta_out[(int64_t)h * D + j] = Theta[pi[j]];
            sign_out[(int64_t)h * D + j] = sgn[pi[j]];
            partner_out[(int64_t)h * D + j] = inv[partner[pi[j]]];
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Decode attention over a cache whose keys were stored BEFORE the rotary embedding (Sec. III, last
// paragraph of the algorithm's description: the keys are fetched from the cache, the correctly
// ordered rotary embedding is applied to them, then the product with pi(q) is taken).
// Per cached token t of a sequence (token index m = t), in the cache's channel order:
//     k_rot[j] = k'[j] cos(m Theta'[j]) + s'[j] k'[i'[j]] sin(m Theta'[j])
// with (Theta', i', s') of the token's kv-head as kvo_permute_rope returns them; the angle is the
// product of the integer m and the fp32 value Theta'[j], taken in double.  Everything else is
// kvo_decode_attention: q is used as given (already rotated at its own position by the caller),
// gathered through perm_k if that is given.
// ---------------------------------------------------------------------------
int kvo_decode_attention_rope(int32_t B, int32_t Hkv, int32_t Hq, int32_t D, int32_t n, int32_t p,
                              int64_t S_max,
                              const uint8_t* k_mant, const uint8_t* k_exp,
                              const uint8_t* v_mant, const uint8_t* v_exp,
                              const float* q, const int64_t* seq_len, double softmax_scale,
                              const int32_t* perm_k, const int32_t* perm_v,
                              const float* rope_theta, const int32_t* rope_partner, const float* rope_sign,
                              double* out) {
    if (!k_mant || !k_exp || !v_mant || !v_exp || !q || !seq_len || !out) return -1;
    if (!rope_theta || !rope_partner || !rope_sign) return -1;
    if (B <= 0 || Hkv <= 0 || Hq <= 0 || Hq % Hkv != 0) return -1;
    if (!bfp_params_ok(D, n, p)) return -1;
    for (int64_t i = 0; i < (int64_t)Hkv * D; ++i)
        if (rope_partner[i] < 0 || rope_partner[i] >= D) return -1;
    RoundingGuard guard;
    const int G = Hq / Hkv;
    const int NB = D / n;
    const int64_t row_bytes = (int64_t)D * p / 8;
    std::vector<double> qp(D), o(D), kraw(D), krot(D);
    std::vector<double> s;
    for (int b = 0; b < B; ++b) {
        const int64_t L = seq_len[b];
        if (L < 0 || L > S_max) return -1;
        s.assign((size_t)L, 0.0);
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const float* qrow = q + ((int64_t)b * Hq + h) * D;
            double* orow = out + ((int64_t)b * Hq + h) * D;
            const int32_t* pk = perm_k ? perm_k + (int64_t)g * D : nullptr;
            const int32_t* pv = perm_v ? perm_v + (int64_t)g * D : nullptr;
            const float* th = rope_theta + (int64_t)g * D;
            const int32_t* pa = rope_partner + (int64_t)g * D;
            const float* sg = rope_sign + (int64_t)g * D;
            for (int j = 0; j < D; ++j) qp[j] = (double)qrow[pk ? pk[j] : j];
            for (int j = 0; j < D; ++j) orow[j] = 0.0;
            if (L == 0) continue;
            const int64_t base = ((int64_t)b * Hkv + g) * S_max;
            double m = -std::numeric_limits<double>::infinity();
            for (int64_t t = 0; t < L; ++t) {
                const uint8_t* mrow = k_mant + (base + t) * row_bytes;
                const uint8_t* erow = k_exp + (base + t) * NB;
                for (int j = 0; j < D; ++j) kraw[j] = decode_code(load_code(mrow, j, p), erow[j / n], p);
                for (int j = 0; j < D; ++j) {
                    const double ang = (double)t * (double)th[j];
                    krot[j] = kraw[j] * std::cos(ang) + (double)sg[j] * kraw[pa[j]] * std::sin(ang);
                }
                double acc = 0.0;
                for (int j = 0; j < D; ++j) acc += qp[j] * krot[j];
                s[(size_t)t] = softmax_scale * acc;
                m = std::max(m, s[(size_t)t]);
            }
            double denom = 0.0;
            for (int j = 0; j < D; ++j) o[j] = 0.0;
            for (int64_t t = 0; t < L; ++t) {
                const double w = std::exp(s[(size_t)t] - m);
                denom += w;
                const uint8_t* mrow = v_mant + (base + t) * row_bytes;
                const uint8_t* erow = v_exp + (base + t) * NB;
                for (int j = 0; j < D; ++j)
                    o[j] += w * decode_code(load_code(mrow, j, p), erow[j / n], p);
            }
            for (int j = 0; j < D; ++j) orow[pv ? pv[j] : j] = o[j] / denom;
        }
    }
    return 0;
}

// Scores only (softmax_scale * q'.K^T) for one (b, h): used by invariance pins.
int kvo_scores(int32_t D, int32_t n, int32_t p, const uint8_t* k_mant, const uint8_t* k_exp,
               int64_t L, const double* q_perm, double softmax_scale, double* s_out) {
    if (!bfp_params_ok(D, n, p) || !k_mant || !k_exp || !q_perm || !s_out || L < 0) return -1;
    const int NB = D / n;
    const int64_t row_bytes = (int64_t)D * p / 8;
    for (int64_t t = 0; t < L; ++t) {
        double acc = 0.0;
        for (int j = 0; j < D; ++j)
            acc += q_perm[j] * decode_code(load_code(k_mant + t * row_bytes, j, p),
                                           k_exp[t * NB + j / n], p);
        s_out[t] = softmax_scale * acc;
    }
    return 0;
}

}  // extern "C"
