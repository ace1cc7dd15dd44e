// Host code of the library (csrc/host_ops.cpp) and the CPU oracle (oracle/kvbfp_oracle.cpp) linked into
// one plain program and driven over seeded inputs, to be built with -fsanitize=address,undefined.  It checks
// nothing numerically that the Python tests do not check better; its job is to walk every host entry
// point and every oracle function, including their error paths and edge cases (empty sequences, one
// token, subnormal and huge inputs, permutations, every block size and mantissa width), so that an
// out-of-bounds access, a misaligned access, a signed overflow or a bad shift would be reported.
// Where the library's host function and the oracle compute the same thing, the results are compared.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "kvbfp.h"
#include "kvbfp_internal.h"

extern "C" {
int kvo_calibrate_perm(const float* x, int64_t n_samples, int32_t n_heads, int32_t D, int64_t sample_stride,
                       int64_t head_stride, int64_t chan_stride, int32_t stat, int32_t descending, int32_t* perm_out);
int kvo_permute_weights(const float* w_in, float* w_out, int32_t n_heads, int32_t D, int64_t row_len,
                        int32_t heads_per_perm, const int32_t* perm);
int kvo_permute_weight_columns(const float* w_in, float* w_out, int64_t n_rows, int32_t n_heads, int32_t D,
                               int32_t heads_per_perm, const int32_t* perm);
int kvo_quantize_append(int32_t B, int32_t H, int32_t D, int32_t n, int32_t p, int64_t S_max, const float* x,
                        int32_t n_new, const int64_t* pos, const int32_t* perm, uint8_t* mant, uint8_t* exp);
int kvo_dequantize(int32_t B, int32_t H, int32_t D, int32_t n, int32_t p, int64_t S_max, const uint8_t* mant,
                   const uint8_t* exp, int64_t t0, int64_t n_tok, const int32_t* perm, double* out);
int kvo_decode_attention(int32_t B, int32_t Hkv, int32_t Hq, int32_t D, int32_t n, int32_t p, int64_t S_max,
                         const uint8_t* k_mant, const uint8_t* k_exp, const uint8_t* v_mant, const uint8_t* v_exp,
                         const float* q, const int64_t* seq_len, double softmax_scale, const int32_t* perm_k,
                         const int32_t* perm_v, int32_t q_mant_bits, double* out);
int kvo_permute_rope(int32_t D, int32_t n_heads, int32_t pair_layout, const float* theta, const int32_t* perm,
                     float* theta_out, int32_t* partner_out, float* sign_out);
int kvo_decode_attention_rope(int32_t B, int32_t Hkv, int32_t Hq, int32_t D, int32_t n, int32_t p, int64_t S_max,
                              const uint8_t* k_mant, const uint8_t* k_exp, const uint8_t* v_mant,
                              const uint8_t* v_exp, const float* q, const int64_t* seq_len, double softmax_scale,
                              const int32_t* perm_k, const int32_t* perm_v, const float* rope_theta,
                              const int32_t* rope_partner, const float* rope_sign, double* out);
int kvo_scores(int32_t D, int32_t n, int32_t p, const uint8_t* k_mant, const uint8_t* k_exp, int64_t L,
               const double* q_perm, double softmax_scale, double* s_out);
}

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint64_t next_u64() {                      // splitmix64
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static float next_normal() {
    const double u1 = ((next_u64() >> 11) + 1.0) / 9007199254740993.0, u2 = (next_u64() >> 11) / 9007199254740992.0;
    return (float)(std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586 * u2));
}
static int g_fail = 0;
#define EXPECT(cond)                                                          \
    do {                                                                      \
        if (!(cond)) { std::printf("FAIL %s:%d  %s\n", __FILE__, __LINE__, #cond); ++g_fail; } \
    } while (0)

static uint16_t to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int main() {
    const int D = 128;
    // ---- Alg. 1 steps 1-2 and 3-4: library host functions against the oracle, all three dtypes' widening
    for (int H : {1, 3}) {
        const int S = 37;
        std::vector<float> x((size_t)S * H * D);
        for (auto& v : x) v = next_normal();
        for (int h = 0; h < H; ++h)
            for (int s = 0; s < S; ++s) x[((size_t)s * H + h) * D + 5] *= 30.f;     // an outlier channel
        x[7] = x[8];                                                                // a tie candidate
        std::vector<int32_t> pl((size_t)H * D), po((size_t)H * D);
        for (int stat : {0, 1})
            for (int desc : {0, 1}) {
                EXPECT(kvbfp_calibrate_perm(x.data(), KVBFP_F32, S, H, D, (int64_t)H * D, D, 1, (kvbfp_stat)stat, desc, pl.data()) == KVBFP_OK);
                EXPECT(kvo_calibrate_perm(x.data(), S, H, D, (int64_t)H * D, D, 1, stat, desc, po.data()) == 0);
                EXPECT(pl == po);
            }
        std::vector<uint16_t> xb(x.size());
        for (size_t i = 0; i < x.size(); ++i) xb[i] = to_bf16(x[i]);
        EXPECT(kvbfp_calibrate_perm(xb.data(), KVBFP_BF16, S, H, D, (int64_t)H * D, D, 1, KVBFP_STAT_MAXABS, 0, pl.data()) == KVBFP_OK);
        EXPECT(kvbfp_calibrate_perm(xb.data(), KVBFP_F16, S, H, D, (int64_t)H * D, D, 1, KVBFP_STAT_MAXABS, 0, pl.data()) == KVBFP_OK);
        // weights: [H*D][row_len]
        const int row_len = 19, G = 2;
        std::vector<float> w((size_t)H * G * D * row_len), wl(w.size()), wo(w.size());
        for (auto& v : w) v = next_normal();
        EXPECT(kvo_calibrate_perm(x.data(), S, H, D, (int64_t)H * D, D, 1, 0, 0, po.data()) == 0);
        EXPECT(kvbfp_permute_weights(w.data(), wl.data(), KVBFP_F32, H * G, D, row_len, G, po.data()) == KVBFP_OK);
        EXPECT(kvo_permute_weights(w.data(), wo.data(), H * G, D, row_len, G, po.data()) == 0);
        EXPECT(wl == wo);
        // the same buffer read as [row_len][H*G*D]: columns
        EXPECT(kvbfp_permute_weight_columns(w.data(), wl.data(), KVBFP_F32, row_len, H * G, D, G, po.data()) == KVBFP_OK);
        EXPECT(kvo_permute_weight_columns(w.data(), wo.data(), row_len, H * G, D, G, po.data()) == 0);
        EXPECT(wl == wo);
        EXPECT(kvbfp_permute_weight_columns(w.data(), w.data() + 1, KVBFP_F32, row_len, H * G, D, G, po.data()) == KVBFP_ERR_INVALID_ARG);
        // error paths
        EXPECT(kvbfp_permute_weights(w.data(), w.data(), KVBFP_F32, H * G, D, row_len, G, po.data()) == KVBFP_ERR_INVALID_ARG);
        std::vector<int32_t> notperm(po);
        notperm[3] = notperm[4];
        EXPECT(kvbfp_permute_weights(w.data(), wl.data(), KVBFP_F32, H * G, D, row_len, G, notperm.data()) == KVBFP_ERR_INVALID_ARG);
        EXPECT(kvbfp_calibrate_perm(nullptr, KVBFP_F32, S, H, D, 1, 1, 1, KVBFP_STAT_L2, 0, pl.data()) == KVBFP_ERR_INVALID_ARG);
        EXPECT(std::strlen(kvbfp_last_error()) > 0);
        // Alg. 1 step 5
        std::vector<float> theta(D / 2), tl((size_t)H * D), to((size_t)H * D), sl((size_t)H * D), so((size_t)H * D);
        std::vector<int32_t> al((size_t)H * D), ao((size_t)H * D);
        for (int i = 0; i < D / 2; ++i) theta[i] = (float)std::pow(10000.0, -2.0 * i / D);
        for (int layout : {0, 1}) {
            EXPECT(kvbfp_permute_rope(theta.data(), (kvbfp_rope_pairs)layout, H, D, po.data(), tl.data(), al.data(), sl.data()) == KVBFP_OK);
            EXPECT(kvo_permute_rope(D, H, layout, theta.data(), po.data(), to.data(), ao.data(), so.data()) == 0);
            EXPECT(tl == to && al == ao && sl == so);
        }
        EXPECT(kvbfp_permute_rope(theta.data(), KVBFP_ROPE_PAIRS_ADJACENT, H, D, notperm.data(), tl.data(), al.data(), sl.data()) == KVBFP_ERR_INVALID_ARG);
    }
    // ---- geometry helpers
    {
        kvbfp_layout L{(uint32_t)sizeof(kvbfp_layout), 128, 32, 4, 8, 8, 32769};
        size_t mb = 0, eb = 0;
        EXPECT(kvbfp_cache_bytes(&L, &mb, &eb) == KVBFP_OK && mb == (size_t)8 * 8 * 32769 * 64 && eb == (size_t)8 * 8 * 32769 * 4);
        L.block = 24;
        EXPECT(kvbfp_cache_bytes(&L, &mb, &eb) != KVBFP_OK);
        L.block = 32;
        EXPECT(kvbfp::plan_splits(&L, 32, 32769).n_splits == 12);
        kvbfp_layout pool{(uint32_t)sizeof(kvbfp_layout), 128, 16, 4, 2, 40, 256}, logical;
        int32_t dummy = 0;
        EXPECT(kvbfp::check_paging(&pool, kvbfp::Paging{&dummy, 5, 3}, &logical) == KVBFP_OK && logical.max_seq == 1280 && logical.batch == 3);
        pool.max_seq = 48;
        EXPECT(kvbfp::check_paging(&pool, kvbfp::Paging{&dummy, 5, 3}, &logical) == KVBFP_ERR_UNSUPPORTED);
        kvbfp_cache c{(uint8_t*)0x1000, (uint8_t*)0x2001, (uint8_t*)0x3008, (uint8_t*)0x4000};
        EXPECT(kvbfp::check_cache(&c, true, false) == KVBFP_OK && kvbfp::check_cache(&c, true, true) == KVBFP_ERR_INVALID_ARG);
    }
    // ---- the oracle: cast, decode, attention (plain, BFP query, rotation at read) over every format
    for (int p : {4, 8})
        for (int n : {16, 32, 64, 128}) {
            const int B = 2, H = 2, G = 3, S_max = 70, n_new = 67;
            const int NB = D / n, rowb = D * p / 8;
            std::vector<float> x((size_t)B * n_new * H * D);
            for (auto& v : x) v = next_normal();
            // edge values: zeros, a subnormal block, the largest finite value, a tie, a negative that rounds to zero
            for (int j = 0; j < n; ++j) x[j] = 0.f;
            for (int j = 0; j < D; ++j) x[(size_t)1 * H * D + j] = std::ldexp(next_normal(), -140);
            x[(size_t)2 * H * D + 3] = 3.4028234663852886e38f;
            x[(size_t)3 * H * D + 0] = 6.5f;
            x[(size_t)3 * H * D + 1] = -0.01f;
            std::vector<int32_t> perm((size_t)H * D);
            for (int h = 0; h < H; ++h)
                for (int j = 0; j < D; ++j) perm[(size_t)h * D + j] = (j * 37 + 11 * h) % D;     // 37 is coprime to 128
            std::vector<uint8_t> km((size_t)B * H * S_max * rowb, 0xA5), ke((size_t)B * H * S_max * NB, 0xA5), vm(km), ve(ke);
            const int64_t pos[2] = {0, 3};
            EXPECT(kvo_quantize_append(B, H, D, n, p, S_max, x.data(), n_new, pos, perm.data(), km.data(), ke.data()) == 0);
            EXPECT(kvo_quantize_append(B, H, D, n, p, S_max, x.data(), n_new, pos, nullptr, vm.data(), ve.data()) == 0);
            EXPECT(km[(size_t)(S_max - 1) * rowb] == 0xA5);                          // rows beyond the append untouched
            std::vector<double> deq((size_t)B * 5 * H * D);
            EXPECT(kvo_dequantize(B, H, D, n, p, S_max, km.data(), ke.data(), 3, 5, perm.data(), deq.data()) == 0);
            EXPECT(kvo_dequantize(B, H, D, n, p, S_max, km.data(), ke.data(), S_max - 1, 2, nullptr, deq.data()) != 0);
            std::vector<float> q((size_t)B * H * G * D);
            for (auto& v : q) v = next_normal();
            std::vector<double> out((size_t)B * H * G * D);
            for (int qb : {0, 4, 8}) {
                const int64_t lens[2] = {67, 1};
                EXPECT(kvo_decode_attention(B, H, H * G, D, n, p, S_max, km.data(), ke.data(), vm.data(), ve.data(), q.data(), lens,
                                            0.0884, perm.data(), perm.data(), qb, out.data()) == 0);
                for (double v : out) EXPECT(std::isfinite(v));
            }
            const int64_t empty[2] = {0, 0};
            EXPECT(kvo_decode_attention(B, H, H * G, D, n, p, S_max, km.data(), ke.data(), vm.data(), ve.data(), q.data(), empty,
                                        0.0884, nullptr, nullptr, 0, out.data()) == 0);
            for (double v : out) EXPECT(v == 0.0);
            std::vector<float> theta(D / 2), th((size_t)H * D), sg((size_t)H * D);
            std::vector<int32_t> pa((size_t)H * D);
            for (int i = 0; i < D / 2; ++i) theta[i] = (float)std::pow(10000.0, -2.0 * i / D);
            EXPECT(kvo_permute_rope(D, H, 1, theta.data(), perm.data(), th.data(), pa.data(), sg.data()) == 0);
            const int64_t lens[2] = {67, 40};
            EXPECT(kvo_decode_attention_rope(B, H, H * G, D, n, p, S_max, km.data(), ke.data(), vm.data(), ve.data(), q.data(), lens,
                                             0.0884, perm.data(), nullptr, th.data(), pa.data(), sg.data(), out.data()) == 0);
            for (double v : out) EXPECT(std::isfinite(v));
            std::vector<double> qd(D), sc(60);
            for (int j = 0; j < D; ++j) qd[j] = q[j];
            EXPECT(kvo_scores(D, n, p, km.data() + 5 * rowb, ke.data() + 5 * NB, 60, qd.data(), 1.0, sc.data()) == 0);
            for (double v : sc) EXPECT(std::isfinite(v));
        }
    if (g_fail) { std::printf("%d checks failed\n", g_fail); return 1; }
    std::printf("sanitize_host ok\n");
    return 0;
}
