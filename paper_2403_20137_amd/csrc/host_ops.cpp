// Host side of libkvbfp: error strings, geometry helpers, and the two compile-time steps of
// K-sort (Alg. 1): ranking channels and reordering weight rows.  No device code here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <utility>
#include <vector>

#include "kvbfp_internal.h"

namespace kvbfp {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
void clear_error() { g_err[0] = '\0'; }

int check_device_layout(const kvbfp_layout* L) {
    if (!L) return fail(KVBFP_ERR_INVALID_ARG, "layout is NULL");
    if (L->struct_bytes != sizeof(kvbfp_layout))
        return fail(KVBFP_ERR_INVALID_ARG, "layout.struct_bytes = %u, expected %zu", L->struct_bytes,
                    sizeof(kvbfp_layout));
    if (L->batch <= 0 || L->n_kv_heads <= 0 || L->max_seq <= 0 || L->head_dim <= 0)
        return fail(KVBFP_ERR_INVALID_ARG, "layout sizes must be positive");
    if (!(L->mant_bits == 4 || L->mant_bits == 8))
        return fail(KVBFP_ERR_UNSUPPORTED, "mant_bits = %d (supported: 4, 8)", L->mant_bits);
    if (!(L->block == 16 || L->block == 32 || L->block == 64 || L->block == 128))
        return fail(KVBFP_ERR_UNSUPPORTED, "block = %d (supported: 16, 32, 64, 128)", L->block);
    if (L->head_dim % L->block != 0)
        return fail(KVBFP_ERR_INVALID_ARG, "head_dim %d is not a multiple of block %d", L->head_dim,
                    L->block);
    if (L->head_dim != 128)
        return fail(KVBFP_ERR_UNSUPPORTED, "head_dim = %d (device kernels support 128)", L->head_dim);
    if (L->max_seq > (int64_t)1 << 30)
        return fail(KVBFP_ERR_UNSUPPORTED, "max_seq too large");
    return KVBFP_OK;
}

int check_cache(const kvbfp_cache* c, bool need_k, bool need_v) {
    if (!c) return fail(KVBFP_ERR_INVALID_ARG, "cache is NULL");
    if (need_k && (!c->k_mant || !c->k_exp))
        return fail(KVBFP_ERR_INVALID_ARG, "cache key planes are NULL");
    if (need_v && (!c->v_mant || !c->v_exp))
        return fail(KVBFP_ERR_INVALID_ARG, "cache value planes are NULL");
    // every kernel moves mantissa rows with 8- and 16-byte accesses; exponent planes are read and written
    // byte-wise wherever they are not 16-byte aligned
    if ((need_k && (uintptr_t)c->k_mant % 16 != 0) || (need_v && (uintptr_t)c->v_mant % 16 != 0))
        return fail(KVBFP_ERR_INVALID_ARG, "cache mantissa planes must be 16-byte aligned");
    return KVBFP_OK;
}

int check_paging(const kvbfp_layout* pool, const Paging& pg, kvbfp_layout* logical) {
    if (int rc = check_device_layout(pool)) return rc;
    if (!pg.block_table) return fail(KVBFP_ERR_INVALID_ARG, "paged cache: block_table is NULL");
    const int64_t page = pool->max_seq;
    if (page < kPageMin || (page & (page - 1)) != 0)
        return fail(KVBFP_ERR_UNSUPPORTED, "paged cache: %lld tokens per page (a power of two, at least %d)",
                    (long long)page, kPageMin);
    if (pg.batch <= 0 || pg.table_stride <= 0)
        return fail(KVBFP_ERR_INVALID_ARG, "paged cache: batch %d, table_stride %lld", pg.batch, (long long)pg.table_stride);
    if (pg.table_stride > ((int64_t)1 << 30) / page)
        return fail(KVBFP_ERR_UNSUPPORTED, "paged cache: more than 2^30 tokens per sequence");
    *logical = *pool;
    logical->batch = pg.batch;
    logical->max_seq = pg.table_stride * page;
    return KVBFP_OK;
}

SplitPlan plan_splits(const kvbfp_layout* L, int32_t n_q_heads, int64_t max_len) {
    // Enough workgroups to fill 256 compute units with as many as are resident per unit - three, or two
    // of the sixteen-head variant of the LDS pipeline (4-bit mantissas, blocks of 16/32, more than 8 heads
    // per kv-head) and of the passes for 8-bit mantissas - but no more splits than there are 256-token
    // tiles: the tiles are dealt out round-robin over the splits.
    const int64_t units = (int64_t)L->batch * L->n_kv_heads;
    const int64_t tiles = (max_len + kTokenTile - 1) / kTokenTile;
    const bool sixteen = L->mant_bits == 4 && L->block <= 32 && n_q_heads / L->n_kv_heads > 8;
    const bool two_per_cu = sixteen || L->mant_bits == 8;      // 8-bit mantissas: twice the staging area per workgroup
    const int64_t target_wgs = 256 * (two_per_cu ? 2 : 3);
    int64_t want = (target_wgs + units - 1) / units;
    if (want > tiles) want = tiles;
    if (want < 1) want = 1;
    SplitPlan p;
    p.n_splits = (int32_t)want;
    return p;
}

// ---- element widening on the host (exact) ------------------------------------------------
static inline float bits_to_float(uint32_t u) {
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}
static inline float widen_bf16(uint16_t h) { return bits_to_float((uint32_t)h << 16); }
static inline float widen_f16(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t ex = (h >> 10) & 0x1Fu;
    const uint32_t fr = h & 0x3FFu;
    if (ex == 0x1F) return bits_to_float(sign | 0x7F800000u | (fr << 13));
    if (ex != 0) return bits_to_float(sign | ((ex + 112u) << 23) | (fr << 13));
    // zero or subnormal: fr * 2^-24
    const float mag = std::ldexp((float)fr, -24);
    return (sign ? -mag : mag);
}
static inline double load_elem(const void* base, int dtype, int64_t idx) {
    switch (dtype) {
        case KVBFP_F32: return (double)((const float*)base)[idx];
        case KVBFP_F16: return (double)widen_f16(((const uint16_t*)base)[idx]);
        default: return (double)widen_bf16(((const uint16_t*)base)[idx]);
    }
}

}  // namespace kvbfp

using namespace kvbfp;

extern "C" {

const char* kvbfp_last_error(void) { return g_err; }
const char* kvbfp_version(void) { return "kvbfp 0.1 (gfx950)"; }

int kvbfp_cache_bytes(const kvbfp_layout* L, size_t* mant_bytes, size_t* exp_bytes) {
    clear_error();
    if (!L || L->struct_bytes != sizeof(kvbfp_layout)) return fail(KVBFP_ERR_INVALID_ARG, "bad layout");
    if (L->batch <= 0 || L->n_kv_heads <= 0 || L->max_seq <= 0 || L->head_dim <= 0 || L->block <= 0 ||
        L->head_dim % L->block != 0 || !(L->mant_bits == 4 || L->mant_bits == 8) ||
        (L->head_dim * L->mant_bits) % 8 != 0)
        return fail(KVBFP_ERR_INVALID_ARG, "bad layout geometry");
    const size_t rows = (size_t)L->batch * (size_t)L->n_kv_heads * (size_t)L->max_seq;
    if (mant_bytes) *mant_bytes = rows * (size_t)(L->head_dim * L->mant_bits / 8);
    if (exp_bytes) *exp_bytes = rows * (size_t)(L->head_dim / L->block);
    return KVBFP_OK;
}

int kvbfp_calibrate_perm(const void* x, kvbfp_dtype dtype, int64_t n_samples, int32_t n_heads,
                         int32_t head_dim, int64_t sample_stride, int64_t head_stride,
                         int64_t chan_stride, kvbfp_stat stat, int32_t descending,
                         int32_t* perm_out) {
    clear_error();
    if (!x || !perm_out) return fail(KVBFP_ERR_INVALID_ARG, "calibrate_perm: NULL pointer");
    if (n_samples <= 0 || n_heads <= 0 || head_dim <= 0)
        return fail(KVBFP_ERR_INVALID_ARG, "calibrate_perm: sizes must be positive");
    if (dtype_size(dtype) == 0) return fail(KVBFP_ERR_INVALID_ARG, "calibrate_perm: unknown dtype %d", (int)dtype);
    if (stat != KVBFP_STAT_MAXABS && stat != KVBFP_STAT_L2)
        return fail(KVBFP_ERR_INVALID_ARG, "calibrate_perm: unknown statistic %d", (int)stat);

    // (statistic, channel) pairs ordered by statistic, then channel: ties resolve to the lower
    // channel index in both directions.
    std::vector<std::pair<double, int32_t>> ranked((size_t)head_dim);
    for (int32_t h = 0; h < n_heads; ++h) {
        for (int32_t c = 0; c < head_dim; ++c) {
            const int64_t base = (int64_t)h * head_stride + (int64_t)c * chan_stride;
            double st = 0.0;
            if (stat == KVBFP_STAT_MAXABS) {
                for (int64_t s = 0; s < n_samples; ++s) {
                    const double a = std::fabs(load_elem(x, dtype, base + s * sample_stride));
                    if (a > st) st = a;
                }
            } else {
                for (int64_t s = 0; s < n_samples; ++s) {
                    const double v = load_elem(x, dtype, base + s * sample_stride);
                    st += v * v;
                }
            }
            ranked[(size_t)c] = {st, c};
        }
        if (descending) {
            std::sort(ranked.begin(), ranked.end(), [](const auto& a, const auto& b) {
                return a.first > b.first || (a.first == b.first && a.second < b.second);
            });
        } else {
            std::sort(ranked.begin(), ranked.end(), [](const auto& a, const auto& b) {
                return a.first < b.first || (a.first == b.first && a.second < b.second);
            });
        }
        for (int32_t j = 0; j < head_dim; ++j) perm_out[(int64_t)h * head_dim + j] = ranked[(size_t)j].second;
    }
    return KVBFP_OK;
}

int kvbfp_permute_weights(const void* w_in, void* w_out, kvbfp_dtype dtype, int32_t n_heads,
                          int32_t head_dim, int64_t row_len, int32_t heads_per_perm,
                          const int32_t* perm) {
    clear_error();
    if (!w_in || !w_out || !perm) return fail(KVBFP_ERR_INVALID_ARG, "permute_weights: NULL pointer");
    const int esz = dtype_size(dtype);
    if (esz == 0) return fail(KVBFP_ERR_INVALID_ARG, "permute_weights: unknown dtype %d", (int)dtype);
    if (n_heads <= 0 || head_dim <= 0 || row_len <= 0 || heads_per_perm <= 0)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_weights: sizes must be positive");
    if (n_heads % heads_per_perm != 0)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_weights: n_heads %d not divisible by heads_per_perm %d",
                    n_heads, heads_per_perm);
    const size_t row_bytes = (size_t)row_len * (size_t)esz;
    const size_t total = (size_t)n_heads * (size_t)head_dim * row_bytes;
    const char* a = (const char*)w_in;
    char* b = (char*)w_out;
    if (!(a + total <= b || b + total <= a))
        return fail(KVBFP_ERR_INVALID_ARG, "permute_weights: w_in and w_out overlap");
    const int32_t n_perms = n_heads / heads_per_perm;
    std::vector<uint8_t> seen((size_t)head_dim);
    for (int32_t g = 0; g < n_perms; ++g) {
        std::fill(seen.begin(), seen.end(), 0);
        for (int32_t j = 0; j < head_dim; ++j) {
            const int32_t c = perm[(int64_t)g * head_dim + j];
            if (c < 0 || c >= head_dim || seen[(size_t)c])
                return fail(KVBFP_ERR_INVALID_ARG, "permute_weights: perm row %d is not a permutation", g);
            seen[(size_t)c] = 1;
        }
    }
    for (int32_t h = 0; h < n_heads; ++h) {
        const int32_t* pi = perm + (int64_t)(h / heads_per_perm) * head_dim;
        const size_t head_off = (size_t)h * (size_t)head_dim * row_bytes;
        for (int32_t j = 0; j < head_dim; ++j)
            std::memcpy(b + head_off + (size_t)j * row_bytes, a + head_off + (size_t)pi[j] * row_bytes, row_bytes);
    }
    return KVBFP_OK;
}

int kvbfp_permute_weight_columns(const void* w_in, void* w_out, kvbfp_dtype dtype, int64_t n_rows,
                                 int32_t n_heads, int32_t head_dim, int32_t heads_per_perm,
                                 const int32_t* perm) {
    clear_error();
    if (!w_in || !w_out || !perm) return fail(KVBFP_ERR_INVALID_ARG, "permute_weight_columns: NULL pointer");
    const int esz = dtype_size(dtype);
    if (esz == 0) return fail(KVBFP_ERR_INVALID_ARG, "permute_weight_columns: unknown dtype %d", (int)dtype);
    if (n_rows <= 0 || n_heads <= 0 || head_dim <= 0 || heads_per_perm <= 0)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_weight_columns: sizes must be positive");
    if (n_heads % heads_per_perm != 0)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_weight_columns: n_heads %d not divisible by heads_per_perm %d",
                    n_heads, heads_per_perm);
    const size_t row_bytes = (size_t)n_heads * (size_t)head_dim * (size_t)esz;
    const size_t total = (size_t)n_rows * row_bytes;
    const char* a = (const char*)w_in;
    char* b = (char*)w_out;
    if (!(a + total <= b || b + total <= a))
        return fail(KVBFP_ERR_INVALID_ARG, "permute_weight_columns: w_in and w_out overlap");
    const int32_t n_perms = n_heads / heads_per_perm;
    std::vector<uint8_t> seen((size_t)head_dim);
    for (int32_t g = 0; g < n_perms; ++g) {
        std::fill(seen.begin(), seen.end(), 0);
        for (int32_t j = 0; j < head_dim; ++j) {
            const int32_t c = perm[(int64_t)g * head_dim + j];
            if (c < 0 || c >= head_dim || seen[(size_t)c])
                return fail(KVBFP_ERR_INVALID_ARG, "permute_weight_columns: perm row %d is not a permutation", g);
            seen[(size_t)c] = 1;
        }
    }
    for (int64_t r = 0; r < n_rows; ++r) {
        const char* src = a + (size_t)r * row_bytes;
        char* dst = b + (size_t)r * row_bytes;
        for (int32_t h = 0; h < n_heads; ++h) {
            const int32_t* pi = perm + (int64_t)(h / heads_per_perm) * head_dim;
            const size_t head_off = (size_t)h * (size_t)head_dim * (size_t)esz;
            for (int32_t j = 0; j < head_dim; ++j)
                std::memcpy(dst + head_off + (size_t)j * (size_t)esz, src + head_off + (size_t)pi[j] * (size_t)esz,
                            (size_t)esz);
        }
    }
    return KVBFP_OK;
}

int kvbfp_permute_rope(const float* theta, kvbfp_rope_pairs pairs, int32_t n_heads, int32_t head_dim,
                       const int32_t* perm, float* theta_out, int32_t* partner_out, float* sign_out) {
    clear_error();
    if (!theta || !perm || !theta_out || !partner_out || !sign_out)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_rope: NULL pointer");
    if (n_heads <= 0 || head_dim <= 0 || head_dim % 2 != 0)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_rope: n_heads %d, head_dim %d (positive, head_dim even)", n_heads,
                    head_dim);
    if (pairs != KVBFP_ROPE_PAIRS_ADJACENT && pairs != KVBFP_ROPE_PAIRS_HALF_SPLIT)
        return fail(KVBFP_ERR_INVALID_ARG, "permute_rope: unknown pair layout %d", (int)pairs);
    const int32_t half = head_dim / 2;
    // channel c rotates in plane pair_of(c) as its first (sine sign -1) or second (+1) coordinate
    auto pair_of = [&](int32_t c) { return pairs == KVBFP_ROPE_PAIRS_ADJACENT ? c >> 1 : (c < half ? c : c - half); };
    auto is_first = [&](int32_t c) { return pairs == KVBFP_ROPE_PAIRS_ADJACENT ? (c & 1) == 0 : c < half; };
    std::vector<int32_t> where((size_t)head_dim);       // where[c] = position of original channel c in the reordered row
    for (int32_t h = 0; h < n_heads; ++h) {
        const int32_t* pi = perm + (int64_t)h * head_dim;
        std::fill(where.begin(), where.end(), -1);
        for (int32_t j = 0; j < head_dim; ++j) {
            if (pi[j] < 0 || pi[j] >= head_dim || where[(size_t)pi[j]] >= 0)
                return fail(KVBFP_ERR_INVALID_ARG, "permute_rope: perm row %d is not a permutation", h);
            where[(size_t)pi[j]] = j;
        }
        for (int32_t j = 0; j < head_dim; ++j) {
            const int32_t c = pi[j], plane = pair_of(c);
            const bool first = is_first(c);
            int32_t mate;                                // the other coordinate of the plane, original numbering
            if (pairs == KVBFP_ROPE_PAIRS_ADJACENT) mate = first ? c + 1 : c - 1;
            else mate = first ? c + half : c - half;
            const int64_t o = (int64_t)h * head_dim + j;
            theta_out[o] = theta[plane];
            sign_out[o] = first ? -1.0f : 1.0f;
            partner_out[o] = where[(size_t)mate];
        }
    }
    return KVBFP_OK;
}

}  // extern "C"
