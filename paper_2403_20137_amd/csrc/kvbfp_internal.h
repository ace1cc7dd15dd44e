// Internal helpers of libkvbfp (not part of the C ABI): error reporting and argument checks.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "kvbfp.h"

namespace kvbfp {

// Records a printf-style message for kvbfp_last_error() and returns `code`.
int fail(int code, const char* fmt, ...);
void clear_error();

inline int dtype_size(int dtype) {
    switch (dtype) {
        case KVBFP_F32: return 4;
        case KVBFP_F16: return 2;
        case KVBFP_BF16: return 2;
        default: return 0;
    }
}

// Checks the layout for the device kernels; returns KVBFP_OK or records an error.
int check_device_layout(const kvbfp_layout* L);
int check_cache(const kvbfp_cache* c, bool need_k, bool need_v);

// Number of splits (partial results per query head) decode attention uses for this geometry.
struct SplitPlan {
    int32_t n_splits;
};
constexpr int kTokenTile = 256;
SplitPlan plan_splits(const kvbfp_layout* L, int32_t n_q_heads, int64_t max_len);

// A paged cache: `pool` describes the pool of pages (batch = pages, max_seq = tokens per page, a power of
// two and at least kPageMin: the 16 tokens of a stage of the decode kernels never straddle two pages);
// sequence b keeps tokens [i page, (i+1) page) in page block_table[b * table_stride + i].
constexpr int kPageMin = 16;
struct Paging {
    const int32_t* block_table;   // DEVICE int32 [batch][table_stride]
    int64_t table_stride;
    int32_t batch;                // sequences
};
// Validates pool and paging; on success *logical is the layout the sequences appear to have
// (batch sequences of table_stride pages each).
int check_paging(const kvbfp_layout* pool, const Paging& pg, kvbfp_layout* logical);

// kvbfp_quantize_append, optionally with sequence lengths in place of positions (len_cap >= 0, see
// quantize.hip) and optionally into a paged cache (L is then the pool); does not clear the error state.
int quantize_append_impl(const kvbfp_layout* L, const kvbfp_cache* cache, const void* k_new,
                         const void* v_new, kvbfp_dtype dtype, int32_t n_new, int64_t stride_b,
                         int64_t stride_t, int64_t stride_h, int64_t pos0, const int32_t* pos_dev,
                         int64_t len_cap, const int32_t* perm_k, const int32_t* perm_v, void* hip_stream,
                         const Paging* paging = nullptr);

}  // namespace kvbfp
