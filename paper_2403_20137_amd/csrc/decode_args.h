// Kernel argument block shared by the decode-attention kernels (internal, not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace kvbfp {

struct DecodeArgs {
    const uint8_t* k_mant;
    const uint8_t* k_exp;
    const uint8_t* v_mant;
    const uint8_t* v_exp;
    const void* q;
    void* out;
    const int32_t* seq_len;   // [B] or nullptr
    const int32_t* perm_k;    // [H_kv][D] or nullptr
    const int32_t* perm_v;
    float* part_ml;           // [B][H_q][n_splits][2]  (m in base-2 units, l)
    float* part_o;            // [B][H_q][n_splits][D]
    int64_t max_seq, max_len;
    // Work division: the sequence is cut into 256-token tiles and split s (blockIdx.x) takes tiles
    // s, s + n_splits, s + 2 n_splits, ...; each split leaves one partial result for the combine pass.
    // With several query tokens per sequence (kvbfp_decode_attention_multi) the kernels see "virtual
    // heads": H_q = n_q_tokens * real_Hq per batch and G = n_q_tokens * real_G per kv-head; virtual head
    // s of a kv-head is query token s / real_G, real head kvh * real_G + s % real_G, and may attend
    // to n_q_tokens - 1 - s / real_G tokens fewer than the sequence holds (causal order of the new tokens).
    int32_t H_kv, H_q, G, n_splits, log2_block;
    int32_t n_q_tokens, real_Hq, real_G;
    int32_t g_base, g_cnt;    // matrix-core passes: this launch serves virtual heads [g_base, g_base + g_cnt) of every kv-head;
                              // g_cnt <= 8, or <= 16 in the LDS pipeline (4-bit mantissas, blocks of 16/32, 16-bit I/O)
    // Appending the current token inside the split pass (kvbfp_append_decode_attention): the new key
    // and value row of (batch b, kv-head h) at k_new/v_new + b * new_stride_b + h * new_stride_h
    // (elements of the call's dtype); nullptr = nothing to append.
    const void* k_new;
    const void* v_new;
    int64_t new_stride_b, new_stride_h;
    int32_t q_mant_bits;      // 0, or the mantissa bits the permuted query is cast to (block = cache block)
    float scale_log2e;
    // Keys cached before the rotary embedding (kvbfp_decode_attention_rope): the reordered frequency,
    // partner-position and sign vectors of Alg. 1 step 5, each [H_kv][D]; nullptr = no rotation at read.
    const float* rope_theta;
    const int32_t* rope_partner;
    const float* rope_sign;
    // Paged cache (kvbfp_decode_attention_paged): the planes are a pool [n_pages][H_kv][2^log2_page][..]
    // and tokens [i 2^log2_page, (i+1) 2^log2_page) of sequence b live in page
    // block_table[b * table_stride + i]; nullptr = one contiguous region of max_seq tokens per sequence.
    // A page holds 16 tokens or a power of two above: a 64-token tile of a wavefront may span up to four pages,
    // one per 16-token stage (StageBases below).
    const int32_t* block_table;
    int64_t table_stride;
    int32_t log2_page, n_pages;
};

// Row index (one row = one token of one kv-head) of token t of sequence b in the four planes.  Page
// numbers come from device memory the host cannot check: they are clamped to the pool.
__device__ inline int64_t cache_row(const DecodeArgs& a, int b, int kvh, int64_t t) {
    if (!a.block_table) return ((int64_t)b * a.H_kv + kvh) * a.max_seq + t;
    int page = a.block_table[(int64_t)b * a.table_stride + (t >> a.log2_page)];
    page = page < 0 ? 0 : (page >= a.n_pages ? a.n_pages - 1 : page);
    return (((int64_t)page * a.H_kv + kvh) << a.log2_page) + (t & (((int64_t)1 << a.log2_page) - 1));
}

// Paged caches: the rows of a 64-token tile that starts at token t_tile (a multiple of 64) of sequence b, one
// additive base per 16-token stage: token t of stage u lies in plane row v[u] + t.  t_end = cached tokens
// (> t_tile).  A stage that starts at or beyond t_end takes the base of the stage that holds the last cached
// token, so that a token index clamped to t_end - 1 can be added to the base of the stage that asks.
struct StageBases { int64_t v[4]; };
__device__ inline StageBases stage_bases(const DecodeArgs& a, int b, int kvh, int64_t t_tile, int64_t t_end) {
    StageBases s;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        int64_t t = t_tile + 16 * u;
        if (t >= t_end) t = (t_end - 1) & ~(int64_t)15;
        s.v[u] = cache_row(a, b, kvh, t) - t;
    }
    return s;
}
// v[st] for a per-lane stage index (compares and selects, no indexed register access)
__device__ inline int64_t stage_base_of(const StageBases& s, int st) {
    const int64_t lo = (st & 1) ? s.v[1] : s.v[0], hi = (st & 1) ? s.v[3] : s.v[2];
    return (st & 2) ? hi : lo;
}

// Row of q / out, in units of head_dim elements, of virtual head s of kv-head kvh in batch b.
__host__ __device__ inline int64_t query_row(const DecodeArgs& a, int b, int kvh, int s) {
    return ((int64_t)b * a.n_q_tokens + s / a.real_G) * a.real_Hq + (int64_t)kvh * a.real_G + s % a.real_G;
}
// Tokens at the end of the sequence that virtual head s must not see.
__host__ __device__ inline int hidden_tokens(const DecodeArgs& a, int s) {
    const int o = a.n_q_tokens - 1 - s / a.real_G;
    return o > 0 ? o : 0;
}

// Matrix-core split pass for 4-bit mantissas (decode_mfma.hip).  Returns hipSuccess after
// enqueuing; the caller has already validated the arguments.
hipError_t launch_decode_split_mfma(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s);
// (a.g_cnt <= 8 heads per launch, 16 where the LDS pipeline applies; larger groups take several launches over
// head subsets.)
// The same for 8-bit mantissas (decode_mfma_p8.hip: the LDS pipeline for 16-bit I/O, the register-staged pass
// for fp32 I/O; a.g_cnt <= 8).
hipError_t launch_decode_split_mfma_p8(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s);
// Rotation at read on the matrix cores (decode_rope.hip): 4-bit mantissas, 16-bit I/O, a.g_cnt <= 4.
hipError_t launch_decode_split_rope(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s);

}  // namespace kvbfp
