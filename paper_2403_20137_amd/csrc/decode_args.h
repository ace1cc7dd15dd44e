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
    int64_t max_seq, max_len, split_len;
    int32_t H_kv, H_q, G, n_splits, log2_block;
    // Appending the current token inside the split pass (kvbfp_append_decode_attention): the new key
    // and value row of (batch b, kv-head h) at k_new/v_new + b * new_stride_b + h * new_stride_h
    // (elements of the call's dtype); nullptr = nothing to append.
    const void* k_new;
    const void* v_new;
    int64_t new_stride_b, new_stride_h;
    int32_t q_mant_bits;      // 0, or the mantissa bits the permuted query is cast to (block = cache block)
    float scale_log2e;
};

// Fast split pass for 4-bit mantissas and 16-bit I/O (decode_mfma.hip).  Returns hipSuccess after
// enqueuing; the caller has already validated the arguments.  group size G <= 8.
hipError_t launch_decode_split_mfma(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s);
// The same for 8-bit mantissas (decode_mfma_p8.hip).
hipError_t launch_decode_split_mfma_p8(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s);

}  // namespace kvbfp
