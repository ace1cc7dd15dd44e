/* kvbfp -- Block-Floating-Point KV cache with offline channel reordering, for AMD MI355X (gfx950).
 *
 * C ABI of libkvbfp.so.  The operations follow "Accurate Block Quantization in LLMs with
 * Outliers" (Trukhanov & Soloveychik): a per-head channel permutation fixed before inference
 * (K-sort, Alg. 1) makes outlier channels share blocks; key/value rows are then stored in a
 * Block Floating Point format (Sec. II-B, Eq. (1)) and attention reads that packed cache
 * directly (Sec. III, run-time flow).
 *
 * General conventions
 *   - "HOST" pointers are ordinary host memory; "DEVICE" pointers are HIP device memory on the
 *     current device.  The library never allocates or frees device memory, keeps no state
 *     between calls and owns none of the buffers passed in.
 *   - Device calls only enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising.
 *   - Every call returns a kvbfp_status.  Everything that can be checked on the host is checked
 *     before anything is launched; kvbfp_last_error() then describes the problem.  Values held in
 *     device memory (positions, sequence lengths) cannot be checked: kernels clamp them so that
 *     all accesses stay inside the cache, and the result is then unspecified.  The same holds for
 *     permutations held in device memory: every entry is reduced modulo head_dim before it is used as
 *     an index (a valid permutation is unchanged; anything else is memory-safe, result unspecified).
 *   - Alignment: the two mantissa planes of a cache must be 16-byte aligned (INVALID_ARG otherwise);
 *     exponent planes may sit at any address (attention then takes its general pass).
 *   - Non-finite inputs (NaN, Inf) are outside the contract: memory-safe, value unspecified.
 *
 * BFP format (Sec. II-B, Eq. (1)): a block is `block` consecutive cache positions of one row.
 * It stores one exponent byte E and `block` mantissa codes of `mant_bits` bits (sign-magnitude:
 * top bit sign, rest magnitude |M| <= 2^(mant_bits-1)-1, zero always stored with sign 0).
 * Decoded value = (-1)^sign * |M| * 2^(E - 127 - (mant_bits - 2)).  E = 0 marks an all-zero
 * block.  The cast picks the smallest E for which round-to-nearest-even of the block's largest
 * magnitude still fits the mantissa range and rounds every element to nearest-even at that scale,
 * so every element is within half a mantissa step of its input.
 *
 * Packed cache (per layer): four planes, token-major inside each (batch, kv-head):
 *     k_mant, v_mant : uint8 [batch][n_kv_heads][max_seq][head_dim * mant_bits / 8]
 *     k_exp,  v_exp  : uint8 [batch][n_kv_heads][max_seq][head_dim / block]
 * Position j of a row holds (permuted) channel j.  mant_bits = 8: byte j is code j.
 * mant_bits = 4: byte i holds code 2i in its low nibble and code 2i+1 in its high nibble.
 * Exponent byte b of a row belongs to positions [b*block, (b+1)*block).
 * Storage is mant_bits + 8/block bits per element (BFP12 with block 32: 4.25 bits).
 */
#ifndef KVBFP_H
#define KVBFP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KVBFP_OK = 0,
    KVBFP_ERR_INVALID_ARG = -1,   /* NULL where not allowed, inconsistent sizes, not a permutation */
    KVBFP_ERR_UNSUPPORTED = -2,   /* valid in principle, not implemented (e.g. head_dim != 128 on device) */
    KVBFP_ERR_WORKSPACE = -3,     /* workspace missing or too small */
    KVBFP_ERR_HIP = -4            /* a HIP runtime call or kernel launch failed */
} kvbfp_status;

typedef enum { KVBFP_F32 = 0, KVBFP_F16 = 1, KVBFP_BF16 = 2 } kvbfp_dtype;

/* Channel statistic used to rank channels (Alg. 1 step 1 and its calibration-data variant). */
typedef enum {
    KVBFP_STAT_MAXABS = 0,        /* max over samples of |x|: calibration key/value rows            */
    KVBFP_STAT_L2 = 1             /* Euclidean norm over samples: rows of W_k, as Alg. 1 states it   */
} kvbfp_stat;

/* Geometry of one layer's packed cache.  Plain data, filled by the caller.
 * struct_bytes must be sizeof(kvbfp_layout).  Device calls need head_dim == 128,
 * block in {16,32,64,128}, mant_bits in {4,8}. */
typedef struct {
    uint32_t struct_bytes;
    int32_t head_dim;
    int32_t block;
    int32_t mant_bits;
    int32_t n_kv_heads;
    int32_t batch;
    int64_t max_seq;
} kvbfp_layout;

/* DEVICE pointers to the four planes described above; caller-owned. */
typedef struct {
    uint8_t* k_mant;
    uint8_t* k_exp;
    uint8_t* v_mant;
    uint8_t* v_exp;
} kvbfp_cache;

/* Size in bytes of one mantissa plane and of one exponent plane for `layout`. */
int kvbfp_cache_bytes(const kvbfp_layout* layout, size_t* mant_bytes_per_plane,
                      size_t* exp_bytes_per_plane);

/* HOST.  Alg. 1 steps 1-2: per head, a statistic per channel and a stable argsort of it.
 *   x        : HOST, element (sample s, head h, channel c) at
 *              x[s*sample_stride + h*head_stride + c*chan_stride] (strides in elements).
 *              Calibration rows: samples are tokens.  Alg. 1 proper: x = W_k, samples are the
 *              input features of a weight row, channels are the rows (stat = KVBFP_STAT_L2).
 *   perm_out : HOST int32 [n_heads][head_dim]; perm_out[h][j] = channel placed at position j,
 *              i.e. permuted[j] = original[perm[j]].  Ascending statistic unless `descending`
 *              (Sec. III allows either); equal statistics keep ascending channel order.
 * The L2 statistic is compared through the sum of squares accumulated in double in sample order.
 * Errors: INVALID_ARG for NULL pointers, non-positive sizes, unknown dtype/stat. */
int kvbfp_calibrate_perm(const void* x, kvbfp_dtype dtype, int64_t n_samples, int32_t n_heads,
                         int32_t head_dim, int64_t sample_stride, int64_t head_stride,
                         int64_t chan_stride, kvbfp_stat stat, int32_t descending,
                         int32_t* perm_out);

/* HOST.  Alg. 1 steps 3-4 (and the value-side analogue of Sec. III): reorder weight rows.
 *   w_in, w_out : HOST [n_heads*head_dim][row_len] row-major, same dtype, must not overlap.
 *   out row (h, j) = in row (h, perm[h / heads_per_perm][j]).
 *   heads_per_perm: 1 for W_k / W_v; the group size for W_q when several query heads share a
 *   KV head.  perm: HOST int32 [n_heads / heads_per_perm][head_dim].
 * By Eq. (2)-(3) the products q.k^T are unchanged when W_q and W_k get the same permutation.
 * Errors: INVALID_ARG for NULL, overlap, n_heads not divisible, perm rows that are not
 * permutations of 0..head_dim-1. */
int kvbfp_permute_weights(const void* w_in, void* w_out, kvbfp_dtype dtype, int32_t n_heads,
                          int32_t head_dim, int64_t row_len, int32_t heads_per_perm,
                          const int32_t* perm);

/* HOST.  Sec. III, last paragraph: the projection that consumes the attention output has its COLUMNS
 * reordered to match the value permutation, so that the output can stay in cache order.
 *   w_in, w_out : HOST [n_rows][n_heads*head_dim] row-major, same dtype, must not overlap (W_o: n_rows =
 *   model width, n_heads = query heads).
 *   out column (h, j) = in column (h, perm[h / heads_per_perm][j]);  perm as in kvbfp_permute_weights.
 * With W_v's rows reordered by the same permutation, w_out . (reordered attention output) equals
 * w_in . (attention output in the original order): nothing is gathered or scattered at run time.
 * Errors: as kvbfp_permute_weights. */
int kvbfp_permute_weight_columns(const void* w_in, void* w_out, kvbfp_dtype dtype, int64_t n_rows,
                                 int32_t n_heads, int32_t head_dim, int32_t heads_per_perm,
                                 const int32_t* perm);

/* DEVICE, asynchronous.  Cast new key/value rows to BFP (Sec. II-B) and store them in the cache
 * (Sec. III: the keys of each head are kept in block format; values likewise).
 *   k_new, v_new : DEVICE [batch][n_new][n_kv_heads][head_dim] of `dtype`, channel stride 1,
 *                  element strides stride_b / stride_t / stride_h; either may be NULL (skipped).
 *   Token i of sequence b goes to position pos0 + i (pos_dev == NULL) or pos_dev[b] + i
 *   (pos_dev: DEVICE int32 [batch]); rows that would fall outside [0, max_seq) are dropped.
 *   perm_k, perm_v : DEVICE int32 [n_kv_heads][head_dim] or NULL.  NULL means the rows already
 *                  arrive in cache channel order (the permutation lives in the weights, Sec. II-C);
 *                  otherwise position j of the stored row is input channel perm[h][j].
 * Errors: INVALID_ARG (NULL layout/cache planes needed, n_new < 0, pos0 + n_new > max_seq when
 * pos_dev is NULL, bad dtype), UNSUPPORTED (geometry), HIP. */
int kvbfp_quantize_append(const kvbfp_layout* layout, const kvbfp_cache* cache, const void* k_new,
                          const void* v_new, kvbfp_dtype dtype, int32_t n_new, int64_t stride_b,
                          int64_t stride_t, int64_t stride_h, int64_t pos0, const int32_t* pos_dev,
                          const int32_t* perm_k, const int32_t* perm_v, void* hip_stream);

/* DEVICE, asynchronous.  Eq. (1): decode cached rows back to numbers.
 *   which : 0 = keys, 1 = values.  Tokens [t0, t0 + n_tok) of every (batch, kv-head).
 *   out   : DEVICE [batch][n_tok][n_kv_heads][head_dim] of `dtype`, dense.
 *   perm  : DEVICE int32 [n_kv_heads][head_dim] or NULL.  NULL leaves cache (permuted) order;
 *           otherwise out[perm[h][j]] = value at cache position j (original channel order).
 *           `out` must be 16-byte aligned.
 *           A perm that is not a permutation is memory-safe (entries are masked to the row); the output
 *           channels it does not reach are then unspecified.
 * fp32 output is exact; fp16/bf16 output is the IEEE round-to-nearest-even conversion.
 * Errors: INVALID_ARG (NULL, range outside [0, max_seq], bad which/dtype, `out` not 16-byte aligned),
 * UNSUPPORTED (also: batch * n_kv_heads * n_tok above 2^31 - 1 in one call), HIP. */
int kvbfp_dequantize(const kvbfp_layout* layout, const kvbfp_cache* cache, int32_t which,
                     int64_t t0, int64_t n_tok, const int32_t* perm, void* out, kvbfp_dtype dtype,
                     void* hip_stream);

/* Bytes of DEVICE workspace kvbfp_decode_attention needs for up to max_len cached tokens
 * (partial results of the sequence splits).  Returns 0 on invalid arguments. */
size_t kvbfp_decode_workspace_bytes(const kvbfp_layout* layout, int32_t n_q_heads, int64_t max_len);

/* DEVICE, asynchronous.  One decode step of attention over the packed cache (Sec. III: the cached
 * keys are read back and multiplied with the permuted query; the rest is ordinary softmax
 * attention; values are handled the same way and the output is brought back to the original
 * channel order, which stands in for permuting the columns of the following projection).
 *   q, out      : DEVICE [batch][n_q_heads][head_dim] of `dtype`, contiguous.
 *                 n_q_heads % n_kv_heads == 0; query head h reads KV head h / (n_q_heads/n_kv_heads).
 *   seq_len_dev : DEVICE int32 [batch] cached tokens per sequence, or NULL = max_len for all.
 *                 Values are clamped to [0, max_len].  A sequence with 0 tokens yields zeros.
 *   max_len     : host-known upper bound of the sequence lengths (<= max_seq); sizes the grid.
 *   out[b][h] = softmax_t(softmax_scale * q'[b][h] . K^[b][g][t]) . V^[b][g][t], all cached tokens
 *   attended (no mask), with q'[j] = q[perm_k[g][j]] and the result scattered as
 *   out[perm_v[g][j]] = o[j]; a NULL perm means identity.
 *   workspace   : DEVICE, at least kvbfp_decode_workspace_bytes(layout, n_q_heads, max_len) bytes,
 *                 256-byte aligned; contents are scratch.
 * Accumulation is fp32; the output is rounded once to `dtype`.
 * Range: up to 32 query heads per kv-head the products run on the matrix cores, whose 16-bit operand
 * format holds every cached block with an exponent byte from 3 to 254 (4-bit mantissas) or 3 to 251
 * (8-bit mantissas) exactly, i.e. magnitudes from 2^-126 to 2^124.  Blocks with exponent byte 1 or 2
 * (every magnitude below 2^-124) lose low-order bits there, an absolute error under 2^-126 per element;
 * blocks above the upper end are not supported there.  The scaled query q * softmax_scale * log2(e) must
 * stay between 2^-100 and 2^100 in magnitude wherever it matters to the scores.  Wider groups, and exponent
 * planes that are not 16-byte aligned, take the general pass (fp32 multiply-adds), which has no such limits
 * beyond those of fp32 itself.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
int kvbfp_decode_attention(const kvbfp_layout* layout, const kvbfp_cache* cache, int32_t n_q_heads,
                           const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                           int64_t max_len, float softmax_scale, const int32_t* perm_k,
                           const int32_t* perm_v, void* out, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/* DEVICE, asynchronous.  kvbfp_decode_attention with the query in Block Floating Point as well
 * (Sec. III and Sec. IV: the activations entering the score product are BFP too, 8-bit mantissas in
 * the paper's experiments).  The permuted query q' of every head is cast exactly like a cached row
 * (Eq. (1); blocks of layout->block channels, q_mant_bits-bit sign-magnitude mantissas, shared
 * exponent from the block's largest magnitude, round to nearest even) before softmax_scale is
 * applied, so each block's contribution to a score is an integer dot product of mantissas times a
 * power of two.  The cast happens inside the kernel; q in memory is not modified.
 *   q_mant_bits : 8 or 4; 0 behaves exactly like kvbfp_decode_attention.
 * All other arguments, the workspace size and the error behaviour are those of
 * kvbfp_decode_attention; a q_mant_bits outside {0, 4, 8} is INVALID_ARG.
 * 8-bit mantissas in blocks of 32 or wider with q_mant_bits = 8 and fp16/bf16 I/O: the scores are integer
 * matrix products of the query's and the keys' codes, one 32-bit sum per 32 channels, scaled once by the sum
 * of the two block exponents (Sec. II-B); every block's partial score is exact. */
int kvbfp_decode_attention_qbfp(const kvbfp_layout* layout, const kvbfp_cache* cache,
                                int32_t n_q_heads, const void* q, kvbfp_dtype dtype,
                                const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits,
                                void* out, void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/* DEVICE, asynchronous.  One decode step in one call: the current token's key and value rows are
 * cast to BFP and stored (Sec. II-B, Eq. (1), exactly as kvbfp_quantize_append does for one row per
 * sequence), then attention runs over the cache including that token (Sec. III), exactly as
 * kvbfp_decode_attention_qbfp does.  Same cache bytes and same output as the two calls one after the
 * other; where the fast split pass applies the cast happens inside it and a launch is saved.
 *   k_new, v_new : DEVICE, row of (batch b, kv-head h) at base + b*new_stride_b + h*new_stride_h
 *                  (strides in elements of `dtype`, >= 0), head_dim contiguous elements, original
 *                  channel order if perm_k/perm_v are given, cache order if they are NULL.
 *   seq_len_dev  : DEVICE int32 [batch], cached tokens per sequence INCLUDING the current one
 *                  (clamped to [0, max_len]); the current token is stored at position seq_len - 1.
 *                  NULL = max_len for all.  A sequence with seq_len 0 stores nothing and yields zeros.
 *   perm_k/perm_v: as in kvbfp_decode_attention; the same permutations order the new rows.
 * Everything else as kvbfp_decode_attention_qbfp (q_mant_bits 0 = query left as it is).
 * Errors: those of kvbfp_decode_attention_qbfp and kvbfp_quantize_append. */
int kvbfp_append_decode_attention(const kvbfp_layout* layout, const kvbfp_cache* cache,
                                  int32_t n_q_heads, const void* k_new, const void* v_new,
                                  int64_t new_stride_b, int64_t new_stride_h, const void* q,
                                  kvbfp_dtype dtype, const int32_t* seq_len_dev, int64_t max_len,
                                  float softmax_scale, const int32_t* perm_k, const int32_t* perm_v,
                                  int32_t q_mant_bits, void* out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);

/* DEVICE, asynchronous.  Attention for the last n_q_tokens tokens of every sequence at once
 * (verification of speculated tokens, a chunk of a prompt): the same products as in
 * kvbfp_decode_attention_qbfp (Sec. III), every cached row still read once.  The tokens are already in
 * the cache; query token i (0-based) of a sequence with seq_len cached tokens attends to the first
 * seq_len - (n_q_tokens - 1 - i) of them (causal order among the new tokens); a query token that
 * sees no cached token yields zeros.
 *   q, out      : DEVICE [batch][n_q_tokens][n_q_heads][head_dim] of `dtype`, contiguous.
 *   workspace   : at least kvbfp_decode_workspace_bytes(layout, n_q_heads * n_q_tokens, max_len) bytes.
 *   n_q_tokens  : 1..64.  With n_q_tokens * (n_q_heads / n_kv_heads) <= 8 the spare rows of the
 *                 matrix-core passes hold the extra tokens and the cost is that of one token; up to
 *                 32 the cache is read once per 16 (4-bit mantissas in blocks of 16/32 with 16-bit
 *                 I/O) or once per 8 (otherwise); more go through the general pass.
 * Everything else as kvbfp_decode_attention_qbfp.  n_q_tokens = 1 is that call. */
int kvbfp_decode_attention_multi(const kvbfp_layout* layout, const kvbfp_cache* cache,
                                 int32_t n_q_heads, int32_t n_q_tokens, const void* q,
                                 kvbfp_dtype dtype, const int32_t* seq_len_dev, int64_t max_len,
                                 float softmax_scale, const int32_t* perm_k, const int32_t* perm_v,
                                 int32_t q_mant_bits, void* out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/* Rotary embeddings under the reorder, parameter side (Sec. II-D; Alg. 1 step 5).  HOST.
 * In the original channel order a row x at token index m is rotated as
 *     (R x)[c] = x[c] cos(m Theta[c]) + s[c] x[i[c]] sin(m Theta[c])
 * where channels come in pairs that share one frequency: KVBFP_ROPE_PAIRS_ADJACENT pairs channels
 * (2k, 2k+1) (the ordering of Sec. II-D: Theta = [th_0, th_0, th_1, th_1, ..], i = [1, 0, 3, 2, ..],
 * s = [-1, +1, -1, +1, ..]); KVBFP_ROPE_PAIRS_HALF_SPLIT pairs (k, k + head_dim/2) (the ordering of the
 * open-source Llama code named in the footnote of Sec. III).  The call applies each head's
 * permutation to the three vectors, for rows that are stored in the reordered order:
 *     theta_out[h][j] = Theta[perm[h][j]],  sign_out[h][j] = s[perm[h][j]],
 *     partner_out[h][j] = the POSITION in the reordered row of channel i[perm[h][j]].
 *   theta : HOST float [head_dim/2];  perm : HOST int32 [n_heads][head_dim] (gather convention)
 *   theta_out, sign_out : HOST float [n_heads][head_dim];  partner_out : HOST int32 [n_heads][head_dim]
 * Errors: INVALID_ARG (NULL, odd head_dim, unknown layout, perm row not a permutation). */
typedef enum { KVBFP_ROPE_PAIRS_ADJACENT = 0, KVBFP_ROPE_PAIRS_HALF_SPLIT = 1 } kvbfp_rope_pairs;
int kvbfp_permute_rope(const float* theta, kvbfp_rope_pairs pairs, int32_t n_heads, int32_t head_dim,
                       const int32_t* perm, float* theta_out, int32_t* partner_out, float* sign_out);

/* Decode attention over keys that were cached BEFORE the rotary embedding (Sec. III: the keys are
 * fetched from the cache, the correctly ordered rotary embedding is applied, then the product with
 * pi(q) is taken; Alg. 1 step 5).  DEVICE, async unless kernel_ms is given.
 * As kvbfp_decode_attention, except that the key of token t of a sequence enters the score as
 *     k_rot[j] = k'[j] cos(t Theta'[j]) + s'[j] k'[i'[j]] sin(t Theta'[j])      (k' = the cached row)
 * with the token index t = its position in the cache and the angle t * Theta'[j] taken exactly (the
 * kernels start their sine/cosine phasors in double precision).  q is used as given: the caller rotates the
 * query at its own token index, in whatever order it keeps it (perm_k gathers it as usual).
 *   rope_theta, rope_sign : DEVICE float [n_kv_heads][head_dim];  rope_partner : DEVICE int32, same shape:
 *       what kvbfp_permute_rope returns for perm_k (identity permutation if the rows were never
 *       reordered).  The kernel relies on their structure: partner is an involution without fixed
 *       points, and a position and its partner have equal theta and opposite signs; other contents
 *       are memory-safe with an unspecified result.
 *   kernel_ms : HOST float[2] or NULL.  Non-NULL: the call waits for its kernels and returns the
 *       durations of the split pass and of the combine pass in milliseconds (HIP events).
 * One query token per sequence, query in its input type.  4-bit mantissas with fp16/bf16 I/O take a
 * matrix-core pass (the rotation is carried by the query operand per 64-token tile and by a table of
 * cos/sin per token offset; same bars as kvbfp_decode_attention, any exponent bytes 3..254, queries
 * and softmax_scale whose product stays finite in fp32); 8-bit mantissas and fp32 I/O take a vector-ALU
 * pass that is several times slower.  Either way the rotation costs arithmetic per cached key element
 * that the plain path does not have: about 2.3x the time of kvbfp_decode_attention on the same cache
 * (a cache of already rotated keys, reordered at append time, needs none of it).
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
int kvbfp_decode_attention_rope(const kvbfp_layout* layout, const kvbfp_cache* cache, int32_t n_q_heads,
                                const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                                int64_t max_len, float softmax_scale, const int32_t* perm_k,
                                const int32_t* perm_v, const float* rope_theta, const int32_t* rope_partner,
                                const float* rope_sign, void* out, void* workspace, size_t workspace_bytes,
                                void* hip_stream, float* kernel_ms);

/* Paged caches.  The four planes form a POOL of pages instead of one region per sequence:
 *   pool layout : batch = number of pages in the pool, max_seq = tokens per page (a power of two, at
 *                 least 16: the decode kernels look a page up per 16 tokens); planes
 *                 [n_pages][n_kv_heads][page_tokens][..] as kvbfp_cache_bytes(pool) sizes them.
 *   block_table : DEVICE int32 [batch][table_stride]; tokens [i * page_tokens, (i + 1) * page_tokens) of
 *                 sequence b live in page block_table[b * table_stride + i].  Entries that no token of the
 *                 call touches are not read.  Page numbers cannot be checked on the host: the kernels
 *                 clamp them to [0, n_pages) (memory-safe, result then unspecified).
 *   batch       : number of sequences (the pool layout's batch field counts pages).
 * A sequence can hold table_stride * page_tokens tokens; positions, lengths and max_len are checked
 * against that.  Everything else (arguments, results, errors) is as in the call without `_paged`:
 * the same bytes land in the same rows of a page that the contiguous call writes into a sequence's
 * region, and attention returns the same values.
 * kvbfp_dequantize_paged returns out [batch][n_tok][n_kv_heads][head_dim] as kvbfp_dequantize does.
 * kvbfp_decode_attention_paged takes q_mant_bits like kvbfp_decode_attention_qbfp (0 = query as given)
 * and kernel_ms like kvbfp_decode_attention_rope (NULL = asynchronous).
 * Errors: as the plain calls, plus UNSUPPORTED for a page size that is not a power of two >= 16. */
int kvbfp_quantize_append_paged(const kvbfp_layout* pool, const kvbfp_cache* cache, const int32_t* block_table,
                                int64_t table_stride, int32_t batch, const void* k_new, const void* v_new,
                                kvbfp_dtype dtype, int32_t n_new, int64_t stride_b, int64_t stride_t,
                                int64_t stride_h, int64_t pos0, const int32_t* pos_dev, const int32_t* perm_k,
                                const int32_t* perm_v, void* hip_stream);
int kvbfp_dequantize_paged(const kvbfp_layout* pool, const kvbfp_cache* cache, const int32_t* block_table,
                           int64_t table_stride, int32_t batch, int32_t which, int64_t t0, int64_t n_tok,
                           const int32_t* perm, void* out, kvbfp_dtype dtype, void* hip_stream);
size_t kvbfp_decode_workspace_bytes_paged(const kvbfp_layout* pool, int64_t table_stride, int32_t batch,
                                          int32_t n_q_heads, int64_t max_len);
int kvbfp_decode_attention_paged(const kvbfp_layout* pool, const kvbfp_cache* cache, const int32_t* block_table,
                                 int64_t table_stride, int32_t batch, int32_t n_q_heads, const void* q,
                                 kvbfp_dtype dtype, const int32_t* seq_len_dev, int64_t max_len,
                                 float softmax_scale, const int32_t* perm_k, const int32_t* perm_v,
                                 int32_t q_mant_bits, void* out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, float* kernel_ms);
/* kvbfp_append_decode_attention and kvbfp_decode_attention_multi over a pool of pages (Sec. III: the
 * current token's K/V rows are cast and written, then read with the rest; Alg. 1 steps 4-6).  The
 * arguments are those of the calls without `_paged`, with the pool, block_table, table_stride and
 * batch as above.  The page that holds position seq_len[b] - 1 (the appended row) must be in the
 * block table before the call.  workspace: kvbfp_decode_workspace_bytes_paged(pool, table_stride,
 * batch, n_q_heads [* n_q_tokens], max_len).  Same bytes in the cache and same values in `out` as the
 * contiguous calls.  DEVICE, async.  Errors: as those calls and as kvbfp_decode_attention_paged. */
int kvbfp_append_decode_attention_paged(const kvbfp_layout* pool, const kvbfp_cache* cache,
                                        const int32_t* block_table, int64_t table_stride, int32_t batch,
                                        int32_t n_q_heads, const void* k_new, const void* v_new,
                                        int64_t new_stride_b, int64_t new_stride_h, const void* q, kvbfp_dtype dtype,
                                        const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                        const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits, void* out,
                                        void* workspace, size_t workspace_bytes, void* hip_stream);
int kvbfp_decode_attention_multi_paged(const kvbfp_layout* pool, const kvbfp_cache* cache,
                                       const int32_t* block_table, int64_t table_stride, int32_t batch,
                                       int32_t n_q_heads, int32_t n_q_tokens, const void* q, kvbfp_dtype dtype,
                                       const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                       const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits, void* out,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* DEVICE, SYNCHRONOUS, for measurement.  Enqueues exactly the launches of
 * kvbfp_decode_attention_qbfp (Sec. III; same arguments, same result in `out`) with HIP events
 * recorded on `hip_stream` before the split pass, between the two passes and after the combine
 * pass, waits for the last one and returns the two durations in milliseconds:
 *   kernel_ms : HOST float[2]; [0] = split pass (the kernel that streams the cache), [1] = combine.
 * Creates and destroys three events per call; not meant for a serving loop.
 * Errors: as kvbfp_decode_attention_qbfp, plus INVALID_ARG for a NULL kernel_ms. */
int kvbfp_decode_attention_profile(const kvbfp_layout* layout, const kvbfp_cache* cache,
                                   int32_t n_q_heads, const void* q, kvbfp_dtype dtype,
                                   const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                   const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits,
                                   void* out, void* workspace, size_t workspace_bytes,
                                   void* hip_stream, float* kernel_ms);

/* DEVICE, SYNCHRONOUS, for measurement.  As kvbfp_decode_attention_profile, over a ring of caches of one
 * layout: the split pass (Sec. III; the kernel that streams the cache) is launched n_launches times back to
 * back, launch i over caches[i % n_caches], between two HIP events on `hip_stream`; then the combine pass
 * n_launches times between two more.  kernel_ms[0] and [1] are the two totals divided by n_launches: average
 * durations per launch that contain the dispatch gaps between successive launches but not the latency of the
 * first one.  A ring larger than the last-level cache keeps every launch reading from memory.  `out` holds
 * the result for the last cache launched.  n_launches = 1 with one cache is kvbfp_decode_attention_profile.
 *   caches : HOST array of n_caches structs of DEVICE plane pointers.
 * Errors: as kvbfp_decode_attention_profile, plus INVALID_ARG for n_caches < 1 or n_launches outside 1..4096. */
int kvbfp_decode_attention_profile_ring(const kvbfp_layout* layout, const kvbfp_cache* caches, int32_t n_caches,
                                        int32_t n_launches, int32_t n_q_heads, const void* q, kvbfp_dtype dtype,
                                        const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                        const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits,
                                        void* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                                        float* kernel_ms);

/* DEVICE, SYNCHRONOUS, for measurement.  Reads rows [0, n_tok) of the four planes of every (batch,
 * kv-head) once -- the bytes one kvbfp_decode_attention call over n_tok cached tokens streams (Sec. III:
 * the cached keys and values are read back each step) -- with plain 16-byte loads and no arithmetic, and
 * returns the kernel's duration (the sweep is launched twice, with two and with eight loads in flight per
 * lane, and the shorter duration is returned).  This is the rate a read-only kernel of the same size reaches on the
 * machine; the split pass of decode attention is reported against it next to the nominal HBM peak.
 *   wgs_per_unit : workgroups per (batch, kv-head); 0 = a default of about eight per compute unit.
 *   sink         : DEVICE, 4 writable bytes (keeps the loads alive; practically never written).
 *   kernel_ms    : HOST float[1], milliseconds between HIP events recorded on `hip_stream` around the faster launch.
 * Up to 15 bytes at either end of an exponent region that is not 16-byte aligned are skipped.
 * Errors: INVALID_ARG (NULL, n_tok outside (0, max_seq]), UNSUPPORTED (geometry), HIP. */
int kvbfp_measure_stream_read(const kvbfp_layout* layout, const kvbfp_cache* cache, int64_t n_tok,
                              int32_t wgs_per_unit, void* sink, void* hip_stream, float* kernel_ms);

/* DEVICE, asynchronous.  For callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same launches and
 * the same result as kvbfp_decode_attention_qbfp (same arguments, minus the workspace), with the partial
 * results of the sequence splits kept in a fixed device array inside the library instead
 * (KVBFP_NOALLOC_SCRATCH_BYTES per GPU, held from the first call on that GPU until the process ends).
 * The call allocates and frees nothing, on the host side of HIP or on the device; the array's address
 * on the current device is looked up once, on the first call made with that device current.
 *   - A geometry whose kvbfp_decode_workspace_bytes(layout, n_q_heads, max_len) exceeds
 *     KVBFP_NOALLOC_SCRATCH_BYTES is refused with KVBFP_ERR_WORKSPACE before anything is launched.
 *   - All calls on one GPU share the one array: calls that may overlap on a GPU (different streams
 *     without ordering between them) race on it and must be serialised by the caller.  Nothing in the
 *     array has to start at zero and nothing of a previous call is read.
 * Errors: as kvbfp_decode_attention_qbfp, plus WORKSPACE as above and HIP if the array's address
 * cannot be obtained. */
#define KVBFP_NOALLOC_SCRATCH_BYTES (4u << 20)
int kvbfp_decode_attention_noalloc(const kvbfp_layout* layout, const kvbfp_cache* cache,
                                   int32_t n_q_heads, const void* q, kvbfp_dtype dtype,
                                   const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                   const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits,
                                   void* out, void* hip_stream);

/* Message describing the last error on the calling thread ("" if none).  Static storage. */
const char* kvbfp_last_error(void);

/* Library version string, static storage. */
const char* kvbfp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVBFP_H */
