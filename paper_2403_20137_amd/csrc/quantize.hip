// Cache write and read-back kernels for gfx950: casting key/value rows to Block Floating Point
// (Sec. II-B, Eq. (1)) into the packed cache, and decoding them again.
//
// Write path (wave64): a 128-channel row is handled by 8 adjacent lanes, 16 consecutive cache
// positions per lane, so a lane never shares a block of 16 and a block of n = 32/64/128 spans
// 2/4/8 adjacent lanes of one DPP row: the per-block maximum is an all-reduce with 0..3 DPP steps.
// A workgroup of 256 threads takes 64 rows in two steps of 32 and issues the loads of both steps
// before it computes, which keeps 32-64 bytes per lane in flight.  Each lane rounds its 16
// mantissas in registers and stores them as one 8-byte (4-bit) or 16-byte (8-bit) word; the 8
// lanes of a row write one contiguous 64/128-byte segment.
//
// Rounding without a division: with e the block's scale exponent, |x| + 2^(23+e) is rounded by the
// adder to a multiple of 2^e (round to nearest, ties to even), and its low mantissa bits are the
// integer |x| / 2^e rounded.  The constant's bit pattern is then removed from all packed codes at
// once.  Blocks so large that 2^(23+e) overflows fp32 take a slower scaling path.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "fastdiv.h"
#include "kvbfp_internal.h"
#include "quantize_dev.h"

namespace {

constexpr int kLanesPerRow = 8;   // 16 channels per lane
constexpr int kRowsPerStep = 32;  // 256 threads
constexpr int kSteps = 2;
constexpr int kRowsPerWg = kRowsPerStep * kSteps;

// How a lane obtains its 16 inputs.
constexpr int kDirect = 0;        // aligned rows, cache order = memory order: 16-byte loads
constexpr int kLdsGather = 1;     // aligned rows + permutation: 16-byte loads, permuted through LDS
constexpr int kElementwise = 2;   // unaligned rows (with or without permutation): one load per element

// Unsigned division of numerators below 2^31 by a fixed divisor: floor(n / d) = (n * mul) >> shift.
using kvbfp::FastDiv;
using kvbfp::fastdiv;
using kvbfp::make_fastdiv;

struct QuantTensor {
    const void* src;       // [B][n_new][H][D] strided
    const int32_t* perm;   // [H][D] or nullptr
    uint8_t* mant;
    uint8_t* exp;
};

struct QuantArgs {
    QuantTensor t[2];
    int64_t stride_b, stride_t, stride_h;   // in elements
    int64_t pos0;
    const int32_t* pos_dev;
    int64_t len_cap;                         // >= 0: pos_dev holds sequence lengths, the row goes to min(max(len, 0), len_cap) - 1
    int64_t max_seq;                         // tokens a sequence can hold (paged: pages per sequence x page)
    const int32_t* block_table;              // paged cache: [B][table_stride], nullptr otherwise
    int64_t table_stride;
    int32_t log2_page, n_pages;
    int32_t H, n_new;
    uint32_t n_rows;                         // B * H * n_new, below 2^31
    FastDiv div_n_new, div_H;
};

using namespace kvbfp::cast;

// One row per 8 lanes, 64 rows per workgroup.  P = mantissa bits, N = block size.
template <int DT, int P, int N, int MODE>
__global__ __launch_bounds__(256) void quantize_rows_kernel(QuantArgs a) {
    constexpr int ESZ = DT == KVBFP_F32 ? 4 : 2;
    constexpr int kRowBytes = kD * ESZ;
    __shared__ __align__(16) uint8_t stage[MODE == kLdsGather ? kRowsPerWg * kRowBytes : 16];

    const QuantTensor T = a.t[blockIdx.y];
    const int sub = threadIdx.x & (kLanesPerRow - 1);
    const int slot = threadIdx.x >> 3;
    const int c0 = sub * 16;

    bool live[kSteps];
    int64_t crow[kSteps];
    int32_t head[kSteps];
    RawRow<DT> raw[kSteps];
    const uint8_t* srow[kSteps];
#pragma unroll
    for (int k = 0; k < kSteps; ++k) {
        // Rows beyond the end keep their lanes active (DPP reads neighbours) but touch no memory.
        const uint32_t r = blockIdx.x * (uint32_t)kRowsPerWg + (uint32_t)(k * kRowsPerStep + slot);
        const bool in_range = r < a.n_rows;
        const uint32_t rr = in_range ? r : 0u;
        const uint32_t bh = fastdiv(rr, a.div_n_new);
        const uint32_t t = rr - bh * (uint32_t)a.n_new;
        const uint32_t b = fastdiv(bh, a.div_H);
        const uint32_t h = bh - b * (uint32_t)a.H;
        int64_t pos = a.pos0;
        if (a.pos_dev) pos = a.len_cap >= 0 ? min(max((int64_t)a.pos_dev[b], (int64_t)0), a.len_cap) - 1 : (int64_t)a.pos_dev[b];
        pos += t;
        live[k] = in_range && pos >= 0 && pos < a.max_seq;
        if (a.block_table) {      // page numbers cannot be checked on the host: clamped to the pool
            int page = live[k] ? a.block_table[(int64_t)b * a.table_stride + (pos >> a.log2_page)] : 0;
            page = page < 0 ? 0 : (page >= a.n_pages ? a.n_pages - 1 : page);
            crow[k] = (((int64_t)page * a.H + h) << a.log2_page) + (pos & (((int64_t)1 << a.log2_page) - 1));
        } else {
            crow[k] = ((int64_t)b * a.H + h) * a.max_seq + pos;
        }
        head[k] = (int32_t)h;
        srow[k] = (const uint8_t*)T.src + ((int64_t)b * a.stride_b + (int64_t)t * a.stride_t + (int64_t)h * a.stride_h) * ESZ;
        if (MODE != kElementwise) {
#pragma unroll
            for (int i = 0; i < ESZ * 16 / 16; ++i)
                if (live[k]) {
                    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
                    const u32x4_t t = *((const u32x4_t*)(srow[k] + c0 * ESZ) + i);
                    raw[k].v[i] = make_uint4(t[0], t[1], t[2], t[3]);
                } else {
                    raw[k].v[i] = make_uint4(0u, 0u, 0u, 0u);
                }
        }
    }

#pragma unroll
    for (int k = 0; k < kSteps; ++k) {
        float x[16];
        if (MODE == kDirect || (MODE == kLdsGather && T.perm == nullptr)) {
            widen16<DT>(raw[k], x);
        } else if (MODE == kLdsGather) {
            // The row goes to LDS in memory order and comes back in cache order: position j of the
            // cache holds channel perm[j].  A row stays inside 8 lanes of one wavefront.
            uint8_t* lrow = stage + (k * kRowsPerStep + slot) * kRowBytes;
#pragma unroll
            for (int i = 0; i < ESZ * 16 / 16; ++i) ((uint4*)(lrow + c0 * ESZ))[i] = raw[k].v[i];
            int4 pi[4];
            const int4* pp = (const int4*)(T.perm + (int64_t)head[k] * kD + c0);
#pragma unroll
            for (int i = 0; i < 4; ++i) pi[i] = pp[i];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = (i & 3) == 0 ? pi[i >> 2].x : ((i & 3) == 1 ? pi[i >> 2].y : ((i & 3) == 2 ? pi[i >> 2].z : pi[i >> 2].w));
                const int cc = c & (kD - 1);          // a valid permutation is unchanged; keeps LDS reads in range
                if (DT == KVBFP_F32) x[i] = ((const float*)lrow)[cc];
                else if (DT == KVBFP_F16) x[i] = widen_f16(((const uint16_t*)lrow)[cc]);
                else x[i] = widen_bf16(((const uint16_t*)lrow)[cc]);
            }
        } else {
            const int32_t* pr = T.perm ? T.perm + (int64_t)head[k] * kD : nullptr;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = 0.f;
                if (live[k]) {
                    const int c = pr ? (pr[c0 + i] & (kD - 1)) : (c0 + i);
                    if (DT == KVBFP_F32) v = ((const float*)srow[k])[c];
                    else if (DT == KVBFP_F16) v = widen_f16(((const uint16_t*)srow[k])[c]);
                    else v = widen_bf16(((const uint16_t*)srow[k])[c]);
                }
                x[i] = v;
            }
        }
        encode_store<P, N>(x, sub, live[k], T.mant, T.exp, crow[k]);
    }
}

// Read-back kernel: one row per 16 lanes, 8 cache positions per lane, four rows per thread (64 per workgroup):
// all of a thread's loads are in flight before the first value is decoded.
constexpr int kDqLanesPerRow = 16;
constexpr int kDqRowsPerStep = 256 / kDqLanesPerRow;
constexpr int kDqSteps = 4;
constexpr int kDqRowsPerBlock = kDqRowsPerStep * kDqSteps;

struct DequantArgs {
    const uint8_t* mant;
    const uint8_t* exp;
    const int32_t* perm;
    void* out;
    int64_t t0, max_seq;
    int32_t H, n_tok;
    int32_t perm_aligned;   // perm is 16-byte aligned: its entries are loaded four at a time
    uint32_t n_rows;   // B * H * n_tok, below 2^31
    FastDiv div_n_tok, div_H;
    const int32_t* block_table;   // paged cache: [B][table_stride], nullptr otherwise
    int64_t table_stride;
    int32_t log2_page, n_pages;
};

__device__ __forceinline__ uint16_t narrow_bf16(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int DT>
__device__ __forceinline__ uint32_t narrow16(float v) {
    return DT == KVBFP_F16 ? (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)v) : (uint32_t)narrow_bf16(v);
}

// 16-byte store that does not displace the caches: the output is written once and read by somebody else later
// (measured on the bulk read-back: 62 -> 58.6 us with these and the non-temporal mantissa loads)
typedef uint32_t dq_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t dq_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store16_stream(void* p, uint32_t x, uint32_t y, uint32_t z, uint32_t w) {
    __builtin_nontemporal_store(dq_u32x4{x, y, z, w}, (dq_u32x4*)p);
}

// PERM: the values leave in the callers' channel order, position j of the cache going to channel perm[j]; the row
// is reordered in LDS (a row stays inside 16 lanes of one wavefront), so the stores are the same 16-byte ones.
template <int DT, int P, int LPB, bool PERM>
__global__ __launch_bounds__(256) void dequantize_rows_kernel(DequantArgs a) {
    constexpr int ESZ = DT == KVBFP_F32 ? 4 : 2;
    __shared__ __align__(16) uint8_t stage[PERM ? kDqRowsPerBlock * kD * ESZ : 16];
    const int lane16 = threadIdx.x & (kDqLanesPerRow - 1);
    const int slot = threadIdx.x >> 4;
    const int c0 = lane16 * 8;

    bool live[kDqSteps];
    int64_t orow[kDqSteps];
    uint32_t w0[kDqSteps], w1[kDqSteps], eb[kDqSteps];
    int4 pi[kDqSteps][2];
#pragma unroll
    for (int k = 0; k < kDqSteps; ++k) {
        const uint32_t r = blockIdx.x * (uint32_t)kDqRowsPerBlock + (uint32_t)(k * kDqRowsPerStep + slot);
        live[k] = r < a.n_rows;
        const uint32_t rr = live[k] ? r : 0u;
        const uint32_t bh = fastdiv(rr, a.div_n_tok);
        const uint32_t t = rr - bh * (uint32_t)a.n_tok;
        const uint32_t b = fastdiv(bh, a.div_H);
        const uint32_t h = bh - b * (uint32_t)a.H;
        int64_t crow = ((int64_t)b * a.H + h) * a.max_seq + a.t0 + t;
        if (a.block_table) {      // page numbers cannot be checked on the host: clamped to the pool
            const int64_t pos = a.t0 + t;
            int page = a.block_table[(int64_t)b * a.table_stride + (pos >> a.log2_page)];
            page = page < 0 ? 0 : (page >= a.n_pages ? a.n_pages - 1 : page);
            crow = (((int64_t)page * a.H + h) << a.log2_page) + (pos & (((int64_t)1 << a.log2_page) - 1));
        }
        orow[k] = (((int64_t)b * a.n_tok + t) * a.H + h) * kD;
        eb[k] = a.exp[crow * (kDqLanesPerRow / LPB) + lane16 / LPB];
        if (P == 4) {
            w0[k] = __builtin_nontemporal_load((const uint32_t*)(a.mant + crow * 64) + lane16);
            w1[k] = 0u;
        } else {
            const dq_u32x2 w = __builtin_nontemporal_load((const dq_u32x2*)(a.mant + crow * 128) + lane16);
            w0[k] = w[0];
            w1[k] = w[1];
        }
        if (PERM) {
            const int32_t* pr = a.perm + (int64_t)h * kD + c0;
            if (a.perm_aligned) {
                pi[k][0] = ((const int4*)pr)[0];
                pi[k][1] = ((const int4*)pr)[1];
            } else {
                pi[k][0] = make_int4(pr[0], pr[1], pr[2], pr[3]);
                pi[k][1] = make_int4(pr[4], pr[5], pr[6], pr[7]);
            }
        }
    }

#pragma unroll
    for (int k = 0; k < kDqSteps; ++k) {
        const int e = (int)eb[k] - 127 - (P - 2);
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t code = P == 4 ? (w0[k] >> (4 * i)) & 0xFu : ((i < 4 ? w0[k] : w1[k]) >> (8 * (i & 3))) & 0xFFu;
            const uint32_t mag = code & ((1u << (P - 1)) - 1u);
            const float m = ldexpf((float)mag, e);
            v[i] = (code >> (P - 1)) ? -m : m;
        }
        if (PERM) {
            uint8_t* lrow = stage + (k * kDqRowsPerStep + slot) * (kD * ESZ);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int4 q = pi[k][i >> 2];
                const int c = ((i & 3) == 0 ? q.x : ((i & 3) == 1 ? q.y : ((i & 3) == 2 ? q.z : q.w))) & (kD - 1);   // masked: stays inside the row
                if (DT == KVBFP_F32) ((float*)lrow)[c] = v[i];
                else ((uint16_t*)lrow)[c] = (uint16_t)narrow16<DT>(v[i]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (live[k]) {
                if (DT == KVBFP_F32) {
                    const uint4 x = ((const uint4*)(lrow + c0 * 4))[0], y = ((const uint4*)(lrow + c0 * 4))[1];
                    store16_stream((float*)a.out + orow[k] + c0, x.x, x.y, x.z, x.w);
                    store16_stream((float*)a.out + orow[k] + c0 + 4, y.x, y.y, y.z, y.w);
                } else {
                    const uint4 x = *(const uint4*)(lrow + c0 * 2);
                    store16_stream((uint16_t*)a.out + orow[k] + c0, x.x, x.y, x.z, x.w);
                }
            }
        } else if (live[k]) {
            if (DT == KVBFP_F32) {
                store16_stream((float*)a.out + orow[k] + c0, __float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
                store16_stream((float*)a.out + orow[k] + c0 + 4, __float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7]));
            } else {
                uint32_t w[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) w[i] = narrow16<DT>(v[2 * i]) | (narrow16<DT>(v[2 * i + 1]) << 16);
                store16_stream((uint16_t*)a.out + orow[k] + c0, w[0], w[1], w[2], w[3]);
            }
        }
    }
}

template <int DT, int P, int MODE>
hipError_t launch_quant_n(int block, const QuantArgs& a, dim3 grid, hipStream_t s) {
    switch (block) {
        case 16: quantize_rows_kernel<DT, P, 16, MODE><<<grid, 256, 0, s>>>(a); break;
        case 32: quantize_rows_kernel<DT, P, 32, MODE><<<grid, 256, 0, s>>>(a); break;
        case 64: quantize_rows_kernel<DT, P, 64, MODE><<<grid, 256, 0, s>>>(a); break;
        default: quantize_rows_kernel<DT, P, 128, MODE><<<grid, 256, 0, s>>>(a); break;
    }
    return hipGetLastError();
}
template <int DT, int MODE>
hipError_t launch_quant_p(int p, int block, const QuantArgs& a, dim3 grid, hipStream_t s) {
    return p == 4 ? launch_quant_n<DT, 4, MODE>(block, a, grid, s) : launch_quant_n<DT, 8, MODE>(block, a, grid, s);
}
template <int MODE>
hipError_t launch_quant(int dt, int p, int block, const QuantArgs& a, dim3 grid, hipStream_t s) {
    switch (dt) {
        case KVBFP_F32: return launch_quant_p<KVBFP_F32, MODE>(p, block, a, grid, s);
        case KVBFP_F16: return launch_quant_p<KVBFP_F16, MODE>(p, block, a, grid, s);
        default: return launch_quant_p<KVBFP_BF16, MODE>(p, block, a, grid, s);
    }
}

template <int DT, int P, bool PERM>
hipError_t launch_dequant_lpb(int block, const DequantArgs& a, dim3 grid, hipStream_t s) {
    switch (block) {
        case 16: dequantize_rows_kernel<DT, P, 2, PERM><<<grid, 256, 0, s>>>(a); break;
        case 32: dequantize_rows_kernel<DT, P, 4, PERM><<<grid, 256, 0, s>>>(a); break;
        case 64: dequantize_rows_kernel<DT, P, 8, PERM><<<grid, 256, 0, s>>>(a); break;
        default: dequantize_rows_kernel<DT, P, 16, PERM><<<grid, 256, 0, s>>>(a); break;
    }
    return hipGetLastError();
}
template <int DT>
hipError_t launch_dequant_p(int p, int block, const DequantArgs& a, dim3 grid, hipStream_t s) {
    if (a.perm) return p == 4 ? launch_dequant_lpb<DT, 4, true>(block, a, grid, s) : launch_dequant_lpb<DT, 8, true>(block, a, grid, s);
    return p == 4 ? launch_dequant_lpb<DT, 4, false>(block, a, grid, s) : launch_dequant_lpb<DT, 8, false>(block, a, grid, s);
}

}  // namespace

using namespace kvbfp;

extern "C" {

int kvbfp_quantize_append(const kvbfp_layout* L, const kvbfp_cache* cache, const void* k_new,
                          const void* v_new, kvbfp_dtype dtype, int32_t n_new, int64_t stride_b,
                          int64_t stride_t, int64_t stride_h, int64_t pos0, const int32_t* pos_dev,
                          const int32_t* perm_k, const int32_t* perm_v, void* hip_stream) {
    clear_error();
    return kvbfp::quantize_append_impl(L, cache, k_new, v_new, dtype, n_new, stride_b, stride_t, stride_h, pos0,
                                       pos_dev, -1, perm_k, perm_v, hip_stream);
}

int kvbfp_quantize_append_paged(const kvbfp_layout* pool, const kvbfp_cache* cache, const int32_t* block_table,
                                int64_t table_stride, int32_t batch, const void* k_new, const void* v_new,
                                kvbfp_dtype dtype, int32_t n_new, int64_t stride_b, int64_t stride_t,
                                int64_t stride_h, int64_t pos0, const int32_t* pos_dev, const int32_t* perm_k,
                                const int32_t* perm_v, void* hip_stream) {
    clear_error();
    const kvbfp::Paging pg{block_table, table_stride, batch};
    return kvbfp::quantize_append_impl(pool, cache, k_new, v_new, dtype, n_new, stride_b, stride_t, stride_h, pos0,
                                       pos_dev, -1, perm_k, perm_v, hip_stream, &pg);
}

}  // extern "C"

// len_cap >= 0: pos_dev holds sequence lengths (clamped to [0, len_cap]) and row i of sequence b goes
// to position length - 1 + i; len_cap < 0: pos_dev holds positions, as in the public call.
int kvbfp::quantize_append_impl(const kvbfp_layout* L, const kvbfp_cache* cache, const void* k_new,
                                const void* v_new, kvbfp_dtype dtype, int32_t n_new, int64_t stride_b,
                                int64_t stride_t, int64_t stride_h, int64_t pos0, const int32_t* pos_dev,
                                int64_t len_cap, const int32_t* perm_k, const int32_t* perm_v,
                                void* hip_stream, const Paging* paging) {
    kvbfp_layout logical;
    const kvbfp_layout* pool = L;
    if (paging) {
        if (int rc = check_paging(pool, *paging, &logical)) return rc;
        L = &logical;             // from here on: what the sequences look like
    }
    if (int rc = check_device_layout(L)) return rc;
    if (int rc = check_cache(cache, k_new != nullptr, v_new != nullptr)) return rc;
    const int esz = dtype_size(dtype);
    if (esz == 0) return fail(KVBFP_ERR_INVALID_ARG, "quantize_append: unknown dtype %d", (int)dtype);
    if (n_new < 0) return fail(KVBFP_ERR_INVALID_ARG, "quantize_append: n_new = %d", n_new);
    if (stride_b < 0 || stride_t < 0 || stride_h < 0)
        return fail(KVBFP_ERR_INVALID_ARG, "quantize_append: negative stride");
    if (!pos_dev && (pos0 < 0 || pos0 + n_new > L->max_seq))
        return fail(KVBFP_ERR_INVALID_ARG, "quantize_append: positions [%lld, %lld) outside max_seq %lld",
                    (long long)pos0, (long long)(pos0 + n_new), (long long)L->max_seq);
    if (n_new == 0 || (!k_new && !v_new)) return KVBFP_OK;

    QuantArgs a{};
    int nt = 0;
    if (k_new) a.t[nt++] = QuantTensor{k_new, perm_k, cache->k_mant, cache->k_exp};
    if (v_new) a.t[nt++] = QuantTensor{v_new, perm_v, cache->v_mant, cache->v_exp};
    a.stride_b = stride_b; a.stride_t = stride_t; a.stride_h = stride_h;
    a.pos0 = pos0; a.pos_dev = pos_dev; a.len_cap = len_cap; a.max_seq = L->max_seq;
    if (paging) {
        a.block_table = paging->block_table; a.table_stride = paging->table_stride;
        a.n_pages = pool->batch;
        a.log2_page = 0;
        while (((int64_t)1 << a.log2_page) < pool->max_seq) ++a.log2_page;
    }
    a.H = L->n_kv_heads; a.n_new = n_new;
    const int64_t n_rows = (int64_t)L->batch * L->n_kv_heads * n_new;
    if (n_rows > 0x7FFFFFFF) return fail(KVBFP_ERR_UNSUPPORTED, "quantize_append: too many rows");
    a.n_rows = (uint32_t)n_rows;
    a.div_n_new = make_fastdiv((uint32_t)n_new);
    a.div_H = make_fastdiv((uint32_t)L->n_kv_heads);
    const dim3 grid((unsigned)((n_rows + kRowsPerWg - 1) / kRowsPerWg), (unsigned)nt, 1);

    // 16-byte vector loads need aligned rows; a permutation is then applied through LDS.  Anything
    // unaligned is gathered element by element.
    auto aligned = [&](const void* p) {
        return p == nullptr || (((uintptr_t)p % 16 == 0) && (stride_b * esz) % 16 == 0 &&
                                (stride_t * esz) % 16 == 0 && (stride_h * esz) % 16 == 0);
    };
    const bool rows_aligned = aligned(k_new) && aligned(v_new);
    const bool perms_aligned = (uintptr_t)perm_k % 16 == 0 && (uintptr_t)perm_v % 16 == 0;
    const bool any_perm = (k_new && perm_k) || (v_new && perm_v);
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t err;
    if (!rows_aligned || (any_perm && !perms_aligned)) err = launch_quant<kElementwise>(dtype, L->mant_bits, L->block, a, grid, s);
    else if (any_perm) err = launch_quant<kLdsGather>(dtype, L->mant_bits, L->block, a, grid, s);
    else err = launch_quant<kDirect>(dtype, L->mant_bits, L->block, a, grid, s);
    if (err != hipSuccess) return fail(KVBFP_ERR_HIP, "quantize_append: %s", hipGetErrorString(err));
    return KVBFP_OK;
}

extern "C" {

static int dequantize_impl(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t which, int64_t t0,
                           int64_t n_tok, const int32_t* perm, void* out, kvbfp_dtype dtype,
                           void* hip_stream, const kvbfp::Paging* paging) {
    clear_error();
    kvbfp_layout logical;
    const kvbfp_layout* pool = L;
    if (paging) {
        if (int rc = check_paging(pool, *paging, &logical)) return rc;
        L = &logical;             // from here on: what the sequences look like
    }
    if (int rc = check_device_layout(L)) return rc;
    if (which != 0 && which != 1) return fail(KVBFP_ERR_INVALID_ARG, "dequantize: which = %d", which);
    if (int rc = check_cache(cache, which == 0, which == 1)) return rc;
    if (dtype_size(dtype) == 0) return fail(KVBFP_ERR_INVALID_ARG, "dequantize: unknown dtype %d", (int)dtype);
    if (t0 < 0 || n_tok < 0 || t0 + n_tok > L->max_seq)
        return fail(KVBFP_ERR_INVALID_ARG, "dequantize: tokens [%lld, %lld) outside max_seq %lld",
                    (long long)t0, (long long)(t0 + n_tok), (long long)L->max_seq);
    if (n_tok == 0) return KVBFP_OK;
    if (!out) return fail(KVBFP_ERR_INVALID_ARG, "dequantize: out is NULL");
    if ((uintptr_t)out % 16 != 0) return fail(KVBFP_ERR_INVALID_ARG, "dequantize: out must be 16-byte aligned");

    DequantArgs a{};
    a.mant = which == 0 ? cache->k_mant : cache->v_mant;
    a.exp = which == 0 ? cache->k_exp : cache->v_exp;
    a.perm = perm; a.out = out; a.t0 = t0; a.n_tok = (int32_t)n_tok; a.max_seq = L->max_seq;
    a.H = L->n_kv_heads;
    const int64_t n_rows = (int64_t)L->batch * L->n_kv_heads * n_tok;
    if (n_rows > 0x7FFFFFFF) return fail(KVBFP_ERR_UNSUPPORTED, "dequantize: more than 2^31 - 1 rows in one call");
    a.n_rows = (uint32_t)n_rows;
    a.div_n_tok = make_fastdiv((uint32_t)n_tok);
    a.div_H = make_fastdiv((uint32_t)L->n_kv_heads);
    a.perm_aligned = (uintptr_t)perm % 16 == 0;
    if (paging) {
        a.block_table = paging->block_table; a.table_stride = paging->table_stride;
        a.n_pages = pool->batch;
        a.log2_page = 0;
        while (((int64_t)1 << a.log2_page) < pool->max_seq) ++a.log2_page;
    }
    const int64_t blocks = (n_rows + kDqRowsPerBlock - 1) / kDqRowsPerBlock;
    const dim3 grid((unsigned)blocks, 1, 1);
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t err;
    switch (dtype) {
        case KVBFP_F32: err = launch_dequant_p<KVBFP_F32>(L->mant_bits, L->block, a, grid, s); break;
        case KVBFP_F16: err = launch_dequant_p<KVBFP_F16>(L->mant_bits, L->block, a, grid, s); break;
        default: err = launch_dequant_p<KVBFP_BF16>(L->mant_bits, L->block, a, grid, s); break;
    }
    if (err != hipSuccess) return fail(KVBFP_ERR_HIP, "dequantize: %s", hipGetErrorString(err));
    return KVBFP_OK;
}

int kvbfp_dequantize(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t which, int64_t t0,
                     int64_t n_tok, const int32_t* perm, void* out, kvbfp_dtype dtype,
                     void* hip_stream) {
    return dequantize_impl(L, cache, which, t0, n_tok, perm, out, dtype, hip_stream, nullptr);
}

int kvbfp_dequantize_paged(const kvbfp_layout* pool, const kvbfp_cache* cache, const int32_t* block_table,
                           int64_t table_stride, int32_t batch, int32_t which, int64_t t0, int64_t n_tok,
                           const int32_t* perm, void* out, kvbfp_dtype dtype, void* hip_stream) {
    const kvbfp::Paging pg{block_table, table_stride, batch};
    return dequantize_impl(pool, cache, which, t0, n_tok, perm, out, dtype, hip_stream, &pg);
}

}  // extern "C"
