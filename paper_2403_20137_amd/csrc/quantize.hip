// Cache write and read-back kernels for gfx950: casting key/value rows to Block Floating Point
// (Sec. II-B, Eq. (1)) into the packed cache, and decoding them again.
//
// Work decomposition (wave64): a 128-channel row is handled by 16 adjacent lanes, 8 consecutive
// cache positions per lane, so one wavefront carries 4 rows.  A lane loads its 8 inputs with one
// or two 16-byte loads, a block of n = 16/32/64/128 positions spans 2/4/8/16 adjacent lanes of one
// DPP row, so the per-block maximum is an all-reduce with 1..4 DPP steps and never leaves the row.
// Each lane then rounds its 8 mantissas in registers and stores one packed dword (4-bit) or two
// (8-bit); the 16 lanes of a row write one contiguous 64/128-byte segment.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kvbfp_internal.h"

namespace {

constexpr int kD = 128;          // channels per row (head_dim)
constexpr int kLanesPerRow = 16; // 8 channels per lane
constexpr int kRowsPerBlock = 16; // 256 threads

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
    int64_t max_seq;
    int32_t H, n_new;
    int64_t n_rows;                          // B * H * n_new
};

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}

// All-reduce maximum over the LPB adjacent lanes that share a block (LPB = block / 8).
// quad_perm[1,0,3,2], quad_perm[2,3,0,1], row_half_mirror, row_mirror: after the first two steps
// every quad is uniform, so the mirrors (which map quad k to quad 1-k resp. 3-k) complete the
// butterfly.
template <int LPB>
__device__ __forceinline__ uint32_t block_allmax(uint32_t a) {
    a = max(a, dpp_mov<0xB1>(a));
    if (LPB >= 4) a = max(a, dpp_mov<0x4E>(a));
    if (LPB >= 8) a = max(a, dpp_mov<0x141>(a));
    if (LPB >= 16) a = max(a, dpp_mov<0x140>(a));
    return a;
}

__device__ __forceinline__ float widen_bf16(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float widen_f16(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// Loads the 8 inputs of this lane: cache positions c0..c0+7 of the row at `row`.
template <int DT, bool GATHER>
__device__ __forceinline__ void load8(const void* row, const int32_t* perm_row, int c0, float (&x)[8]) {
    if (GATHER) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = perm_row ? perm_row[c0 + i] : (c0 + i);
            if (DT == KVBFP_F32) x[i] = ((const float*)row)[c];
            else if (DT == KVBFP_F16) x[i] = widen_f16(((const uint16_t*)row)[c]);
            else x[i] = widen_bf16(((const uint16_t*)row)[c]);
        }
    } else if (DT == KVBFP_F32) {
        const float4 a = *(const float4*)((const float*)row + c0);
        const float4 b = *(const float4*)((const float*)row + c0 + 4);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
        const uint4 v = *(const uint4*)((const uint16_t*)row + c0);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DT == KVBFP_F16) {
                x[2 * i] = widen_f16(w[i] & 0xFFFFu);
                x[2 * i + 1] = widen_f16(w[i] >> 16);
            } else {
                x[2 * i] = widen_bf16(w[i] & 0xFFFFu);
                x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
            }
        }
    }
}

// One row per 16 lanes.  P = mantissa bits, LPB = lanes per block.
template <int DT, int P, int LPB, bool GATHER>
__global__ __launch_bounds__(256) void quantize_rows_kernel(QuantArgs a) {
    const QuantTensor T = a.t[blockIdx.y];
    const int lane16 = threadIdx.x & (kLanesPerRow - 1);
    const int64_t r = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 4);
    // Rows beyond the end keep their lanes active (DPP reads neighbours) but touch no memory.
    const bool in_range = r < a.n_rows;
    const int64_t rr = in_range ? r : 0;
    const int32_t t = (int32_t)(rr % a.n_new);
    const int32_t h = (int32_t)((rr / a.n_new) % a.H);
    const int32_t b = (int32_t)(rr / ((int64_t)a.n_new * a.H));
    const int64_t pos = (a.pos_dev ? (int64_t)a.pos_dev[b] : a.pos0) + t;
    const bool live = in_range && pos >= 0 && pos < a.max_seq;

    const int c0 = lane16 * 8;
    float x[8];
    if (live) {
        const int64_t off = b * a.stride_b + t * a.stride_t + h * a.stride_h;
        const void* row = (DT == KVBFP_F32) ? (const void*)((const float*)T.src + off)
                                            : (const void*)((const uint16_t*)T.src + off);
        load8<DT, GATHER>(row, T.perm ? T.perm + (int64_t)h * kD : nullptr, c0, x);
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = 0.f;
    }

    // Largest magnitude of the block, compared on the bit patterns (monotone for finite values).
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = max(amax, __float_as_uint(x[i]) & 0x7FFFFFFFu);
    amax = block_allmax<LPB>(amax);

    // Shared exponent byte: the fp32 exponent field of the maximum, one higher when rounding the
    // maximum to P-1 magnitude bits would carry (its top P-1 fraction bits are all ones); at least
    // 1 so that subnormal blocks use the scale of the smallest normal; 0 marks an all-zero block.
    const uint32_t bumped = (amax + (1u << (24 - P))) >> 23;
    const int E = amax == 0 ? 0 : (int)max(bumped, 1u);
    const int e = E - 127 - (P - 2);

    // Mantissas: scaling by a power of two is exact, adding 2^23 rounds to nearest-even integer.
    uint32_t code[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float scaled = ldexpf(x[i], -e);
        const uint32_t mag = __float_as_uint(fabsf(scaled) + 8388608.0f) & 0xFFu;
        const uint32_t sign = (__float_as_uint(x[i]) >> 31) << (P - 1);
        code[i] = mag ? (mag | sign) : 0u;
    }

    if (!live) return;
    const int64_t crow = ((int64_t)b * a.H + h) * a.max_seq + pos;
    if (P == 4) {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) w |= code[i] << (4 * i);
        ((uint32_t*)(T.mant + crow * 64))[lane16] = w;
    } else {
        uint2 w = make_uint2(0u, 0u);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w.x |= code[i] << (8 * i);
            w.y |= code[4 + i] << (8 * i);
        }
        ((uint2*)(T.mant + crow * 128))[lane16] = w;
    }
    if ((lane16 & (LPB - 1)) == 0) T.exp[crow * (kLanesPerRow / LPB) + lane16 / LPB] = (uint8_t)E;
}

struct DequantArgs {
    const uint8_t* mant;
    const uint8_t* exp;
    const int32_t* perm;
    void* out;
    int64_t t0, n_tok, max_seq;
    int32_t H;
    int64_t n_rows;   // B * H * n_tok
};

__device__ __forceinline__ uint16_t narrow_bf16(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int DT, int P, int LPB>
__global__ __launch_bounds__(256) void dequantize_rows_kernel(DequantArgs a) {
    const int lane16 = threadIdx.x & (kLanesPerRow - 1);
    const int64_t r = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 4);
    if (r >= a.n_rows) return;
    const int64_t t = r % a.n_tok;
    const int32_t h = (int32_t)((r / a.n_tok) % a.H);
    const int64_t b = r / (a.n_tok * a.H);
    const int64_t crow = (b * a.H + h) * a.max_seq + a.t0 + t;
    const int E = a.exp[crow * (kLanesPerRow / LPB) + lane16 / LPB];
    const int e = E - 127 - (P - 2);
    uint32_t code[8];
    if (P == 4) {
        const uint32_t w = ((const uint32_t*)(a.mant + crow * 64))[lane16];
#pragma unroll
        for (int i = 0; i < 8; ++i) code[i] = (w >> (4 * i)) & 0xFu;
    } else {
        const uint2 w = ((const uint2*)(a.mant + crow * 128))[lane16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            code[i] = (w.x >> (8 * i)) & 0xFFu;
            code[4 + i] = (w.y >> (8 * i)) & 0xFFu;
        }
    }
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t mag = code[i] & ((1u << (P - 1)) - 1u);
        const float m = ldexpf((float)mag, e);
        v[i] = (code[i] >> (P - 1)) ? -m : m;
    }
    const int c0 = lane16 * 8;
    const int64_t orow = ((b * a.n_tok + t) * a.H + h) * kD;
    if (a.perm) {
        const int32_t* pr = a.perm + (int64_t)h * kD;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = pr[c0 + i];
            if (DT == KVBFP_F32) ((float*)a.out)[orow + c] = v[i];
            else if (DT == KVBFP_F16)
                ((uint16_t*)a.out)[orow + c] = __builtin_bit_cast(unsigned short, (_Float16)v[i]);
            else ((uint16_t*)a.out)[orow + c] = narrow_bf16(v[i]);
        }
    } else if (DT == KVBFP_F32) {
        float4* o = (float4*)((float*)a.out + orow + c0);
        o[0] = make_float4(v[0], v[1], v[2], v[3]);
        o[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t lo, hi;
            if (DT == KVBFP_F16) {
                lo = __builtin_bit_cast(unsigned short, (_Float16)v[2 * i]);
                hi = __builtin_bit_cast(unsigned short, (_Float16)v[2 * i + 1]);
            } else {
                lo = narrow_bf16(v[2 * i]);
                hi = narrow_bf16(v[2 * i + 1]);
            }
            w[i] = lo | (hi << 16);
        }
        *(uint4*)((uint16_t*)a.out + orow + c0) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <int DT, int P, bool GATHER>
hipError_t launch_quant_lpb(int block, const QuantArgs& a, dim3 grid, hipStream_t s) {
    switch (block) {
        case 16: quantize_rows_kernel<DT, P, 2, GATHER><<<grid, 256, 0, s>>>(a); break;
        case 32: quantize_rows_kernel<DT, P, 4, GATHER><<<grid, 256, 0, s>>>(a); break;
        case 64: quantize_rows_kernel<DT, P, 8, GATHER><<<grid, 256, 0, s>>>(a); break;
        default: quantize_rows_kernel<DT, P, 16, GATHER><<<grid, 256, 0, s>>>(a); break;
    }
    return hipGetLastError();
}
template <int DT, bool GATHER>
hipError_t launch_quant_p(int p, int block, const QuantArgs& a, dim3 grid, hipStream_t s) {
    return p == 4 ? launch_quant_lpb<DT, 4, GATHER>(block, a, grid, s)
                  : launch_quant_lpb<DT, 8, GATHER>(block, a, grid, s);
}
template <bool GATHER>
hipError_t launch_quant(int dt, int p, int block, const QuantArgs& a, dim3 grid, hipStream_t s) {
    switch (dt) {
        case KVBFP_F32: return launch_quant_p<KVBFP_F32, GATHER>(p, block, a, grid, s);
        case KVBFP_F16: return launch_quant_p<KVBFP_F16, GATHER>(p, block, a, grid, s);
        default: return launch_quant_p<KVBFP_BF16, GATHER>(p, block, a, grid, s);
    }
}

template <int DT, int P>
hipError_t launch_dequant_lpb(int block, const DequantArgs& a, dim3 grid, hipStream_t s) {
    switch (block) {
        case 16: dequantize_rows_kernel<DT, P, 2><<<grid, 256, 0, s>>>(a); break;
        case 32: dequantize_rows_kernel<DT, P, 4><<<grid, 256, 0, s>>>(a); break;
        case 64: dequantize_rows_kernel<DT, P, 8><<<grid, 256, 0, s>>>(a); break;
        default: dequantize_rows_kernel<DT, P, 16><<<grid, 256, 0, s>>>(a); break;
    }
    return hipGetLastError();
}
template <int DT>
hipError_t launch_dequant_p(int p, int block, const DequantArgs& a, dim3 grid, hipStream_t s) {
    return p == 4 ? launch_dequant_lpb<DT, 4>(block, a, grid, s) : launch_dequant_lpb<DT, 8>(block, a, grid, s);
}

}  // namespace

using namespace kvbfp;

extern "C" {

int kvbfp_quantize_append(const kvbfp_layout* L, const kvbfp_cache* cache, const void* k_new,
                          const void* v_new, kvbfp_dtype dtype, int32_t n_new, int64_t stride_b,
                          int64_t stride_t, int64_t stride_h, int64_t pos0, const int32_t* pos_dev,
                          const int32_t* perm_k, const int32_t* perm_v, void* hip_stream) {
    clear_error();
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
    a.pos0 = pos0; a.pos_dev = pos_dev; a.max_seq = L->max_seq;
    a.H = L->n_kv_heads; a.n_new = n_new;
    a.n_rows = (int64_t)L->batch * L->n_kv_heads * n_new;
    const int64_t blocks = (a.n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
    if (blocks > 0x7FFFFFFF) return fail(KVBFP_ERR_UNSUPPORTED, "quantize_append: too many rows");
    const dim3 grid((unsigned)blocks, (unsigned)nt, 1);

    // 16-byte vector loads need aligned rows; otherwise (or with a permutation) gather elementwise.
    auto aligned = [&](const void* p) {
        return p == nullptr || (((uintptr_t)p % 16 == 0) && (stride_b * esz) % 16 == 0 &&
                                (stride_t * esz) % 16 == 0 && (stride_h * esz) % 16 == 0);
    };
    const bool gather = perm_k || perm_v || !aligned(k_new) || !aligned(v_new);
    hipStream_t s = (hipStream_t)hip_stream;
    const hipError_t err = gather ? launch_quant<true>(dtype, L->mant_bits, L->block, a, grid, s)
                                  : launch_quant<false>(dtype, L->mant_bits, L->block, a, grid, s);
    if (err != hipSuccess) return fail(KVBFP_ERR_HIP, "quantize_append: %s", hipGetErrorString(err));
    return KVBFP_OK;
}

int kvbfp_dequantize(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t which, int64_t t0,
                     int64_t n_tok, const int32_t* perm, void* out, kvbfp_dtype dtype,
                     void* hip_stream) {
    clear_error();
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
    a.perm = perm; a.out = out; a.t0 = t0; a.n_tok = n_tok; a.max_seq = L->max_seq;
    a.H = L->n_kv_heads;
    a.n_rows = (int64_t)L->batch * L->n_kv_heads * n_tok;
    const int64_t blocks = (a.n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
    if (blocks > 0x7FFFFFFF) return fail(KVBFP_ERR_UNSUPPORTED, "dequantize: too many rows");
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

}  // extern "C"
