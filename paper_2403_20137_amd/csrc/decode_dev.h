// Device helpers shared by the matrix-core decode kernels (internal).
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "kvbfp.h"

namespace kvbfp {
namespace dev {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int kD = 128;
constexpr int kWaves = 4;
constexpr int kSuper = 64;   // tokens per wavefront iteration (4 MFMA column tiles of 16)
// The conversions produce cached values as value * 2^-kShift, with kShift chosen per mantissa width so
// that the conversion's scale operand is the stored exponent byte itself (kShift4, kShift8 in the kernel
// files).  The inverse factor rides on the other operand of each product (the query for scores, the
// probabilities for outputs), so the fp32 accumulators hold true-scale numbers: nothing is lost at either
// end of the fp32 range that the bf16 operand format can hold.

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xF, 0xF, false));
}
// all-reduce over the 16 lanes of a DPP row
__device__ __forceinline__ float row_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
__device__ __forceinline__ float row_sum(float v) {
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    return v;
}

__device__ __forceinline__ float load_as_float(const void* p, int dt, int64_t i) {
    if (dt == KVBFP_F32) return ((const float*)p)[i];
    const uint32_t h = ((const uint16_t*)p)[i];
    if (dt == KVBFP_F16) return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
    return __uint_as_float(h << 16);
}

// 2^x by the hardware instruction alone (1 ulp; results below 2^-126 come out as 0 instead of as
// denormals, which is all a softmax weight relative to the running maximum needs; 2^-inf = 0).
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 join(bf16x2 a, bf16x2 b, bf16x2 c, bf16x2 d) {
    bf16x8 r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
    r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// vector-memory operation of the wavefront, which a kernel with cache rows in flight cannot afford
// during its set-up.
__device__ __forceinline__ void lds_only_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Casts the queries in q_s[n_heads][128] (cache channel order, fp32, unscaled) to Block Floating Point
// in place: blocks of 2^log2_block channels, `bits`-bit sign-magnitude mantissas, the shared exponent
// chosen by the same rule as for cached rows (Sec. II-B, Eq. (1); Sec. III: the activations of the
// score product are BFP as well).  The decoded values are written back, so what follows is a product
// of exact small integers per block.  amax_s: n_heads * 8 words of LDS scratch.  Called by every
// thread of the workgroup after q_s is complete (barrier before); ends with a barrier (LDS only).
__device__ __forceinline__ void bfp_round_queries(float* q_s, uint32_t* amax_s, int n_heads, int log2_block, int bits) {
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int i = tid; i < n_heads * 8; i += nt) amax_s[i] = 0u;
    lds_only_barrier();
    for (int i = tid; i < n_heads * kD; i += nt)
        atomicMax(&amax_s[(i / kD) * 8 + ((i % kD) >> log2_block)], __float_as_uint(q_s[i]) & 0x7FFFFFFFu);
    lds_only_barrier();
    for (int i = tid; i < n_heads * kD; i += nt) {
        const uint32_t amax = amax_s[(i / kD) * 8 + ((i % kD) >> log2_block)];
        const uint32_t bumped = (amax + (1u << (24 - bits))) >> 23;
        const int E = amax == 0 ? 0 : (int)max(bumped, 1u);
        const int e = E - 127 - (bits - 2);
        q_s[i] = ldexpf(rintf(ldexpf(q_s[i], -e)), e);     // both scalings exact; rintf rounds to nearest even
    }
    lds_only_barrier();
}

}  // namespace dev
}  // namespace kvbfp
