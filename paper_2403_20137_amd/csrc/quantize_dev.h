// The cast of one row to Block Floating Point (Sec. II-B, Eq. (1)) as device code shared by the
// cache-write kernel and by the decode kernel that appends the current token itself (internal).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "kvbfp.h"

namespace kvbfp {
namespace cast {

constexpr int kD = 128;           // channels per row (head_dim)

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}

// All-reduce maximum over the LPB adjacent lanes that share a block (LPB = block / 16).
// quad_perm[1,0,3,2], quad_perm[2,3,0,1], row_half_mirror: after the first two steps every quad is
// uniform, so the mirror (which swaps the two quads of a half row) completes the butterfly.
template <int LPB>
__device__ __forceinline__ uint32_t block_allmax(uint32_t a) {
    if (LPB >= 2) a = max(a, dpp_mov<0xB1>(a));
    if (LPB >= 4) a = max(a, dpp_mov<0x4E>(a));
    if (LPB >= 8) a = max(a, dpp_mov<0x141>(a));
    return a;
}

__device__ __forceinline__ float widen_bf16(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float widen_f16(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

template <int DT>
struct RawRow { uint4 v[DT == KVBFP_F32 ? 4 : 2]; };   // this lane's 16 inputs as loaded

template <int DT>
__device__ __forceinline__ void widen16(const RawRow<DT>& raw, float (&x)[16]) {
    if (DT == KVBFP_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[4 * i] = __uint_as_float(raw.v[i].x);
            x[4 * i + 1] = __uint_as_float(raw.v[i].y);
            x[4 * i + 2] = __uint_as_float(raw.v[i].z);
            x[4 * i + 3] = __uint_as_float(raw.v[i].w);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t w[4] = {raw.v[i].x, raw.v[i].y, raw.v[i].z, raw.v[i].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (DT == KVBFP_F16) {
                    x[8 * i + 2 * k] = widen_f16(w[k] & 0xFFFFu);
                    x[8 * i + 2 * k + 1] = widen_f16(w[k] >> 16);
                } else {
                    x[8 * i + 2 * k] = widen_bf16(w[k] & 0xFFFFu);
                    x[8 * i + 2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
                }
            }
        }
    }
}

// Casts the 16 values of this lane (cache positions c0..c0+15 of one row) and stores them.
// Every lane of a row group calls this (the DPP steps read neighbours); only `live` rows store.
template <int P, int N>
__device__ __forceinline__ void encode_store(const float (&x)[16], int sub, bool live, uint8_t* mant_plane,
                                             uint8_t* exp_plane, int64_t crow) {
    constexpr int LPB = N / 16;
    constexpr int NB = kD / N;
    // Largest magnitude of the block, compared on the bit patterns (monotone for finite values).
    float am = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) am = fmaxf(am, fabsf(x[i]));
    const uint32_t amax = block_allmax<LPB>(__float_as_uint(am));

    // Shared exponent byte: the fp32 exponent field of the maximum, one higher when rounding the
    // maximum to P-1 magnitude bits would carry (its top P-1 fraction bits are all ones); at least
    // 1 so that subnormal blocks use the scale of the smallest normal; 0 marks an all-zero block.
    const uint32_t bumped = (amax + (1u << (24 - P))) >> 23;
    const uint32_t E = amax == 0 ? 0u : max(bumped, 1u);

    // q[i]: a word whose low P-1 bits are the rounded magnitude; `bias` is what the other bits add
    // up to once the words are packed at P-bit spacing.
    constexpr int kPerWord = 32 / P;
    constexpr uint32_t kOnes = P == 4 ? 0x11111111u : 0x01010101u;
    uint32_t q[16];
    uint32_t bias;
    const uint32_t cfield = E + 25 - P;              // exponent field of 2^(23+e), e = E - 127 - (P-2)
    if (cfield <= 254) {
        const float C = __uint_as_float(cfield << 23);
#pragma unroll
        for (int i = 0; i < 16; ++i) q[i] = __float_as_uint(fabsf(x[i]) + C);
        bias = (cfield << 23) * kOnes;
    } else {                                         // enormous block: scale down first (exact), then round
        const int e = (int)E - 127 - (P - 2);
#pragma unroll
        for (int i = 0; i < 16; ++i) q[i] = __float_as_uint(fabsf(ldexpf(x[i], -e)) + 8388608.0f) & 0xFFu;
        bias = 0u;
    }

    uint32_t word[16 / kPerWord];
#pragma unroll
    for (int w = 0; w < 16 / kPerWord; ++w) {
        uint32_t m = 0, sg = 0;
#pragma unroll
        for (int k = 0; k < kPerWord; ++k) {
            const int i = w * kPerWord + k;
            m += q[i] << (P * k);
            sg |= (__float_as_uint(x[i]) >> 31) << (P * k + P - 1);
        }
        m -= bias;
        // the sign bit only where the magnitude is non-zero: minus zero is stored as plus zero
        const uint32_t nz = (m + (P == 4 ? 0x77777777u : 0x7F7F7F7Fu)) & (P == 4 ? 0x88888888u : 0x80808080u);
        word[w] = m | (sg & nz);
    }

    if (!live) return;
    // written once and not read back by this kernel: nontemporal stores (the bulk cast runs ~5 % faster with them)
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    if (P == 4) __builtin_nontemporal_store(u32x2_t{word[0], word[1]}, (u32x2_t*)(mant_plane + crow * 64 + sub * 8));
    else __builtin_nontemporal_store(u32x4_t{word[0], word[1], word[2], word[3]}, (u32x4_t*)(mant_plane + crow * 128 + sub * 16));
    if ((sub & (LPB - 1)) == 0) exp_plane[crow * NB + sub / LPB] = (uint8_t)E;
}

}  // namespace cast
}  // namespace kvbfp
