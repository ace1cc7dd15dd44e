// Split pass of decode attention over keys cached BEFORE the rotary embedding, on the matrix cores
// (Alg. 1 step 5; Sec. II-D; Sec. III run-time flow: rows are fetched, rotated in the reordered channel
// order, then multiplied with the reordered query).  4-bit mantissas, 16-bit I/O, up to four query heads
// of a KV head per workgroup.
//
// The rotation is moved from the keys to the operands around them.  With q2[m] = -s'[m] q[i'[m]]
// (partner and sign vectors of the reordered pairs), the score of token t is
//     sum_m k'[m] ( q[m] cos(t Th[m]) + q2[m] sin(t Th[m]) ),
// and with t = t0 + tau (t0 = first token of a wavefront's 64-token tile, tau = 0..63)
//     = sum_m (k'[m] cos(tau Th[m])) A1[m] + (k'[m] sin(tau Th[m])) A2[m],
//     A1 = q cos(t0 Th) + q2 sin(t0 Th),   A2 = q2 cos(t0 Th) - q sin(t0 Th).
//   * cos/sin(tau Th[m]), tau < 64, never change: one table per workgroup in LDS, as two binary16 limbs
//     each: the high limb keeps 8 significant bits, so that its product with a 3-bit code is exact in
//     binary16, and the low limb carries the next 11 (products good to 2^-20 of the code).
//   * A1, A2 are rebuilt once per tile from the phasor of t0, which advances by a fixed step
//     (the phasor starts from a double-precision sine/cosine and is rotated in fp32 from tile to tile).
//   * A cached code is an integer m in [-7, 7]: it is converted to binary16 exactly, multiplied by the
//     four table limbs with packed binary16 multiplies, and the products feed
//     v_mfma_f32_16x16x32_f16 -- 3.25 vector instructions per cached key element instead of the
//     dozens a per-element rotation in fp32 takes.
//   * Block exponents are applied AFTER the matrix product, in fp32: every MFMA reduces over the 32
//     channels of one 16-byte chunk of a key row, so its result takes one power of two per
//     (token, chunk) -- the integer-mantissa products plus one exponent addition per block of Sec. II-B.
//     The query side is normalised per (head, chunk) the same way, which keeps binary16 in range for
//     every exponent byte.  For that, the four lanes that hold the four chunks of a row exchange
//     dwords (a 4 x 4 transposition with two lane-swap instructions per register pair), so that lane
//     (token j, kg) ends up with dword kg of every chunk.
//     Blocks of 16: a chunk holds two blocks; the one with the smaller exponent is scaled down by the
//     difference inside the conversion (exact down to 2^-24 of the other block's unit).
// Values, softmax and the merge of the four wavefronts are those of the register-staged plain pass.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>

#include "decode_args.h"
#include "decode_dev.h"
#include "kvbfp_internal.h"

namespace {

using kvbfp::DecodeArgs;
using namespace kvbfp::dev;

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// values: as in the plain pass, value * 2^-kShift in bf16 with the exponent byte as the scale operand
constexpr int kShift = 7;
__device__ __forceinline__ float scale_operand(uint32_t E) { return __uint_as_float(E << 23); }

// 8 sign-magnitude nibbles -> 8 numbers in slot order [c0,c2,c4,c6,c1,c3,c5,c7]: the nibble s|mmm widened
// to the byte s0000mmm is the FP8-E4M3 subnormal (-1)^s m 2^-9
__device__ __forceinline__ void spread(uint32_t w, uint32_t& lo, uint32_t& hi) {
    lo = ((w << 4) & 0x80808080u) | (w & 0x07070707u);          // even nibbles as FP8 bytes
    hi = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);          // odd nibbles
}
struct UnpackedB { bf16x2 p[4]; };
__device__ __forceinline__ UnpackedB unpack8_bf16(uint32_t w, float scale) {
    uint32_t lo, hi;
    spread(w, lo, hi);
    UnpackedB u;
    u.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, false);
    u.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, true);
    u.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, false);
    u.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, true);
    return u;
}
struct UnpackedH { f16x2 p[4]; };
__device__ __forceinline__ UnpackedH unpack8_f16(uint32_t w, float scale) {
    uint32_t lo, hi;
    spread(w, lo, hi);
    UnpackedH u;
    u.p[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lo, scale, false);
    u.p[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lo, scale, true);
    u.p[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hi, scale, false);
    u.p[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hi, scale, true);
    return u;
}
__device__ __forceinline__ int slot_channel(int x) { return (x < 4) ? 2 * x : 2 * (x - 4) + 1; }
// position of channel c in "slot order": chunk, dword, slot inside the dword
__device__ __forceinline__ int slot_index(int c) {
    const int i8 = c & 7;
    return (c & ~7) | ((i8 & 1) ? 4 + (i8 >> 1) : (i8 >> 1));
}
__device__ __forceinline__ f16x8 join_h(f16x2 a, f16x2 b, f16x2 c, f16x2 d) {
    f16x8 r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
    r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

// Lane (j, row) of a wavefront, row = lane / 16, holds M[row][r] in v[r].  Afterwards v[r] holds M[r][row]:
// first the 2 x 2 blocks are exchanged between the two halves of the wavefront, then single rows
// between neighbouring 16-lane rows.
__device__ __forceinline__ void transpose_rows(u32x4& v) {
    const auto a = __builtin_amdgcn_permlane32_swap(v[0], v[2], false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(v[1], v[3], false, false);
    const auto c = __builtin_amdgcn_permlane16_swap(a[0], b[0], false, false);
    const auto d = __builtin_amdgcn_permlane16_swap(a[1], b[1], false, false);
    v[0] = c[0]; v[1] = c[1]; v[2] = d[0]; v[3] = d[1];
}

// f(std::integral_constant<int, 0>{}) ... f(std::integral_constant<int, 3>{})
template <class F>
__device__ __forceinline__ void static_for4(F&& f) {
    f(std::integral_constant<int, 0>{}); f(std::integral_constant<int, 1>{});
    f(std::integral_constant<int, 2>{}); f(std::integral_constant<int, 3>{});
}

constexpr int kHeadStride = kD + 4;     // fp32 words per head of the normalised queries: four heads hit different banks

template <int N>
__global__ __launch_bounds__(256) void decode_split_rope_p4(DecodeArgs a, int dt) {
    constexpr int NB = kD / N;
    constexpr int NH = 4;
    // cos/sin(tau Th[m]) in binary16 limbs: 16-byte entries [chunk][cos hi|sin hi|cos lo|sin lo][kg][tau / 16][tau % 16],
    // eight slots each.  Before the table is built the same memory holds the queries in channel order, after
    // the main loop the per-wavefront outputs for the merge.
    constexpr int kKind = 4 * 4 * 16;                            // entries from one kind of limb to the next
    __shared__ __align__(16) unsigned char tab_raw[4 * 4 * kKind * 16];
    float (*q1_s)[kD] = reinterpret_cast<float (*)[kD]>(tab_raw);                // [NH][kD], scaled
    float (*q2_s)[kD] = q1_s + NH;
    __shared__ __align__(16) float q1n_s[NH * kHeadStride];      // slot order, normalised per (head, chunk)
    __shared__ __align__(16) float q2n_s[NH * kHeadStride];
    __shared__ int qe_s[NH][4];
    __shared__ __align__(16) float ph_s[kWaves][2][kD];          // phasor of each wavefront's current t0, slot order
    __shared__ float step_s[2][kD];                              // phasor of the step from a tile to the wavefront's next
    __shared__ __align__(16) uint16_t p_s[kWaves][2][4][kSuper]; // probabilities, bf16 limbs
    __shared__ float ml_s[kWaves][NH][2];
    static_assert(sizeof(tab_raw) >= sizeof(float) * kWaves * NH * kD, "the merge buffer fits the table");
    float (*o_s)[NH][kD] = reinterpret_cast<float (*)[NH][kD]>(tab_raw);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;    // scalar: tile bases stay in SGPRs
    const int j = lane & 15, kg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int h0 = kvh * a.G + a.g_base;

    int64_t L = a.seq_len ? (int64_t)a.seq_len[b] : a.max_len;
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    const int64_t t_begin = (int64_t)split * 256;
    const int64_t t_end = L;

    if (t_begin >= t_end) {
        for (int i = tid; i < a.g_cnt * kD; i += 256)
            a.part_o[(((int64_t)b * a.H_q + h0 + i / kD) * a.n_splits + split) * kD + (i % kD)] = 0.f;
        if (tid < a.g_cnt) {
            float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + tid) * a.n_splits + split) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        return;
    }

    // ---------------- set-up
    for (int i = tid; i < NH * kD; i += 256) {
        const int g = i / kD, c = i % kD;
        float v = 0.f;
        if (g < a.g_cnt) {
            const int src = a.perm_k ? (a.perm_k[kvh * kD + c] & (kD - 1)) : c;
            v = load_as_float(a.q, dt, kvbfp::query_row(a, b, kvh, a.g_base + g) * kD + src) * a.scale_log2e;
        }
        q1_s[g][c] = v;
    }
    __syncthreads();
    for (int i = tid; i < NH * kD; i += 256) {
        const int g = i / kD, c = i % kD;
        q2_s[g][c] = -a.rope_sign[kvh * kD + c] * q1_s[g][a.rope_partner[kvh * kD + c] & (kD - 1)];
    }
    __syncthreads();
    if (tid < NH * 4) {     // per (head, chunk): the power of two that brings |A1|, |A2| <= |q| + |q2| below 2^14
        const int g = tid >> 2, blk = tid & 3;
        uint32_t mx = 0u;
        for (int c = 0; c < 32; ++c) {
            mx = max(mx, __float_as_uint(q1_s[g][32 * blk + c]) & 0x7FFFFFFFu);
            mx = max(mx, __float_as_uint(q2_s[g][32 * blk + c]) & 0x7FFFFFFFu);
        }
        qe_s[g][blk] = (int)min(mx >> 23, 254u) - 139;          // mx < 2^(e - 126)  =>  |A| 2^-qe < 2^14
    }
    __syncthreads();
    for (int i = tid; i < NH * kD; i += 256) {
        const int g = i / kD, c = i % kD;
        const int e = qe_s[g][c >> 5];
        q1n_s[g * kHeadStride + slot_index(c)] = ldexpf(q1_s[g][c], -e);
        q2n_s[g * kHeadStride + slot_index(c)] = ldexpf(q2_s[g][c], -e);
    }
    __syncthreads();        // the channel-order queries give way to the table
    {
        _Float16* tab_h = reinterpret_cast<_Float16*>(tab_raw);
        for (int i = tid; i < kSuper * kD; i += 256) {
            const int tau = i >> 7, c = i & (kD - 1);
            float sn, cs;
            sincosf((float)tau * a.rope_theta[kvh * kD + c], &sn, &cs);
            const int blk = c >> 5, dw = (c >> 3) & 3, slot = slot_index(c) & 7;
            const int e16 = ((blk * 4 * 4 + dw) * 4 + (tau >> 4)) * 16 + (tau & 15);    // 16-byte entry of the cosine's high limb
            const _Float16 ch = (_Float16)(float)(__bf16)cs, sh = (_Float16)(float)(__bf16)sn;   // 8 significant bits
            tab_h[e16 * 8 + slot] = ch;
            tab_h[(e16 + kKind) * 8 + slot] = sh;
            tab_h[(e16 + 2 * kKind) * 8 + slot] = (_Float16)(cs - (float)ch);
            tab_h[(e16 + 3 * kKind) * 8 + slot] = (_Float16)(sn - (float)sh);
        }
    }
    const int64_t tile_step = (int64_t)a.n_splits * 256;
    if (tid < kD) {
        const double th = (double)a.rope_theta[kvh * kD + tid];
        const int at = slot_index(tid);
        double sn, cs;
        sincos((double)tile_step * th, &sn, &cs);
        step_s[0][at] = (float)cs;
        step_s[1][at] = (float)sn;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            sincos((double)(t_begin + w * kSuper) * th, &sn, &cs);
            ph_s[w][0][at] = (float)cs;
            ph_s[w][1][at] = (float)sn;
        }
    }
    __syncthreads();

    // this lane's rows of every score MFMA belong to head kg
    int qe[4];
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) qe[blk] = qe_s[kg][blk];

    const int a_head = j >> 2, a_par = (j >> 1) & 1, a_limb = j & 1;
    const uint32_t sel_even = a_par ? 0x01000c0cu : 0x0c0c0100u;
    const uint32_t sel_odd = a_par ? 0x03020c0cu : 0x0c0c0302u;

    const int64_t base = ((int64_t)b * a.H_kv + kvh) * a.max_seq + t_begin;
    const uint8_t* __restrict__ k_mant = a.k_mant + base * 64;
    const uint8_t* __restrict__ v_mant = a.v_mant + base * 64;
    const uint8_t* __restrict__ k_exp = a.k_exp + base * NB;
    const uint8_t* __restrict__ v_exp = a.v_exp + base * NB;
    const int n_tok = (int)(t_end - t_begin);

    float m_run = -INFINITY, l_run = 0.f;
    f32x4 o_acc[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) o_acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint4* tab = reinterpret_cast<const uint4*>(tab_raw);

    // The rows of one 64-token tile as this lane loads them: key chunk kg of rows 16u + j with the row's
    // exponent bytes, requested before the tile's query operands are built; value dword j of rows
    // 16u + 4kg + i with that dword's exponent byte, requested before the score phase.
    struct KeyRows {
        u32x4 kw[4];
        uint32_t kex[4][N == 16 ? 2 : 1];
    };
    struct ValueRows {
        uint32_t vw[16];
        uint32_t vex[16];
    };
    auto fetch = [&](const int T0, auto full_tag, KeyRows& d) {
        constexpr bool FULL = decltype(full_tag)::value;
        const size_t R0 = (size_t)T0;   // wave-uniform
        const uint8_t* __restrict__ kp = k_mant + R0 * 64;
        const uint8_t* __restrict__ kep = k_exp + R0 * NB;
        const int left = n_tok - T0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t r = FULL ? (uint32_t)(16 * u + j) : (uint32_t)min(16 * u + j, left - 1);
            d.kw[u] = __builtin_nontemporal_load((const u32x4*)(kp + r * 64u + (uint32_t)kg * 16u));
            if constexpr (N == 16) {
                const u32x2 e2 = *(const u32x2*)(kep + r * 8u);
                d.kex[u][0] = e2[0]; d.kex[u][1] = e2[1];
            } else if constexpr (N == 32) {
                d.kex[u][0] = *(const uint32_t*)(kep + r * 4u);
            } else if constexpr (N == 64) {
                d.kex[u][0] = *(const uint16_t*)(kep + r * 2u);
            } else {
                d.kex[u][0] = kep[r];
            }
        }
    };

    auto tile = [&](const int T0, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const int left = n_tok - T0;
        KeyRows d;
        fetch(T0, full_tag, d);          // the operand build below covers part of the wait
        // ---------------- the tile's query operands: row j = 4 * head + limb, two binary16 limbs (rows of limb 0, 1;
        // what sits in the rows of limb 2, 3 never reaches a score).  The four lanes of a head and lane group share
        // the work: lane `limb` builds both limbs of chunk `limb`, and the quad exchanges them -- the rows of
        // even limbs take the high limb of every chunk, those of odd limbs the low one.
        f16x8 A1[4], A2[4];
        {
            const int gi = j >> 2, limb = j & 3;
            const int at = limb * 32 + kg * 8;
            float x[8], y[8], c0[8], s0[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 xv = *(const float4*)&q1n_s[gi * kHeadStride + at + 4 * h];
                const float4 yv = *(const float4*)&q2n_s[gi * kHeadStride + at + 4 * h];
                const float4 cv = *(const float4*)&ph_s[wave][0][at + 4 * h];
                const float4 sv = *(const float4*)&ph_s[wave][1][at + 4 * h];
                x[4 * h] = xv.x; x[4 * h + 1] = xv.y; x[4 * h + 2] = xv.z; x[4 * h + 3] = xv.w;
                y[4 * h] = yv.x; y[4 * h + 1] = yv.y; y[4 * h + 2] = yv.z; y[4 * h + 3] = yv.w;
                c0[4 * h] = cv.x; c0[4 * h + 1] = cv.y; c0[4 * h + 2] = cv.z; c0[4 * h + 3] = cv.w;
                s0[4 * h] = sv.x; s0[4 * h + 1] = sv.y; s0[4 * h + 2] = sv.z; s0[4 * h + 3] = sv.w;
            }
            uint32_t hi1[4], lo1[4], hi2[4], lo2[4];      // this lane's chunk: A1 and A2, high and low limbs, two slots per register
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                const f32x2 a1 = {fmaf(x[i], c0[i], y[i] * s0[i]), fmaf(x[i + 1], c0[i + 1], y[i + 1] * s0[i + 1])};
                const f32x2 a2 = {fmaf(y[i], c0[i], -(x[i] * s0[i])), fmaf(y[i + 1], c0[i + 1], -(x[i + 1] * s0[i + 1]))};
                // high limb = the value cut to binary16 (one pack instruction for two values), low limb = what is left,
                // cut again: the pair carries 22 bits whichever way each part is rounded
                const f16x2 h1 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(a1[0], a1[1]));
                const f16x2 h2 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(a2[0], a2[1]));
                const f32x2 r1 = a1 - __builtin_convertvector(h1, f32x2), r2 = a2 - __builtin_convertvector(h2, f32x2);
                hi1[i / 2] = __builtin_bit_cast(uint32_t, h1);
                hi2[i / 2] = __builtin_bit_cast(uint32_t, h2);
                lo1[i / 2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r1[0], r1[1]));
                lo2[i / 2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r2[0], r2[1]));
            }
            // Lane `blk` of the quad built chunk blk.  Its low limb first goes to the neighbour lane blk ^ 1, so that one
            // register holds the high limb in one lane of the pair and the low limb in the other; a quad permute
            // [blk, blk^1, blk, blk^1] then hands the high limb to the even lanes and the low limb to the odd ones.
            const bool odd = (limb & 1) != 0;
            uint32_t ze1[4], zo1[4], ze2[4], zo2[4];       // for even / odd blk
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t x1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo1[r], 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
                const uint32_t x2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo2[r], 0xB1, 0xF, 0xF, false);
                ze1[r] = odd ? x1 : hi1[r];
                zo1[r] = odd ? hi1[r] : x1;
                ze2[r] = odd ? x2 : hi2[r];
                zo2[r] = odd ? hi2[r] : x2;
            }
            static_for4([&](auto BLK) {
                constexpr int blk = decltype(BLK)::value;
                constexpr int ctrl = blk | ((blk ^ 1) << 2) | (blk << 4) | ((blk ^ 1) << 6);
                uint32_t p1[4], p2[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p1[r] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)((blk & 1) ? zo1[r] : ze1[r]), ctrl, 0xF, 0xF, false);
                    p2[r] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)((blk & 1) ? zo2[r] : ze2[r]), ctrl, 0xF, 0xF, false);
                }
                A1[blk] = __builtin_bit_cast(f16x8, u32x4{p1[0], p1[1], p1[2], p1[3]});
                A2[blk] = __builtin_bit_cast(f16x8, u32x4{p2[0], p2[1], p2[2], p2[3]});
            });
            // everybody has read the phasor of this tile: advance it to the wavefront's next tile
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e = lane + 64 * h;
                const float c = ph_s[wave][0][e], s = ph_s[wave][1][e];
                const float dc = step_s[0][e], ds = step_s[1][e];
                ph_s[wave][0][e] = fmaf(c, dc, -(s * ds));
                ph_s[wave][1][e] = fmaf(s, dc, c * ds);
            }
        }

        ValueRows dv;
        {
            const size_t R0 = (size_t)T0;   // wave-uniform
            const uint8_t* __restrict__ vp = v_mant + R0 * 64;
            const uint8_t* __restrict__ vep = v_exp + R0 * NB;
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t r = FULL ? (uint32_t)(16 * u + 4 * kg + i) : (uint32_t)min(16 * u + 4 * kg + i, left - 1);
                    dv.vw[4 * u + i] = __builtin_nontemporal_load((const uint32_t*)(vp + r * 64u + 4u * (uint32_t)j));
                    dv.vex[4 * u + i] = vep[r * NB + (uint32_t)((8 * j) / N)];
                }
        }

        // ---------------- scores of 64 tokens: sixteen (stage u, chunk blk) steps; the table entries of a step
        // are read one step ahead, and the scheduling barriers keep later reads from piling up in registers
        float s[4];
        {
            uint4 tb[2][4];
            auto read_table = [&](const int c, uint4 (&t)[4]) {
                const int e16 = (((c & 3) * 4 * 4 + kg) * 4 + (c >> 2)) * 16 + j;
#pragma unroll
                for (int kind = 0; kind < 4; ++kind) t[kind] = tab[e16 + kind * kKind];     // cos hi, sin hi, cos lo, sin lo
            };
            read_table(0, tb[0]);
            u32x4 w = {0u, 0u, 0u, 0u};
            float acc_s = 0.f;
            // the partial sums of a step are picked up one step later, when its MFMAs have long finished
            f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
            float post_scale[2] = {0.f, 0.f};
            auto finish = [&](const int c) {                // step c: scale by the powers of two, add, close a stage
                const int u = c >> 2, blk = c & 3;
                if (blk == 0) acc_s = 0.f;
                acc_s = fmaf(acc[c & 1][0] + acc[c & 1][1], post_scale[c & 1], acc_s);
                if (blk == 3) s[u] = (FULL || 16 * u + j < left) ? acc_s : -INFINITY;
            };
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                const int u = c >> 2, blk = c & 3;
                if (c + 1 < 16) read_table(c + 1, tb[(c + 1) & 1]);
                const uint32_t* ex = d.kex[u];      // the row's exponent bytes
                if (blk == 0) {
                    w = d.kw[u];
                    transpose_rows(w);              // w[blk] = dword kg of chunk blk: channels 32 blk + 8 kg ..+7
                }
                uint32_t Ec;
                float cvt_scale = 512.0f;           // FP8 subnormal m 2^-9 -> the integer m
                if (N == 16) {
                    const uint32_t pair = (ex[N == 16 ? (blk >> 1) : 0] >> (16 * (blk & 1))) & 0xFFFFu;
                    const uint32_t e0 = pair & 0xFFu, e1 = pair >> 8;
                    Ec = max(e0, e1);
                    const uint32_t dd = min(Ec - (kg < 2 ? e0 : e1), 40u);
                    cvt_scale = __uint_as_float((136u - dd) << 23);
                } else if (N == 32) {
                    Ec = (ex[0] >> (8 * blk)) & 0xFFu;
                } else if (N == 64) {
                    Ec = (ex[0] >> (8 * (blk >> 1))) & 0xFFu;
                } else {
                    Ec = ex[0];
                }
                const UnpackedH m = unpack8_f16(w[blk], cvt_scale);
                f32x4 a4 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kind = 0; kind < 4; ++kind) {
                    const uint4 t = tb[c & 1][kind];
                    const f16x8 kt = join_h(m.p[0] * __builtin_bit_cast(f16x2, t.x), m.p[1] * __builtin_bit_cast(f16x2, t.y),
                                            m.p[2] * __builtin_bit_cast(f16x2, t.z), m.p[3] * __builtin_bit_cast(f16x2, t.w));
                    a4 = __builtin_amdgcn_mfma_f32_16x16x32_f16((kind & 1) ? A2[blk] : A1[blk], kt, a4, 0, 0, 0);
                }
                acc[c & 1] = a4;
                // code m of exponent byte E is m 2^(E - 129); the query was divided by 2^qe
                const int F = min(max((int)Ec + qe[blk] - 2, 0), 254);
                post_scale[c & 1] = __uint_as_float((uint32_t)F << 23);
                if (c > 0) finish(c - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            finish(15);
        }

        // ---------------- online softmax; lane (j, kg) owns head kg, tokens 16u + j
        {
            float tmax = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
            tmax = row_max(tmax);
            const float m_new = fmaxf(m_run, tmax);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = exp2_raw(m_run - m_ref);
            const float m_p = m_ref - (float)kShift;
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float pw = exp2_raw(s[u] - m_p);
                const __bf16 ph = (__bf16)pw;
                const float r1 = pw - (float)ph;
                const __bf16 pl = (__bf16)r1;
                p_s[wave][0][kg][16 * u + j] = __builtin_bit_cast(unsigned short, ph);
                p_s[wave][1][kg][16 * u + j] = __builtin_bit_cast(unsigned short, pl);
                psum += (float)ph + (float)pl;
            }
            l_run = l_run * alpha + psum;
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int m = 0; m < 4; ++m) o_acc[m] *= alpha;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---------------- values of the same 64 tokens: lane (j, kg) takes dword j of rows 4kg .. 4kg+3
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            UnpackedB vv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) vv[i] = unpack8_bf16(dv.vw[4 * u + i], scale_operand(dv.vex[4 * u + i]));
            uint2 pp = *(const uint2*)&p_s[wave][a_limb][a_head][16 * u + 4 * kg];
            uint32_t ar[4];
            ar[0] = __builtin_amdgcn_perm(pp.x, pp.x, sel_even);
            ar[1] = __builtin_amdgcn_perm(pp.x, pp.x, sel_odd);
            ar[2] = __builtin_amdgcn_perm(pp.y, pp.y, sel_even);
            ar[3] = __builtin_amdgcn_perm(pp.y, pp.y, sel_odd);
            const bf16x8 ap = __builtin_bit_cast(bf16x8, u32x4{ar[0], ar[1], ar[2], ar[3]});
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const bf16x8 bv = join(vv[0].p[m], vv[1].p[m], vv[2].p[m], vv[3].p[m]);
                o_acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, bv, o_acc[m], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    {
        int T0 = wave * kSuper;
        const int step = a.n_splits * kWaves * kSuper;
        for (; T0 + kSuper <= n_tok; T0 += step) tile(T0, std::true_type{});
        if (T0 < n_tok) tile(T0, std::false_type{});     // at most one ragged tile per wavefront
    }

    // ---------------- per-wavefront result to LDS (nobody needs the table any more after the barrier)
    __syncthreads();
    {
        const float lsum = row_sum(l_run);
        const int head = kg;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int c_even = 8 * j + slot_channel(2 * m);
            const int c_odd = 8 * j + slot_channel(2 * m + 1);
            o_s[wave][head][c_even] = o_acc[m][0] + o_acc[m][1];
            o_s[wave][head][c_odd] = o_acc[m][2] + o_acc[m][3];
        }
        if (j == 0) {
            ml_s[wave][head][0] = m_run;
            ml_s[wave][head][1] = lsum * (1.0f / (float)(1 << kShift));
        }
    }
    __syncthreads();

    for (int i = tid; i < a.g_cnt * kD; i += 256) {
        const int g = i / kD, c = i % kD;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, ml_s[w][g][0]);
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = ml_s[w][g][0];
            if (mw > -INFINITY) acc = fmaf(exp2f(mw - M), o_s[w][g][c], acc);
        }
        a.part_o[(((int64_t)b * a.H_q + h0 + g) * a.n_splits + split) * kD + c] = acc;
    }
    if (tid < a.g_cnt) {
        const int g = tid;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, ml_s[w][g][0]);
        float lsum = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = ml_s[w][g][0];
            if (mw > -INFINITY) lsum = fmaf(exp2f(mw - M), ml_s[w][g][1], lsum);
        }
        float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + g) * a.n_splits + split) * 2;
        ml[0] = M;
        ml[1] = lsum;
    }
}

hipError_t launch_rope(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    if (block == 16) decode_split_rope_p4<16><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 32) decode_split_rope_p4<32><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 64) decode_split_rope_p4<64><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 128) decode_split_rope_p4<128><<<grid, 256, 0, s>>>(a, dt);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

namespace kvbfp {

// 4-bit mantissas, 16-bit I/O, contiguous cache, a.g_cnt <= 4 heads [a.g_base, a.g_base + a.g_cnt) of every KV
// head per launch.
hipError_t launch_decode_split_rope(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s) {
    if (dtype == KVBFP_F32 || a.g_cnt > 4 || a.block_table || !a.rope_theta || !a.rope_partner || !a.rope_sign)
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)a.n_splits, (unsigned)a.H_kv, (unsigned)batch);
    return launch_rope(a, dtype, block, grid, s);
}

}  // namespace kvbfp
