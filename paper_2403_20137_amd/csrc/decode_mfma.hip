// Fast split pass of decode attention for 4-bit mantissas on gfx950 (Sec. III run-time flow).
//
// Why matrix cores: with G query heads sharing one KV head, a cached element takes 2*G multiply-
// adds but arrives at 0.53 bytes.  At 8 TB/s the vector ALUs (64 lanes x 4 SIMDs x 256 CUs, one
// fp32 op per lane per clock without packed math) can spend about 2.5 instructions per element;
// unpacking a sign-magnitude nibble costs >= 1.25 of them, which leaves no room for even G = 1
// worth of dot2 instructions at full bandwidth, let alone G = 4.  The skinny products
// (G x 128) . (128 x T) and (G x T) . (T x 128) therefore go to the MFMA pipe, which is otherwise
// idle, and the vector ALUs only unpack.
//
// Unpacking without integer->float conversions: a code s|mmm widened to the byte s0000mmm is the
// OCP FP8-E4M3 subnormal (-1)^s * m * 2^-9, so v_cvt_scalef32_pk_bf16_fp8 turns two codes into
// two exact bf16 values and applies the block's power-of-two scale in the same instruction.
// Cost per 8 codes: 6 bit operations + 4 conversions.
//
// Score product  S = Q . K^T  (v_mfma_f32_16x16x32_bf16, A = query rows, B = keys):
//   lane (j = lane%16, kg = lane/16) loads the 16-byte chunk kg of the key row of token j
//   (32 channels, i.e. whole blocks) and feeds it to 4 MFMAs; A holds the query split into three
//   bf16 limbs (24 significant bits) in rows 4*head + limb, so the product keeps fp32 accuracy.
// Value product  O = P . V  (same instruction, A = probabilities, B = values):
//   the reduction index enumerates (token, channel parity): a converted register already holds
//   the two channels of one token, and the probabilities sit in rows (head, parity, limb) with
//   zeros in the other parity's slots, so no transposition of the 4-bit data is ever needed.
//   Lane (j, kg) loads dword j (8 channels) of the value rows of tokens 4kg..4kg+3.
// Each wavefront owns every fourth 64-token tile of its split and keeps its own online-softmax
// state; the four wavefronts of a workgroup merge once at the end.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>
#include <utility>

#include "decode_args.h"
#include "decode_dev.h"
#include "kvbfp_internal.h"
#include "quantize_dev.h"

namespace {

using kvbfp::DecodeArgs;

using namespace kvbfp::dev;

// A code m of a block with exponent byte E stands for m * 2^(E - 129).  Read as the FP8 subnormal
// m * 2^-9 and converted with the scale operand 2^(E - 127) -- the byte E itself in the exponent field,
// which is all the conversion looks at -- it becomes the bf16 value m * 2^(E - 136) = value * 2^-kShift,
// exact for every E >= 3 (bf16 keeps denormals down to 2^-133; blocks with E = 1, 2, magnitudes below
// 2^-124, lose low-order bits, an absolute error under 2^-126).  E = 255 (a block maximum within a
// factor 1.07 of the largest fp32 number) would read as an infinite scale and is not supported here.
constexpr int kShift = 7;
__device__ __forceinline__ float scale_operand(uint32_t E) { return __uint_as_float(E << 23); }

// 8 sign-magnitude nibbles -> 8 bf16 values in slot order [c0,c2,c4,c6,c1,c3,c5,c7]
struct Unpacked { bf16x2 p[4]; };
__device__ __forceinline__ Unpacked unpack8(uint32_t w, float scale) {
    const uint32_t lo = ((w << 4) & 0x80808080u) | (w & 0x07070707u);          // even nibbles as FP8 bytes
    const uint32_t hi = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);          // odd nibbles
    Unpacked u;
    u.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, false);      // (c0, c2)
    u.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, true);       // (c4, c6)
    u.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, false);      // (c1, c3)
    u.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, true);       // (c5, c7)
    return u;
}
// channel offset inside a dword of MFMA slot x
__device__ __forceinline__ int slot_channel(int x) { return (x < 4) ? 2 * x : 2 * (x - 4) + 1; }

// N = block size, HG = groups of four query heads per KV head (G <= 4*HG).
// grid = (n_splits, H_kv, B), block = 256 (four wavefronts).
// PL = bf16 limbs of a probability: 2 (16 bits, enough for 16-bit outputs) or 3 (24 bits, fp32 outputs).
// PAGED: the planes are a pool of pages and every tile looks up its page (a separate instantiation: the
// contiguous case keeps its 32-bit offsets from one scalar base).
template <int N, int HG, int PL, bool PAGED>
__global__ __launch_bounds__(256) void decode_split_mfma_p4(DecodeArgs a, int dt) {
    constexpr int NB = kD / N;
    constexpr int NH = HG * 4;
    __shared__ float q_s[NH][kD];                               // scaled, permuted queries
    __shared__ __align__(16) uint16_t p_s[kWaves][HG][PL][4][kSuper];  // probabilities, bf16 limbs
    __shared__ float o_s[kWaves][NH][kD];                       // per-wavefront outputs for the merge
    __shared__ float ml_s[kWaves][NH][2];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int j = lane & 15, kg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int h0 = kvh * a.G + a.g_base;      // first (virtual) head of this launch

    int64_t L = a.seq_len ? (int64_t)a.seq_len[b] : a.max_len;
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    // 256-token tiles are dealt out round-robin: split s takes tiles s, s + n_splits, s + 2 n_splits, ...;
    // "split-relative" tokens below count from t_begin
    const int64_t t_begin = (int64_t)split * 256;
    const int64_t t_end = L;

    if (t_begin >= t_end) {   // nothing cached in this split
        for (int i = tid; i < a.g_cnt * kD; i += 256)
            a.part_o[(((int64_t)b * a.H_q + h0 + i / kD) * a.n_splits + split) * kD + (i % kD)] = 0.f;
        if (tid < a.g_cnt) {
            float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + tid) * a.n_splits + split) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        return;
    }

    // q' = permuted query (optionally cast to BFP) * softmax_scale*log2(e) * 2^kShift; head slots beyond G are zero
    {
        const float two_k = (float)(1 << kShift);
        for (int i = tid; i < NH * kD; i += 256) {
            const int g = i / kD, c = i % kD;
            float v = 0.f;
            if (g < a.g_cnt) {
                const int src = a.perm_k ? (a.perm_k[kvh * kD + c] & (kD - 1)) : c;
                v = load_as_float(a.q, dt, kvbfp::query_row(a, b, kvh, a.g_base + g) * kD + src);
            }
            q_s[g][c] = a.q_mant_bits ? v : (v * a.scale_log2e) * two_k;
        }
        __syncthreads();
        if (a.q_mant_bits) {
            bfp_round_queries(&q_s[0][0], (uint32_t*)&o_s[0][0][0], NH, a.log2_block, a.q_mant_bits);
            for (int i = tid; i < NH * kD; i += 256) (&q_s[0][0])[i] = ((&q_s[0][0])[i] * a.scale_log2e) * two_k;
            __syncthreads();
        }
    }

    // A operands of the score product: row r = lane%16 = 4*head + limb, k-slot (kg, x) of MFMA d
    // is channel 32*kg + 8*d + slot_channel(x).
    bf16x8 aq[HG][4];
    {
        const int gi = j >> 2, limb = j & 3;
#pragma unroll
        for (int hg = 0; hg < HG; ++hg)
#pragma unroll
            for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const float f = q_s[hg * 4 + gi][32 * kg + 8 * d + slot_channel(x)];
                    const __bf16 l0 = (__bf16)f;
                    const float r1 = f - (float)l0;
                    const __bf16 l1 = (__bf16)r1;
                    const float r2 = r1 - (float)l1;
                    const __bf16 l2 = (__bf16)r2;
                    aq[hg][d][x] = limb == 0 ? l0 : (limb == 1 ? l1 : (limb == 2 ? l2 : (__bf16)0.0f));
                }
    }

    // selectors that place a probability in the low (parity 0) or high (parity 1) half of an
    // A register of the value product; row r = j = 4*head + 2*parity + limb
    const int a_head = j >> 2, a_par = (j >> 1) & 1, a_limb = j & 1;
    const uint32_t sel_even = a_par ? 0x01000c0cu : 0x0c0c0100u;   // halfword 0 of the source
    const uint32_t sel_odd = a_par ? 0x03020c0cu : 0x0c0c0302u;    // halfword 1 of the source

    // Plane bases of this (batch, kv-head) are wave-uniform (scalar registers); everything inside
    // the split is addressed with 32-bit offsets from them.
    // (Paged cache: the bases are those of the pool and every tile looks up its page.)
    const int64_t base = PAGED ? 0 : ((int64_t)b * a.H_kv + kvh) * a.max_seq + t_begin;
    const uint8_t* __restrict__ k_mant = a.k_mant + base * 64;
    const uint8_t* __restrict__ v_mant = a.v_mant + base * 64;
    const uint8_t* __restrict__ k_exp = a.k_exp + base * NB;
    const uint8_t* __restrict__ v_exp = a.v_exp + base * NB;
    const int n_tok = (int)(t_end - t_begin);       // tokens from this split's first tile to the end of the sequence
    // several query tokens: head slot s sees tokens below lim[.] only (split-relative), and a tile counts
    // as full only if every head sees all of it
    const int n_vis = (int)(L - t_begin);
    const int n_full = min(n_tok, n_vis - (a.n_q_tokens - 1));
    int lim[HG];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) lim[hg] = n_vis - kvbfp::hidden_tokens(a, a.g_base + hg * 4 + kg);

    float m_run[HG], l_run[HG];
    f32x4 o_acc[HG][4];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        m_run[hg] = -INFINITY;
        l_run[hg] = 0.f;
#pragma unroll
        for (int m = 0; m < 4; ++m) o_acc[hg][m] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Per-lane byte offsets inside a 64-token tile; the tile's base pointers are wave-uniform, so a
    // load is (scalar base) + (this lane offset) + (compile-time constant).
    const uint32_t koff = (uint32_t)j * 64u + (uint32_t)kg * 16u;                       // key row j, chunk kg
    const uint32_t keoff = (uint32_t)j * NB + (N == 16 ? 2u * kg : (N == 32 ? (uint32_t)kg : (N == 64 ? (uint32_t)(kg >> 1) : 0u)));
    const uint32_t voff = (uint32_t)(4 * kg) * 64u + 4u * (uint32_t)j;                  // value rows 4kg.., dword j
    const uint32_t veoff = (uint32_t)(4 * kg) * NB + (uint32_t)((8 * j) / N);

    // One 64-token tile starting at token T0 of the split.  FULL: all 64 tokens are cached, no
    // clamping or masking; otherwise rows are clamped to the last cached token and masked.
    auto tile = [&](const int T0, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const size_t R0 = PAGED ? (size_t)kvbfp::cache_row(a, b, kvh, t_begin + T0) : (size_t)T0;   // wave-uniform
        const uint8_t* __restrict__ kp = k_mant + R0 * 64;
        const uint8_t* __restrict__ vp = v_mant + R0 * 64;
        const uint8_t* __restrict__ kep = k_exp + R0 * NB;
        const uint8_t* __restrict__ vep = v_exp + R0 * NB;
        const int left = n_tok - T0;                 // cached tokens from T0 on (>= 1)

        // ---------------- scores of 64 tokens
        f32x4 s_acc[HG][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t mo, eo;
            if (FULL) {
                mo = koff + 1024u * u;
                eo = keoff + 16u * NB * u;
            } else {
                const uint32_t r = (uint32_t)min(16 * u + j, left - 1);
                mo = r * 64u + (uint32_t)kg * 16u;
                eo = r * NB + (keoff - (uint32_t)j * NB);
            }
            const u32x4 raw = __builtin_nontemporal_load((const u32x4*)(kp + mo));   // streamed once: keep it out of the caches' way
            float sc0, sc1;
            if (N == 16) {
                const uint32_t e2 = *(const uint16_t*)(kep + eo);
                sc0 = scale_operand(e2 & 0xFFu);
                sc1 = scale_operand(e2 >> 8);
            } else {
                sc0 = sc1 = scale_operand(kep[eo]);
            }
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) s_acc[hg][u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const Unpacked kk = unpack8(raw[d], d < 2 ? sc0 : sc1);
                const bf16x8 bk = join(kk.p[0], kk.p[1], kk.p[2], kk.p[3]);
#pragma unroll
                for (int hg = 0; hg < HG; ++hg)
                    s_acc[hg][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[hg][d], bk, s_acc[hg][u], 0, 0, 0);
            }
        }

        // ---------------- online softmax; lane (j, kg) owns head kg of each group, tokens 16u + j
#pragma unroll
        for (int hg = 0; hg < HG; ++hg) {
            float s[4];
            float tmax = -INFINITY;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float v = s_acc[hg][u][0] + s_acc[hg][u][1] + s_acc[hg][u][2];   // the three limbs
                s[u] = (FULL || 16 * u + j < min(left, lim[hg] - T0)) ? v : -INFINITY;
                tmax = fmaxf(tmax, s[u]);
            }
            tmax = row_max(tmax);           // -inf only if this head sees none of the tile (several query tokens)
            const float m_new = fmaxf(m_run[hg], tmax);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;   // keeps the differences below well defined
            const float alpha = exp2_raw(m_run[hg] - m_ref);           // 0 on the first tile, 1 when the maximum stays
            const float m_p = m_ref - (float)kShift;                    // probabilities carry 2^kShift (values come as 2^-kShift)
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float pw = exp2_raw(s[u] - m_p);
                const __bf16 ph = (__bf16)pw;
                const float r1 = pw - (float)ph;
                const __bf16 pl = (__bf16)r1;
                p_s[wave][hg][0][kg][16 * u + j] = __builtin_bit_cast(unsigned short, ph);
                p_s[wave][hg][1][kg][16 * u + j] = __builtin_bit_cast(unsigned short, pl);
                if (PL == 3) {
                    const __bf16 p3 = (__bf16)(r1 - (float)pl);
                    p_s[wave][hg][PL - 1][kg][16 * u + j] = __builtin_bit_cast(unsigned short, p3);
                    psum += ((float)ph + (float)pl) + (float)p3;
                } else {
                    psum += (float)ph + (float)pl;
                }
            }
            l_run[hg] = l_run[hg] * alpha + psum;                   // per-lane partial; summed at the end
            m_run[hg] = m_new;
            // Rescale the running output only when some head's maximum moved (exact: alpha == 1
            // otherwise).  The accumulators sit in the MFMA result registers, so skipping saves the
            // round trip.  This lane's rows all belong to head kg.
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int m = 0; m < 4; ++m) o_acc[hg][m] *= alpha;
            }
        }

        // the probabilities just written are read back below by other lanes of this wavefront
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---------------- values of the same 64 tokens
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            Unpacked vv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t mo, eo;
                if (FULL) {
                    mo = voff + 64u * (16 * u + i);
                    eo = veoff + NB * (16 * u + i);
                } else {
                    const uint32_t r = (uint32_t)min(16 * u + 4 * kg + i, left - 1);
                    mo = r * 64u + 4u * (uint32_t)j;
                    eo = r * NB + (uint32_t)((8 * j) / N);
                }
                const uint32_t w = __builtin_nontemporal_load((const uint32_t*)(vp + mo));
                vv[i] = unpack8(w, scale_operand(vep[eo]));
            }
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) {
                // probabilities of tokens 16u + 4kg .. +3 for this lane's row (head, parity, limb); a third
                // limb takes a second round with that limb in the rows of limb 0 and zeros in the others
#pragma unroll
                for (int round = 0; round < (PL == 3 ? 2 : 1); ++round) {
                    uint2 pp = *(const uint2*)&p_s[wave][hg][round == 0 ? a_limb : PL - 1][a_head][16 * u + 4 * kg];
                    if (round == 1 && a_limb == 1) pp = make_uint2(0u, 0u);
                    uint32_t ar[4];
                    ar[0] = __builtin_amdgcn_perm(pp.x, pp.x, sel_even);
                    ar[1] = __builtin_amdgcn_perm(pp.x, pp.x, sel_odd);
                    ar[2] = __builtin_amdgcn_perm(pp.y, pp.y, sel_even);
                    ar[3] = __builtin_amdgcn_perm(pp.y, pp.y, sel_odd);
                    const bf16x8 ap = __builtin_bit_cast(bf16x8, u32x4{ar[0], ar[1], ar[2], ar[3]});
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const bf16x8 bv = join(vv[0].p[m], vv[1].p[m], vv[2].p[m], vv[3].p[m]);
                        o_acc[hg][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, bv, o_acc[hg][m], 0, 0, 0);
                    }
                }
            }
        }
        // the next tile overwrites the probability buffer
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    {
        int T0 = wave * kSuper;
        const int step = a.n_splits * kWaves * kSuper;      // this workgroup's next 256-token tile
        for (; T0 + kSuper <= n_full; T0 += step) tile(T0, std::true_type{});
        if (T0 < n_tok) tile(T0, std::false_type{});     // at most one ragged tile per wavefront
    }

    // ---------------- per-wavefront result to LDS: lane (j, kg) holds head kg, channels 8j..8j+7
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        const float lsum = row_sum(l_run[hg]);
        const int head = hg * 4 + kg;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            // rows (parity 0: hi, lo), (parity 1: hi, lo); MFMA m holds slots (m) -> channels below
            const int c_even = 8 * j + slot_channel(2 * m);       // parity 0 channel of pair m
            const int c_odd = 8 * j + slot_channel(2 * m + 1);    // parity 1 channel of pair m
            o_s[wave][head][c_even] = o_acc[hg][m][0] + o_acc[hg][m][1];
            o_s[wave][head][c_odd] = o_acc[hg][m][2] + o_acc[hg][m][3];
        }
        if (j == 0) {
            ml_s[wave][head][0] = m_run[hg];
            ml_s[wave][head][1] = lsum * (1.0f / (float)(1 << kShift));      // the probabilities carried 2^kShift
        }
    }
    __syncthreads();

    // ---------------- merge the four wavefronts, write this split's partial result
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


// ------------------------------------------------------------------------------------------------
// LDS-staged pass (blocks of 16 and 32, the default for them): the packed rows travel
// global -> LDS by DMA (global_load_lds) instead of through registers, so every wavefront keeps
// most of a 64-token tile in flight without holding registers for it.  Values are unpacked as
// above; keys are not unpacked at all: the raw nibbles are the FP4 operand of the scaled
// FP8 x FP4 MFMA (v_mfma_scale_f32_16x16x128_f8f6f4), the block exponent byte is its E8M0 scale,
// and the query is four FP8 limbs with a power-of-two scale per 32 channels.
//
// Each wavefront owns a private staging area of four 16-token stages for keys and four for values
// (mantissas 1 KB + exponent bytes per stage).  A stage is re-filled for the wavefront's next tile
// right after its last read, in the fixed order K0..K3, V0..V3, two DMA instructions per stage.
// DMA completes in issue order, so when a stage is about to be read exactly seven younger stages
// (14 instructions) may still be outstanding: one s_waitcnt vmcnt(14) per stage is the whole
// synchronisation (vmcnt(0) once nothing is being re-filled any more).  The compiler does not
// model the DMA -> ds_read dependency, hence the explicit waits and scheduling barriers; the main
// loop contains no other vector-memory instruction.
//
// Key stage: DMA lane 4r+c fetches chunk c ^ (r/4 % 4) of row r (four neighbouring lanes cover one
// 64-byte row, so the global access coalesces like a linear copy); lane (j, kg) then reads slot
// 4j + (kg ^ (j/4 % 4)), which spreads every group of 16 lanes over all banks.  Value stage: the 16 rows are stored in the order 4*(row%4) + row/4, which makes the
// dword reads of lanes (j, kg) -> row 4kg+i, dword j hit 64 different banks.
#define KVBFP_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define KVBFP_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

// LDS byte address of a pointer into __shared__ memory.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(unsigned long)(__attribute__((address_space(3))) const uint8_t*)p;
}

// Reads of DMA-staged data are written in assembly: the compiler's wait-count pass half-knows about
// LDS DMA and would otherwise put a full vmcnt(0) in front of some of these loads, which serialises
// the whole pipeline.  They come as issue / wait pairs for the software pipeline of the main loop: the
// registers named at the issue are written when the LDS answers; the wait comes before their first use
// and names them again, so that the compiler keeps them where they are in between.
template <int OFF>
__device__ __forceinline__ void lds_issue_b128(uint32_t addr, u32x4& v) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_issue_b64(uint32_t addr, uint64_t& v) {
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=&v"(v) : "v"(addr), "n"(OFF) : "memory");
}
// four reads of one or two bytes, STRIDE apart
template <int OFF, int STRIDE, bool E16>
__device__ __forceinline__ void lds_issue_4(uint32_t addr, uint32_t (&e)[4]) {
    if (E16)
        asm volatile("ds_read_u16 %0, %4 offset:%5\n\tds_read_u16 %1, %4 offset:%6\n\tds_read_u16 %2, %4 offset:%7\n\tds_read_u16 %3, %4 offset:%8"
                     : "=&v"(e[0]), "=&v"(e[1]), "=&v"(e[2]), "=&v"(e[3])
                     : "v"(addr), "n"(OFF), "n"(OFF + STRIDE), "n"(OFF + 2 * STRIDE), "n"(OFF + 3 * STRIDE) : "memory");
    else
        asm volatile("ds_read_u8 %0, %4 offset:%5\n\tds_read_u8 %1, %4 offset:%6\n\tds_read_u8 %2, %4 offset:%7\n\tds_read_u8 %3, %4 offset:%8"
                     : "=&v"(e[0]), "=&v"(e[1]), "=&v"(e[2]), "=&v"(e[3])
                     : "v"(addr), "n"(OFF), "n"(OFF + STRIDE), "n"(OFF + 2 * STRIDE), "n"(OFF + 3 * STRIDE) : "memory");
}
// value mantissas of stage U: dwords at m_addr + 256 * (4U + i), i = 0..3
template <int U>
__device__ __forceinline__ void lds_issue_val_mant(uint32_t m_addr, uint64_t& w01, uint64_t& w23) {
    asm volatile("ds_read2st64_b32 %0, %2 offset0:%3 offset1:%4\n\tds_read2st64_b32 %1, %2 offset0:%5 offset1:%6"
                 : "=&v"(w01), "=&v"(w23) : "v"(m_addr), "n"(4 * U), "n"(4 * U + 1), "n"(4 * U + 2), "n"(4 * U + 3) : "memory");
}
__device__ __forceinline__ void lds_wait(u32x4& a) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a) : : "memory"); }
__device__ __forceinline__ void lds_wait(u32x4& a, uint32_t (&e)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]) : : "memory");
}
template <int HG>
__device__ __forceinline__ void lds_wait(uint64_t& w01, uint64_t& w23, uint64_t (&pp)[HG]) {
    if constexpr (HG == 1) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w01), "+v"(w23), "+v"(pp[0]) : : "memory");
    else if constexpr (HG == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w01), "+v"(w23), "+v"(pp[0]), "+v"(pp[1]) : : "memory");
    else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w01), "+v"(w23), "+v"(pp[0]), "+v"(pp[1]), "+v"(pp[2]), "+v"(pp[3]) : : "memory");
}
__device__ __forceinline__ void lds_wait(u32x4 (&e)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]) : : "memory");
}
__device__ __forceinline__ void lds_wait(uint32_t (&e)[16]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]), "+v"(e[4]), "+v"(e[5]), "+v"(e[6]), "+v"(e[7]),
                 "+v"(e[8]), "+v"(e[9]), "+v"(e[10]), "+v"(e[11]), "+v"(e[12]), "+v"(e[13]), "+v"(e[14]), "+v"(e[15]) : : "memory");
}

// max over the 16 lanes of a DPP row, the shuffle folded into the max instruction (two wait states between
// a vector write and a DPP read of the same register)
__device__ __forceinline__ float row_max_dpp(float v) {
    float r;
    asm volatile("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"
                 : "=&v"(r) : "v"(v));
    return r;
}

// Cache policy of the DMA loads: the "nt" bit.  The cache is read once per call, and a read-only stream
// of this size moves about 10 % faster with it on this machine (measured with and without, same requests).
constexpr int kStreamAux = 2;

constexpr int vmcnt_imm(int n) { return (n & 0xF) | (0x7 << 4) | (0xF << 8) | ((n >> 4) << 14); }

// PAGED: the planes are a pool of pages and every 64-token tile looks up its page (a scalar load, issued a
// tile ahead of the requests that need it); a separate instantiation, so the contiguous case is untouched.
template <int N, int HG, bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(HG == 4 ? 2 : ((N != 32 && HG == 2) ? 2 : 3), 4)))
void decode_split_lds_p4(DecodeArgs a, int dt) {
    static_assert(N == 16 || N == 32 || N == 64 || N == 128, "block sizes of the format");
    static_assert(HG < 4 || N <= 32, "the sixteen-head variant is built for blocks of 16 and 32");
    constexpr int NB = kD / N;
    constexpr int NH = HG * 4;
    constexpr int kTileTok = 64;
    // per-wavefront staging area
    constexpr int kKm = 0;                         // 4 stages x 1024 B key mantissas
    constexpr int kVm = kKm + 4096;                // 4 stages x 1024 B value mantissas
    // Exponents of a whole 64-token tile: [64 tokens][kExpRow bytes] in LDS.  Blocks of 16 / 32: the 8 / 4 bytes of a
    // token as they lie in the plane, fetched as dwords (two DMA instructions / one).  Blocks of 64 / 128: a token has
    // 2 / 1 bytes, the plane's rows are not dword-aligned, so each lane fetches its token's bytes with a 2- / 1-byte
    // DMA element, which lands zero-extended in the lane's own dword.
    constexpr int kExpRow = NB >= 4 ? NB : 4;
    constexpr int kExpElt = NB >= 4 ? 4 : NB;      // bytes per lane and DMA instruction
    constexpr int kEt = kTileTok * kExpRow;
    constexpr int kKe = kVm + 4096;
    constexpr int kVe = kKe + kEt;
    constexpr int kWaveBytes = kVe + kEt;
    constexpr int kExpDma = kEt / 256;             // DMA instructions per exponent tile (2 for blocks of 16, else 1)
    // Keys go to the scaled FP8 x FP4 MFMA as raw nibbles: a block of 32 is exactly its MX block; a
    // block of 16 takes two products per 32 channels, each with the other block's nibbles zeroed.
    constexpr int kRings = kWaves * kWaveBytes;
    static_assert(kWaves * NH * kD * 4 + kWaves * NH * 8 <= kRings, "merge buffers alias the staging area");
    // The DMA rings are an LDS object of their own: the compiler waits for every outstanding DMA
    // before it touches an object that a DMA may write, and the set-up must not wait for the first tile.
    // (padded so that at most three workgroups fit a compute unit: with four, placement over the units gets uneven)
    constexpr int kSmem = kRings + HG * 4096 + NH * 16 >= 42 * 1024 ? kRings : 42 * 1024 - HG * 4096 - NH * 16;
    __shared__ __align__(16) uint8_t smem[kSmem];
    // probabilities of the current tile, bf16 hi/lo limbs: [wave][HG][2 limbs][4 heads][64 tokens].  A separate
    // LDS object, so the compiler can tell its reads apart from the DMA targets inside smem.
    __shared__ __align__(16) uint16_t p_lds[kWaves][HG * 2 * 4 * kTileTok];
    // Until the main loop starts the same bytes stage the query: q' as fp32 [NH][128] in the first half,
    // its FP8 limbs [NH*4 rows][128] in the second (the permutation and the block maxima of the BFP cast
    // pass through there before the limbs are written); the limbs' scale bytes [NH*4][4] sit beside.
    static_assert(sizeof(p_lds) == NH * kD * 4 + NH * 4 * kD, "query staging fills the probability buffer exactly");
    __shared__ __align__(16) uint8_t qsc_lds[NH * 16];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS bases stay in scalar registers
    const int lane = tid & 63;
    const int j = lane & 15, kg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int h0 = kvh * a.G + a.g_base;      // first (virtual) head of this launch

    int64_t L = a.seq_len ? (int64_t)a.seq_len[b] : a.max_len;
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    // Tiles are dealt out round-robin: split s takes the 256-token tiles s, s + n_splits, s + 2 n_splits, ...
    // The workgroups of one (batch, kv-head) then sweep the sequence side by side instead of each
    // streaming a distant region of its own, which the memory system serves a few percent faster, and no
    // split is more than one tile longer than another.  "Split-relative" tokens below count from t_begin.
    const int64_t t_begin = (int64_t)split * 256;
    const int64_t t_end = L;

    if (t_begin >= t_end) {   // nothing cached in this split
        for (int i = tid; i < a.g_cnt * kD; i += 256)
            a.part_o[(((int64_t)b * a.H_q + h0 + i / kD) * a.n_splits + split) * kD + (i % kD)] = 0.f;
        if (tid < a.g_cnt) {
            float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + tid) * a.n_splits + split) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        return;
    }

    // ---- kvbfp_append_decode_attention: the current token, position L - 1, is cast and stored by the
    // one wavefront whose 64-token tiles include that position (nobody else ever reads the row), off
    // everybody else's path.  Lanes 0-7 take the key row, lanes 8-15 the value row; the rest of the
    // wavefront runs along with zeros (the block maximum is a cross-lane reduction) and stores nothing.
    //   * The row and its permutation are requested here, ahead of the first tile, as raw bits (once
    //     the cache streams, a round trip to memory takes several microseconds).
    //   * After the set-up below (so that its barriers are not held up) the row is reordered through
    //     this wavefront's part of the probability buffer, cast and stored.
    //   * Before the wavefront requests its last tile, the one that holds the row, it waits for the
    //     stores (new_row_stored below).
    // If that tile is the wavefront's first, all of this happens right here instead, before the first
    // request.
    const bool appends = a.k_new != nullptr && (int)(((L - 1) >> 8) % a.n_splits) == split &&
                         (int)(((L - 1) & 255) >> 6) == wave;                       // wave-uniform
    const bool appends_first = appends && (L - 1) < t_begin + 256;
    const int nr_sub = lane & 7, nr_which = (lane >> 3) & 1;
    const bool nr_live = lane < 16;
    uint32_t nr_bits[16];
    int nr_perm[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        nr_bits[i] = 0u;
        nr_perm[i] = nr_sub * 16 + i;
    }
    auto widen = [&](uint32_t h) {
        return dt == KVBFP_F16 ? (float)__builtin_bit_cast(_Float16, (unsigned short)h) : __uint_as_float(h << 16);
    };
    auto store_new_row = [&](const float (&x)[16]) {
        kvbfp::cast::encode_store<4, N>(x, nr_sub, nr_live, const_cast<uint8_t*>(nr_which ? a.v_mant : a.k_mant),
                                        const_cast<uint8_t*>(nr_which ? a.v_exp : a.k_exp),
                                        kvbfp::cache_row(a, b, kvh, L - 1));
    };
    if (appends) {
        const uint16_t* src = (const uint16_t*)(nr_which ? a.v_new : a.k_new) + (int64_t)b * a.new_stride_b +
                              (int64_t)kvh * a.new_stride_h;
        const int32_t* pr = nr_which ? a.perm_v : a.perm_k;
        if (appends_first) {      // short sequence: nothing streams yet, gather straight from memory
            float x[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int c = pr ? (pr[kvh * kD + nr_sub * 16 + i] & (kD - 1)) : (nr_sub * 16 + i);
                x[i] = nr_live ? widen(src[c]) : 0.f;
            }
            store_new_row(x);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __builtin_amdgcn_sched_barrier(0);
        } else if (nr_live) {
#pragma unroll
            for (int i = 0; i < 16; ++i) nr_bits[i] = src[nr_sub * 16 + i];
            if (pr) {
#pragma unroll
                for (int i = 0; i < 16; ++i) nr_perm[i] = pr[kvh * kD + nr_sub * 16 + i] & (kD - 1);
            }
        }
    }

    const int64_t base = PAGED ? 0 : ((int64_t)b * a.H_kv + kvh) * a.max_seq + t_begin;
    // row (relative to the bases below) of the 64-token tile that starts at token T of the split
    auto tile_row = [&](const int T) -> int64_t { return PAGED ? kvbfp::cache_row(a, b, kvh, t_begin + T) : (int64_t)T; };
    const uint8_t* __restrict__ k_mant = a.k_mant + base * 64;
    const uint8_t* __restrict__ v_mant = a.v_mant + base * 64;
    const uint8_t* __restrict__ k_exp = a.k_exp + base * NB;
    const uint8_t* __restrict__ v_exp = a.v_exp + base * NB;
    const int n_tok = (int)(t_end - t_begin);
    // several query tokens: head slot s sees tokens below lim[.] only (split-relative)
    int lim[HG];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) lim[hg] = (int)(L - t_begin) - kvbfp::hidden_tokens(a, a.g_base + hg * 4 + (lane >> 4));

    uint8_t* const wbase = smem + wave * kWaveBytes;

    // ---- DMA source offsets of this lane inside a 16-token stage (full stage) -------------------
    // keys: own chunk; values: slot (position p = lane/4, chunk c = lane%4) <- row 4*(p%4) + p/4
    const int vp_pos = lane >> 2, vp_c = lane & 3;
    const int vrow_of_slot = 4 * (vp_pos & 3) + (vp_pos >> 2);
    const int kd_row = lane >> 2, kd_chunk = (lane & 3) ^ ((lane >> 4) & 3);            // DMA lane -> (row, chunk)
    const uint32_t k_src = (uint32_t)kd_row * 64u + (uint32_t)kd_chunk * 16u;
    const uint32_t v_src = (uint32_t)vrow_of_slot * 64u + (uint32_t)vp_c * 16u;
    const uint32_t e_src = (uint32_t)lane * kExpElt;   // exponents: element `lane` (+64 per further instruction) of the tile's rows

    // Re-fills of the staging area.  Mantissas: stage u of a tile that starts at token t of the split = plane
    // row `row` (tile_row of the tile).  A full tile takes the immediate-offset form (the offset applies to the
    // global and to the LDS address alike, 1024 bytes per stage in both); in a ragged one rows past the last
    // cached token re-read that token.  `left` values are wave-uniform, so these are scalar branches.
    auto fill_mant = [&](auto U, const bool keys, const bool tile_full, const int t, const int64_t row) {
        constexpr int u = decltype(U)::value;
        const uint8_t* __restrict__ mp = (keys ? k_mant : v_mant) + row * 64;
        uint8_t* const lm = wbase + (keys ? kKm : kVm);
        if (tile_full) {
            __builtin_amdgcn_global_load_lds(KVBFP_GPTR(mp + (keys ? k_src : v_src)), KVBFP_LPTR(lm), 16, u * 1024, kStreamAux);
        } else {
            const int left = n_tok - (t + 16 * u);       // may be <= 0: then every lane re-reads the last cached token
            const int r = keys ? kd_row : vrow_of_slot, c = keys ? kd_chunk : vp_c;
            const int mo = (16 * u + min(r, left - 1)) * 64 + c * 16;
            __builtin_amdgcn_global_load_lds(KVBFP_GPTR(mp + mo), KVBFP_LPTR(lm + u * 1024), 16, 0, kStreamAux);
        }
    };
    // Exponents of a whole tile, [64 tokens][NB] as they lie in the plane.
    auto fill_exp = [&](const bool keys, const bool tile_full, const int t, const int64_t row) {
        const uint8_t* __restrict__ ep = (keys ? k_exp : v_exp) + row * NB;
        uint8_t* const le = wbase + (keys ? kKe : kVe);
        if (tile_full) {
            if constexpr (NB >= 4) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + e_src), KVBFP_LPTR(le), 4, 0, kStreamAux);
            else if constexpr (NB == 2) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + e_src), KVBFP_LPTR(le), 2, 0, kStreamAux);
            else __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + e_src), KVBFP_LPTR(le), 1, 0, kStreamAux);
            if (kExpDma == 2) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + e_src), KVBFP_LPTR(le), 4, 256, kStreamAux);
        } else {
            const int left = n_tok - t;                    // >= 1
#pragma unroll
            for (int x = 0; x < kExpDma; ++x) {
                const int byte = (int)e_src + 256 * x;      // offset in the tile's exponent rows
                const int eo = min(byte / NB, left - 1) * NB + byte % NB;
                if constexpr (NB >= 4) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + eo), KVBFP_LPTR(le + 256 * x), 4, 0, kStreamAux);
                else if constexpr (NB == 2) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + eo), KVBFP_LPTR(le + 256 * x), 2, 0, kStreamAux);
                else __builtin_amdgcn_global_load_lds(KVBFP_GPTR(ep + eo), KVBFP_LPTR(le + 256 * x), 1, 0, kStreamAux);
            }
        }
    };

    // ---- the query and its permutation are requested first, the first tile of this wavefront right
    // after them, and only then does anybody wait: issued later, these small loads would queue
    // behind the first tiles of every workgroup of the grid (tens of megabytes).
    // (Loaded as raw bits and widened later: a conversion right here would make the compiler wait for
    // each load in turn.  For the same reason the set-up below synchronises with LDS-only barriers:
    // __syncthreads() also waits for every vector-memory operation, i.e. for the whole first tile.)
    constexpr int kQPerThread = NH * kD / 256;
    uint32_t q_bits[kQPerThread];
#pragma unroll
    for (int k = 0; k < kQPerThread; ++k) {
        const int i = tid + 256 * k, g = i / kD, c = i % kD;
        const int64_t idx = kvbfp::query_row(a, b, kvh, a.g_base + min(g, a.g_cnt - 1)) * kD + c;   // clamped: rows beyond the count are zeroed below
        q_bits[k] = dt == KVBFP_F32 ? ((const uint32_t*)a.q)[idx] : (uint32_t)((const uint16_t*)a.q)[idx];
    }
    // This thread builds the operand bytes at position `qpos` of the heads tid / 128 + 2k.  FP8 operand layout
    // (measured): byte i of lane-group g is channel 64*(i/16) + 16*g + i%16, and the E8M0 scale of channel block kb
    // (32 consecutive channels) is taken from lane-group kb.
    const int qpos = tid & (kD - 1);
    const int qchan = (qpos & 16) ? 64 + 16 * (qpos >> 5) + (qpos & 15) : 16 * (qpos >> 5) + (qpos & 15);
    int perm_c = qchan;                 // source channel of cache channel qchan
    if (a.perm_k) perm_c = a.perm_k[kvh * kD + qchan];
    auto lds_barrier = [] { lds_only_barrier(); };
    // The permuted (and, on request, BFP-cast) queries wait in the probability buffer, which is free
    // until the main loop; the operand builders below read them from there.  The raw values go to LDS
    // before the first tile is requested (the sequence length, needed for that request, was loaded
    // after them, so they have arrived by now); everything after works on LDS only.
    float* const qr = (float*)&p_lds[0][0];                 // [NH][kD], unscaled
    int* const scratch = (int*)(qr + NH * kD);              // permutation, then block maxima of the cast
#pragma unroll
    for (int k = 0; k < kQPerThread; ++k) {
        const int g = (tid + 256 * k) / kD;
        float f;
        if (dt == KVBFP_F32) f = __uint_as_float(q_bits[k]);
        else if (dt == KVBFP_F16) f = (float)__builtin_bit_cast(_Float16, (unsigned short)q_bits[k]);
        else f = __uint_as_float(q_bits[k] << 16);
        qr[tid + 256 * k] = g < a.g_cnt ? f : 0.f;
    }
    perm_c &= kD - 1;                   // a valid permutation is unchanged; keeps LDS reads in range

    const int T_first = wave * kTileTok;
    const bool has_work = T_first < n_tok;
    if (has_work) {
        const int64_t row0 = tile_row(T_first);
        const bool full0 = n_tok - T_first >= kTileTok;
        static_for<4>([&](auto U) {
            fill_mant(U, true, full0, T_first, row0);
            if (decltype(U)::value == 0) fill_exp(true, full0, T_first, row0);
        });
        static_for<4>([&](auto U) {
            fill_mant(U, false, full0, T_first, row0);
            if (decltype(U)::value == 0) fill_exp(false, full0, T_first, row0);
        });
    }

    // ---- query operand of the score product (whole workgroup) ---------------------------------------
    v8i aq8[HG];           // row 4*head + limb (4 FP8 limbs), one MFMA of 128 channels
    int sa8[HG];           // E8M0 scale of this lane's 32 query values
    {
        // Each block of 32 query values shares a power-of-two scale 2^sh chosen so that the largest lands in
        // [128, 256); limb l holds the FP8 rounding of the residual at scale 2^(sh - 4l), so four limbs carry 16
        // bits relative to the block's maximum.  A wavefront holds 64 consecutive operand positions of one head:
        // the 16-lane rows r and r + 2 are the two halves of one block of 32 channels, so the block maximum is a
        // DPP row reduction and one exchange across 32 lanes.
        float qv[kQPerThread];             // q'[head][qchan] * softmax_scale * log2(e)
        lds_barrier();                     // the raw queries are in LDS
        if (a.q_mant_bits) {               // query cast to BFP: reorder in LDS, cast there (blocks may span wavefronts)
            float q_perm[kQPerThread];
#pragma unroll
            for (int k = 0; k < kQPerThread; ++k) q_perm[k] = qr[((tid + 256 * k) / kD) * kD + perm_c];
            lds_barrier();
#pragma unroll
            for (int k = 0; k < kQPerThread; ++k) qr[((tid + 256 * k) / kD) * kD + qchan] = q_perm[k];
            lds_barrier();
            bfp_round_queries(qr, (uint32_t*)scratch, NH, a.log2_block, a.q_mant_bits);
#pragma unroll
            for (int k = 0; k < kQPerThread; ++k) qv[k] = qr[((tid + 256 * k) / kD) * kD + qchan] * a.scale_log2e;
            lds_barrier();                 // the limbs below overwrite the scratch area
        } else {
#pragma unroll
            for (int k = 0; k < kQPerThread; ++k) qv[k] = qr[((tid + 256 * k) / kD) * kD + perm_c] * a.scale_log2e;
        }
        uint8_t* q8 = (uint8_t*)(qr + NH * kD);           // [NH * 4 limb rows][kD positions], beside the fp32 values
        uint8_t* qsc = qsc_lds;
        const int kb = qchan >> 5;
#pragma unroll
        for (int k = 0; k < kQPerThread; ++k) {
            const int g = (tid + 256 * k) / kD;
            float mx = row_max(fabsf(qv[k]));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            int e = 0;
            if (mx > 0.f) (void)frexpf(mx, &e);            // mx = f * 2^e, f in [0.5, 1)
            int sh = mx > 0.f ? e - 8 : 0;                  // mx * 2^-sh in [128, 256)
            sh = max(-114, min(118, sh));                   // every limb's scale byte sh - 4 limb + 127 - 1 stays in 0..254
            float v = qv[k];
#pragma unroll
            for (int limb = 0; limb < 4; ++limb) {
                const int sl = sh - 4 * limb;
                const uint32_t packed = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(v, -sl), 0.f, 0, false);
                v -= ldexpf(__builtin_amdgcn_cvt_f32_fp8((int)packed, 0), sl);
                q8[(4 * g + limb) * kD + qpos] = (uint8_t)(packed & 0xFFu);
                if ((qchan & 31) == 0) qsc[(4 * g + limb) * 4 + kb] = (uint8_t)(sl + 127);
            }
        }
        lds_barrier();
#pragma unroll
        for (int hg = 0; hg < HG; ++hg) {
            const u32x4 lo = *(const u32x4*)(q8 + (hg * 16 + j) * kD + kg * 32);
            const u32x4 hi = *(const u32x4*)(q8 + (hg * 16 + j) * kD + kg * 32 + 16);
            aq8[hg] = v8i{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            sa8[hg] = qsc[(hg * 16 + j) * 4 + kg] - 1;      // - 1: the key operand below is magnitude / 2 at the block's own exponent byte
        }
        lds_barrier();                                    // the buffer goes over to the probabilities
    }
    if (appends && !appends_first) {
        float* const row = (float*)&p_lds[wave][0] + nr_which * kD;     // [2][kD] floats: this wavefront's 1 KB
        if (nr_live) {
#pragma unroll
            for (int i = 0; i < 16; ++i) row[nr_sub * 16 + i] = widen(nr_bits[i]);
        }
        // the row is read back below by other lanes of this wavefront
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = nr_live ? row[nr_perm[i]] : 0.f;
        store_new_row(x);
    }

    const int a_head = j >> 2, a_par = (j >> 1) & 1, a_limb = j & 1;
    const uint32_t sel_even = a_par ? 0x01000c0cu : 0x0c0c0100u;
    const uint32_t sel_odd = a_par ? 0x03020c0cu : 0x0c0c0302u;

    float m_run[HG], l_run[HG];
    f32x4 o_acc[HG][4];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        m_run[hg] = -INFINITY;
        l_run[hg] = 0.f;
#pragma unroll
        for (int m = 0; m < 4; ++m) o_acc[hg][m] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- LDS read offsets of this lane inside a stage --------------------------------------------
    const uint32_t kq = lds_addr(wbase + kKm + (4 * j + (kg ^ ((j >> 2) & 3))) * 16);       // row j, chunk kg
    // own exponent byte(s): the block of channels 32 kg .. 32 kg + 31 (two blocks of 16: a 16-bit read)
    const uint32_t keq = lds_addr(wbase + kKe + j * kExpRow + (N == 16 ? 2 * kg : (32 * kg) / N));   // + 16 kExpRow per stage
    const uint32_t vq = lds_addr(wbase + kVm + kg * 64 + j * 4);                           // + i*256: row 4kg+i sits at position 4i+kg
    // value exponents: blocks of 32 -> the 16 bytes of tokens 4kg..4kg+3 in one read per stage, this lane's block is
    // byte j/4 of each dword; blocks of 16 -> byte (4kg + i) NB + j/2, one read each
    const uint32_t veq = lds_addr(wbase + kVe + (4 * kg) * kExpRow + (N == 32 ? 0 : (8 * j) / N));
    const uint32_t ve_rot = (uint32_t)((8 * (j >> 2) + 32 - 23) & 31);   // rotation that brings byte j/4 to the exponent field
    uint16_t* const ps = &p_lds[wave][0];
    const uint32_t ps_rd = lds_addr(&p_lds[wave][(a_limb * 4 + a_head) * kTileTok + 4 * kg]);   // + head group and column tile

    if (has_work) {
        // Software pipeline over the eight stages of a tile (K0..K3, V0..V3): the LDS reads of a stage are issued
        // one stage ahead of its arithmetic, so their latency is covered by the arithmetic of the stage before,
        // and a stage is re-filled for the wavefront's next tile as soon as its reads have returned.  The
        // exponent bytes of a whole tile are read with its first stage (and re-filled right after).
        const int kStep = a.n_splits * kWaves * kTileTok;      // this workgroup's next 256-token tile
        // (Where registers are short -- four head groups, or two with blocks of 32, which keep three wavefronts per
        // SIMD -- every stage issues its own reads and waits for them; the probabilities look ahead with one group only.)
        constexpr bool kPipe = HG == 1 || (HG == 2 && N != 32), kPipeP = HG == 1;
        u32x4 rawk[kPipe ? 2 : 1];
        uint32_t kexp[4];
        uint64_t vw01[kPipe ? 2 : 1], vw23[kPipe ? 2 : 1], ppv[kPipeP ? 2 : 1][HG];
        u32x4 vexp32[4];          // blocks of 32: per stage the exponent dwords of tokens 4kg..4kg+3
        uint32_t vexp16[16];      // blocks of 16: per (stage, token) this lane's exponent byte
        // DMA completes in issue order; per tile that is K0, key exponents, K1..K3, V0, value exponents, V1..V3.
        // "The oldest stage still outstanding has landed" = at most (instructions issued after it) outstanding:
        // 7 + kExpDma after the first stage of a plane (it ends with the exponents), 7 + 2 kExpDma after any other,
        // while the next tile is being requested; on the last tile only what is left of the tile itself.
        auto wait_dma = [&](const bool refilling, auto steady_tag, auto tail_tag) {
            __builtin_amdgcn_sched_barrier(0);
            if (refilling) __builtin_amdgcn_s_waitcnt(vmcnt_imm(decltype(steady_tag)::value));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(decltype(tail_tag)::value));
            __builtin_amdgcn_sched_barrier(0);
        };
        constexpr int kAfterFirst = 7 + kExpDma, kAfterOther = 7 + 2 * kExpDma;
        auto issue_k0 = [&] {
            lds_issue_b128<0>(kq, rawk[0]);
            lds_issue_4<0, 16 * kExpRow, N == 16>(keq, kexp);
        };
        // wait for the DMA of a stage and issue its LDS reads (`more`: the next tile is being requested meanwhile)
        auto start_k = [&](auto U, const bool more) {             // key stage U >= 1
            constexpr int u = decltype(U)::value;
            wait_dma(more, std::integral_constant<int, kAfterOther>{}, std::integral_constant<int, 7 + kExpDma - u>{});
            lds_issue_b128<u * 1024>(kq, rawk[kPipe ? (u & 1) : 0]);
        };
        auto start_v0 = [&](const bool more) {                    // value stage 0 and the tile's value exponents
            wait_dma(more, std::integral_constant<int, kAfterFirst>{}, std::integral_constant<int, 3>{});
            lds_issue_val_mant<0>(vq, vw01[0], vw23[0]);
            if (N == 32) {
                lds_issue_b128<0>(veq, vexp32[0]); lds_issue_b128<64>(veq, vexp32[1]);
                lds_issue_b128<128>(veq, vexp32[2]); lds_issue_b128<192>(veq, vexp32[3]);
            } else {
                static_for<4>([&](auto V) {
                    constexpr int v = decltype(V)::value;
                    lds_issue_4<v * 16 * kExpRow, kExpRow, false>(veq, *(uint32_t(*)[4])&vexp16[4 * v]);
                });
            }
        };
        auto issue_p = [&](auto U, auto BUF) {                    // probabilities of value stage U
            static_for<HG>([&](auto HGI) {
                constexpr int hg = decltype(HGI)::value;
                lds_issue_b64<(hg * 2 * 4 * kTileTok + 16 * decltype(U)::value) * 2>(ps_rd, ppv[decltype(BUF)::value][hg]);
            });
        };
        auto start_v = [&](auto U, const bool more) {             // value stage U >= 1
            constexpr int u = decltype(U)::value;
            wait_dma(more, std::integral_constant<int, kAfterOther>{}, std::integral_constant<int, 3 - u>{});
            lds_issue_val_mant<u>(vq, vw01[kPipe ? (u & 1) : 0], vw23[kPipe ? (u & 1) : 0]);
            if constexpr (kPipeP) issue_p(U, std::integral_constant<int, u & 1>{});
        };
        // One tile.  STEADY: this tile is complete and seen whole by every head, and a complete next tile is being
        // requested -- the common case, compiled without the ragged-tile branches, clamps and masks.
        auto tile_body = [&](auto steady_tag, const int T0, const int T1, const bool more_rt, const bool full1_rt,
                             const bool masked_rt, const int64_t row1) {
            constexpr bool STEADY = decltype(steady_tag)::value;
            const bool more = STEADY ? true : more_rt;
            const bool full1 = STEADY ? true : full1_rt;
            const bool masked = STEADY ? false : masked_rt;
            const int left = n_tok - T0;
            // the first stage of a tile is read here and not ahead, at the end of the tile before: a register with a
            // read pending must not be live across the loop's back edge (the compiler may copy it there)
            wait_dma(true, std::integral_constant<int, kAfterFirst>{}, std::integral_constant<int, 0>{});
            issue_k0();

            // ---------------- scores
            f32x4 s_acc[HG][4];
            static_for<4>([&](auto U) {
                constexpr int u = decltype(U)::value;
                constexpr int cur = kPipe ? (u & 1) : 0;
                if constexpr (!kPipe && u > 0) start_k(U, more);
                if (u == 0) lds_wait(rawk[0], kexp); else lds_wait(rawk[cur]);
                __builtin_amdgcn_sched_barrier(0);
                if (more) {
                    fill_mant(U, true, full1, T1, row1);
                    if (u == 0) fill_exp(true, full1, T1, row1);
                }
                if constexpr (kPipe) {
                    if constexpr (u < 3) start_k(std::integral_constant<int, u + 1>{}, more); else start_v0(more);
                }
                __builtin_amdgcn_sched_barrier(0);
                const u32x4 raw = rawk[cur];
#pragma unroll
                for (int hg = 0; hg < HG; ++hg) s_acc[hg][u] = f32x4{0.f, 0.f, 0.f, 0.f};
                // magnitude/2 = FP4(s,0,m1,m0) + FP4(s,m2,0,0): two masked copies of the raw nibbles are the B
                // operands and the block's exponent byte is their E8M0 scale (the halving sits in the query's scale).
                if (N >= 32) {                 // one exponent byte per 32 channels (the same byte for wider blocks)
                    const int sb = (int)kexp[u];
                    const v8i b1 = {(int)(raw[0] & 0xBBBBBBBBu), (int)(raw[1] & 0xBBBBBBBBu), (int)(raw[2] & 0xBBBBBBBBu),
                                    (int)(raw[3] & 0xBBBBBBBBu), 0, 0, 0, 0};
                    const v8i b2 = {(int)(raw[0] & 0xCCCCCCCCu), (int)(raw[1] & 0xCCCCCCCCu), (int)(raw[2] & 0xCCCCCCCCu),
                                    (int)(raw[3] & 0xCCCCCCCCu), 0, 0, 0, 0};
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg) {
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], b1, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb);
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], b2, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb);
                    }
                } else {
                    // the lane's 32 nibbles are two blocks of 16 (dwords 0-1 and 2-3) with an exponent each
                    const int sb0 = (int)(kexp[u] & 0xFFu), sb1 = (int)(kexp[u] >> 8);
                    const v8i lo1 = {(int)(raw[0] & 0xBBBBBBBBu), (int)(raw[1] & 0xBBBBBBBBu), 0, 0, 0, 0, 0, 0};
                    const v8i lo2 = {(int)(raw[0] & 0xCCCCCCCCu), (int)(raw[1] & 0xCCCCCCCCu), 0, 0, 0, 0, 0, 0};
                    const v8i hi1 = {0, 0, (int)(raw[2] & 0xBBBBBBBBu), (int)(raw[3] & 0xBBBBBBBBu), 0, 0, 0, 0};
                    const v8i hi2 = {0, 0, (int)(raw[2] & 0xCCCCCCCCu), (int)(raw[3] & 0xCCCCCCCCu), 0, 0, 0, 0};
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg) {
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], lo1, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb0);
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], lo2, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb0);
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], hi1, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb1);
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], hi2, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb1);
                    }
                }
            });

            // ---------------- online softmax; lane (j, kg) owns head kg of each group, tokens 16u + j
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) {
                float s[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) s[u] = (s_acc[hg][u][0] + s_acc[hg][u][1]) + (s_acc[hg][u][2] + s_acc[hg][u][3]);   // the limb rows
                if (masked) {
                    const int vis = min(left, lim[hg] - T0);
#pragma unroll
                    for (int u = 0; u < 4; ++u) s[u] = (16 * u + j < vis) ? s[u] : -INFINITY;
                }
                const float tmax = row_max_dpp(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])));   // -inf only if this head sees none of the tile
                const float m_new = fmaxf(m_run[hg], tmax);
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = exp2_raw(m_run[hg] - m_ref);
                const float m_p = m_ref - (float)kShift;     // probabilities carry 2^kShift (values come as 2^-kShift)
                float psum = 0.f;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // two bf16 limbs: the upper half of the fp32 pattern as it is, and the rest rounded
                    const float pw = exp2_raw(s[u] - m_p);
                    const uint32_t hi_bits = __float_as_uint(pw) & 0xFFFF0000u;
                    const __bf16 pl = (__bf16)(pw - __uint_as_float(hi_bits));
                    psum += pw;
                    ps[((hg * 2 + 0) * 4 + kg) * kTileTok + 16 * u + j] = (uint16_t)(hi_bits >> 16);
                    ps[((hg * 2 + 1) * 4 + kg) * kTileTok + 16 * u + j] = __builtin_bit_cast(unsigned short, pl);
                }
                l_run[hg] = l_run[hg] * alpha + psum;
                m_run[hg] = m_new;
                if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                    for (int m = 0; m < 4; ++m) o_acc[hg][m] *= alpha;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kPipeP) issue_p(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});

            // ---------------- values
            static_for<4>([&](auto U) {
                constexpr int u = decltype(U)::value;
                constexpr int cur = kPipe ? (u & 1) : 0;
                constexpr int pc = kPipeP ? (u & 1) : 0;
                if constexpr (!kPipe) { if constexpr (u == 0) start_v0(more); else start_v(U, more); }
                if constexpr (!kPipeP) issue_p(U, std::integral_constant<int, 0>{});
                lds_wait<HG>(vw01[cur], vw23[cur], ppv[pc]);
                if (u == 0) { if (N == 32) lds_wait(vexp32); else lds_wait(vexp16); }
                __builtin_amdgcn_sched_barrier(0);
                if (more) {
                    fill_mant(U, false, full1, T1, row1);
                    if (u == 0) fill_exp(false, full1, T1, row1);
                }
                if constexpr (kPipe && u < 3) start_v(std::integral_constant<int, u + 1>{}, more);
                __builtin_amdgcn_sched_barrier(0);
                const uint32_t vw[4] = {(uint32_t)vw01[cur], (uint32_t)(vw01[cur] >> 32), (uint32_t)vw23[cur], (uint32_t)(vw23[cur] >> 32)};
                Unpacked vv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // scale operand: the exponent byte in the exponent field (the conversion looks at nothing else:
                    // for blocks of 32 the other bytes of the dword stay where the rotation leaves them)
                    const float sc = N == 32 ? __uint_as_float(__builtin_amdgcn_alignbit(vexp32[u][i], vexp32[u][i], ve_rot))
                                             : scale_operand(vexp16[4 * u + i]);
                    vv[i] = unpack8(vw[i], sc);
                }
#pragma unroll
                for (int hg = 0; hg < HG; ++hg) {
                    const uint32_t px = (uint32_t)ppv[pc][hg], py = (uint32_t)(ppv[pc][hg] >> 32);
                    uint32_t ar[4];
                    ar[0] = __builtin_amdgcn_perm(px, px, sel_even);
                    ar[1] = __builtin_amdgcn_perm(px, px, sel_odd);
                    ar[2] = __builtin_amdgcn_perm(py, py, sel_even);
                    ar[3] = __builtin_amdgcn_perm(py, py, sel_odd);
                    const bf16x8 ap = __builtin_bit_cast(bf16x8, u32x4{ar[0], ar[1], ar[2], ar[3]});
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        const bf16x8 bv = join(vv[0].p[m], vv[1].p[m], vv[2].p[m], vv[3].p[m]);
                        o_acc[hg][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, bv, o_acc[hg][m], 0, 0, 0);
                    }
                }
            });
            // (the next tile writes its probabilities after its score phase; every read of this tile's has returned)
        };
        for (int T0 = T_first; T0 < n_tok; T0 += kStep) {
            const int T1 = T0 + kStep;
            const bool more = T1 < n_tok;            // wave-uniform
            const int64_t row1 = more ? tile_row(T1) : 0;
            const bool full1 = n_tok - T1 >= kTileTok;       // the next tile is complete
            if (appends && more && T1 + kStep >= n_tok) {      // next comes the tile with the new row: its stores first
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                __builtin_amdgcn_sched_barrier(0);
            }
            // masking is needed only where the tile is ragged or a head must not see all of it (several query tokens)
            bool masked = n_tok - T0 < kTileTok;
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) masked = masked || __builtin_amdgcn_ballot_w64(lim[hg] - T0 < kTileTok) != 0;
            if (more && full1 && !masked) tile_body(std::true_type{}, T0, T1, true, true, false, row1);
            else tile_body(std::false_type{}, T0, T1, more, full1, masked, row1);
        }
    }

    // ---- merge the four wavefronts (buffers alias the staging areas, all DMA has landed) ---------
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    float* const o_s = (float*)smem;                              // [kWaves][NH][kD]
    float* const ml_s = (float*)(smem + kWaves * NH * kD * 4);    // [kWaves][NH][2]
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        const float lsum = row_sum(l_run[hg]);
        const int head = hg * 4 + kg;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int c_even = 8 * j + slot_channel(2 * m);
            const int c_odd = 8 * j + slot_channel(2 * m + 1);
            o_s[(wave * NH + head) * kD + c_even] = o_acc[hg][m][0] + o_acc[hg][m][1];
            o_s[(wave * NH + head) * kD + c_odd] = o_acc[hg][m][2] + o_acc[hg][m][3];
        }
        if (j == 0) {
            ml_s[(wave * NH + head) * 2 + 0] = m_run[hg];
            ml_s[(wave * NH + head) * 2 + 1] = lsum * (1.0f / (float)(1 << kShift));   // the probabilities carried 2^kShift
        }
    }
    __syncthreads();
    for (int i = tid; i < a.g_cnt * kD; i += 256) {
        const int g = i / kD, c = i % kD;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, ml_s[(w * NH + g) * 2]);
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = ml_s[(w * NH + g) * 2];
            if (mw > -INFINITY) acc = fmaf(exp2f(mw - M), o_s[(w * NH + g) * kD + c], acc);
        }
        a.part_o[(((int64_t)b * a.H_q + h0 + g) * a.n_splits + split) * kD + c] = acc;
    }
    if (tid < a.g_cnt) {
        const int g = tid;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, ml_s[(w * NH + g) * 2]);
        float lsum = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = ml_s[(w * NH + g) * 2];
            if (mw > -INFINITY) lsum = fmaf(exp2f(mw - M), ml_s[(w * NH + g) * 2 + 1], lsum);
        }
        float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + g) * a.n_splits + split) * 2;
        ml[0] = M;
        ml[1] = lsum;
    }
}

// 16-bit I/O: the LDS pipeline, every block size.  fp32 I/O: the register-staged pass with three probability
// limbs and the three-limb bf16 query (the FP8 query limbs of the LDS pipeline carry 16 bits, too few for the
// 1e-5 bar).
template <int HG, bool PAGED>
hipError_t launch_reg(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    if (block == 16) decode_split_mfma_p4<16, HG, 3, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 32) decode_split_mfma_p4<32, HG, 3, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 64) decode_split_mfma_p4<64, HG, 3, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 128) decode_split_mfma_p4<128, HG, 3, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int HG, bool PAGED>
hipError_t launch_n(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    if (dt == KVBFP_F32) return launch_reg<HG, PAGED>(a, dt, block, grid, s);
    if (block == 16) decode_split_lds_p4<16, HG, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 32) decode_split_lds_p4<32, HG, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 64) decode_split_lds_p4<64, HG, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else if (block == 128) decode_split_lds_p4<128, HG, PAGED><<<grid, 256, 0, s>>>(a, dt);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

namespace kvbfp {

hipError_t launch_decode_split_mfma(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s) {
    const dim3 grid((unsigned)a.n_splits, (unsigned)a.H_kv, (unsigned)batch);
    if (a.g_cnt > 8) {      // sixteen heads per workgroup: LDS pipeline only (the host asks for it nowhere else)
        if (dtype == KVBFP_F32 || block > 32) return hipErrorInvalidValue;
        if (a.block_table) {
            if (block == 16) decode_split_lds_p4<16, 4, true><<<grid, 256, 0, s>>>(a, dtype);
            else decode_split_lds_p4<32, 4, true><<<grid, 256, 0, s>>>(a, dtype);
        } else {
            if (block == 16) decode_split_lds_p4<16, 4, false><<<grid, 256, 0, s>>>(a, dtype);
            else decode_split_lds_p4<32, 4, false><<<grid, 256, 0, s>>>(a, dtype);
        }
        return hipGetLastError();
    }
    if (a.block_table) return a.g_cnt <= 4 ? launch_n<1, true>(a, dtype, block, grid, s) : launch_n<2, true>(a, dtype, block, grid, s);
    return a.g_cnt <= 4 ? launch_n<1, false>(a, dtype, block, grid, s) : launch_n<2, false>(a, dtype, block, grid, s);
}

}  // namespace kvbfp
