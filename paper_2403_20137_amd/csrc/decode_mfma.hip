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
#include "decode_lds.h"

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
// PAGED: the planes are a pool of pages and every 16-token stage of a tile looks up its page (a separate instantiation: the
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
    // (Paged cache: the bases are those of the pool and every 16-token stage of a tile looks up its page.)
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
        // first row of the tile, wave-uniform; a pool of pages has one base per 16-token stage (a page may hold 16 tokens)
        kvbfp::StageBases sb{};
        if constexpr (PAGED) sb = kvbfp::stage_bases(a, b, kvh, t_begin + T0, t_end);
        auto tile_base = [&](const int u) -> size_t { return PAGED ? (size_t)(sb.v[u] + t_begin + T0) : (size_t)T0; };
        const int left = n_tok - T0;                 // cached tokens from T0 on (>= 1)

        // ---------------- scores of 64 tokens
        f32x4 s_acc[HG][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint8_t* __restrict__ kp = k_mant + tile_base(u) * 64;
            const uint8_t* __restrict__ kep = k_exp + tile_base(u) * NB;
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
            const uint8_t* __restrict__ vp = v_mant + tile_base(u) * 64;
            const uint8_t* __restrict__ vep = v_exp + tile_base(u) * NB;
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


// The LDS-DMA pipeline (decode_lds.h) for 4-bit mantissas.
template <int N, int HG, bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(HG == 4 ? 2 : ((N != 32 && HG == 2) ? 2 : 3), 4)))
void decode_split_lds_p4(DecodeArgs a, int dt) {
    kvbfp::lds::decode_split_lds_body<4, N, HG, PAGED>(a, dt);
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
