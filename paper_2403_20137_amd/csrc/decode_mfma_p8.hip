// Decode attention over the packed cache with 8-bit mantissas on the gfx950 matrix cores.
//
// Method: the cache holds keys and values as Block Floating Point (Sec. II-B, Eq. (1)): one
// sign-magnitude byte per position plus one shared exponent byte per block.  The product q.K^T reads
// that format directly (Sec. III, Eq. (2)-(3): the channel order is whatever the cache uses, the
// query arrives in the same order), softmax and the product with V follow.
//
// From code byte to matrix-core operand without integer-to-float arithmetic:
//   code = s mmmm lll (sign, 7 magnitude bits).  The magnitude is 8 * hi + lo with hi = mmmm (0..15)
//   and lo = lll (0..7).  The bytes  s000 mmmm  and  s0000 lll  are both valid OCP FP8 (E4M3) numbers:
//   the subnormals and the first binade of E4M3 share one spacing, so s000xxxx reads as exactly
//   +-x * 2^-9 for every x in 0..15.  v_cvt_scalef32_pk_bf16_fp8 turns two such bytes into two bf16
//   values and multiplies by a power of two on the way, which is where the block exponent goes in
//   (the hi piece gets the scale times 8).  Both pieces enter the matrix product as separate terms of
//   the reduction, next to the same query (resp. probability) entry, so they are added in fp32 inside
//   the MFMA.  Cost per 4 codes: 4 bit operations + 4 conversions.
//
// Score product  S = Q . K^T  (v_mfma_f32_16x16x32_bf16, A = query rows, B = keys):
//   lane (j = lane%16, kg = lane/16) loads the 16-byte chunks kg and kg+4 of the key row of token j
//   (channels 16kg.. and 64+16kg..); each of its 8 dwords feeds one MFMA whose reduction slots are
//   (hi piece, lo piece) x 4 channels.  A holds the query in three bf16 limbs, rows 4*head + limb.
// Value product  O = P . V: lane (j, kg) loads the 8 bytes of channels 8j..8j+7 of the value rows of
//   tokens 4kg..4kg+3; a converted register holds two adjacent channels of one token, the reduction
//   index enumerates (token, channel parity) and the probabilities sit in rows (head, parity, limb)
//   with zeros in the other parity's slots.
// Each wavefront owns every fourth 64-token tile of its split and keeps its own online-softmax
// state; the four wavefronts of a workgroup merge once at the end.
//
// This register-staged kernel serves fp32 I/O (three bf16 limbs for the query and the probabilities).
// fp16/bf16 I/O goes through the LDS-DMA pipeline of decode_lds.h, instantiated at the end of this file
// for 8-bit mantissas, where the key pieces enter the scaled FP8 MFMA without any conversion.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>

#include "decode_args.h"
#include "decode_dev.h"
#include "kvbfp_internal.h"
#include "decode_lds.h"

namespace {

using kvbfp::DecodeArgs;
using namespace kvbfp::dev;

// fp32 scale operands for the two pieces of a code with stored exponent byte E.  A code m stands for
// m * 2^(E - 133); the lo piece read as FP8 is lo * 2^-9, and with the byte E itself as the exponent
// field of its scale operand (all the conversion looks at) it becomes lo * 2^(E - 136) = its value
// * 2^-kShift; the hi piece weighs 8 times as much (field E + 3).  Exact in bf16 (denormals included) for
// every E >= 3; E = 1, 2 (magnitudes below 2^-124) lose low-order bits, an absolute error under 2^-126;
// E >= 252 (block maxima above 2^124) would overflow the field and is not supported here.
constexpr int kShift = 3;
__device__ __forceinline__ float scale_lo(uint32_t E) { return __uint_as_float(E << 23); }
__device__ __forceinline__ float scale_hi(uint32_t E) { return __uint_as_float((E + 3u) << 23); }

// 4 sign-magnitude bytes -> hi pieces (c0,c1), (c2,c3) and lo pieces (c0,c1), (c2,c3) as bf16 pairs
struct Pieces { bf16x2 h01, h23, l01, l23; };
__device__ __forceinline__ Pieces unpack4(uint32_t w, float s_hi, float s_lo) {
    const uint32_t sign = w & 0x80808080u;
    const uint32_t hi = ((w >> 3) & 0x0F0F0F0Fu) | sign;
    const uint32_t lo = w & 0x87878787u;
    Pieces r;
    r.h01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, s_hi, false);
    r.h23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, s_hi, true);
    r.l01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, s_lo, false);
    r.l23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, s_lo, true);
    return r;
}

// N = block size, HG = groups of four query heads per KV head (G <= 4*HG).
// grid = (n_splits, H_kv, B), block = 256 (four wavefronts).
// PL = bf16 limbs of a probability: 2 (16 bits, enough for 16-bit outputs) or 3 (24 bits, fp32 outputs).
// PAGED: the planes are a pool of pages and every 16-token stage of a tile looks up its page (a separate instantiation: the
// contiguous case keeps its 32-bit offsets from one scalar base).
template <int N, int HG, int PL, bool PAGED>
__global__ __launch_bounds__(256) void decode_split_mfma_p8(DecodeArgs a, int dt) {
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

    // A operands of the score product: row r = lane%16 = 4*head + limb; MFMA d (0..7) reduces over
    // the four channels 64*(d/4) + 16*kg + 4*(d%4) + (0..3), slots 0-3 against the hi pieces and
    // slots 4-7 against the lo pieces.
    bf16x8 aq[HG][8];
    {
        const int gi = j >> 2, limb = j & 3;
#pragma unroll
        for (int hg = 0; hg < HG; ++hg)
#pragma unroll
            for (int d = 0; d < 8; ++d)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float f = q_s[hg * 4 + gi][64 * (d >> 2) + 16 * kg + 4 * (d & 3) + x];
                    const __bf16 l0 = (__bf16)f;
                    const float r1 = f - (float)l0;
                    const __bf16 l1 = (__bf16)r1;
                    const float r2 = r1 - (float)l1;
                    const __bf16 l2 = (__bf16)r2;
                    const __bf16 v = limb == 0 ? l0 : (limb == 1 ? l1 : (limb == 2 ? l2 : (__bf16)0.0f));
                    aq[hg][d][x] = v;
                    aq[hg][d][4 + x] = v;
                }
    }

    // selectors that place a probability in the low (parity 0) or high (parity 1) half of an
    // A register of the value product; row r = j = 4*head + 2*parity + limb
    const int a_head = j >> 2, a_par = (j >> 1) & 1, a_limb = j & 1;
    const uint32_t sel_even = a_par ? 0x01000c0cu : 0x0c0c0100u;   // halfword 0 of the source
    const uint32_t sel_odd = a_par ? 0x03020c0cu : 0x0c0c0302u;    // halfword 1 of the source

    // Plane bases of this (batch, kv-head) are wave-uniform; everything inside the split is
    // addressed with 32-bit offsets from them.
    // (Paged cache: the bases are those of the pool and every 16-token stage of a tile looks up its page.)
    const int64_t base = PAGED ? 0 : ((int64_t)b * a.H_kv + kvh) * a.max_seq + t_begin;
    const uint8_t* __restrict__ k_mant = a.k_mant + base * 128;
    const uint8_t* __restrict__ v_mant = a.v_mant + base * 128;
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

    const uint32_t kchunk = (uint32_t)kg * 16u;                 // first chunk; the second is 64 bytes on
    const uint32_t keb0 = (uint32_t)((16 * kg) / N);            // exponent byte of the first chunk
    const uint32_t keb1 = (uint32_t)((64 + 16 * kg) / N);       // and of the second
    const uint32_t veb = (uint32_t)((8 * j) / N);               // exponent byte of value channels 8j..8j+7

    // One 64-token tile starting at token T0 of the split.  FULL: all 64 tokens are cached;
    // otherwise rows are clamped to the last cached token and masked.
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
            const uint8_t* __restrict__ kp = k_mant + tile_base(u) * 128;
            const uint8_t* __restrict__ kep = k_exp + tile_base(u) * NB;
            const uint32_t r = FULL ? (uint32_t)(16 * u + j) : (uint32_t)min(16 * u + j, left - 1);
            const u32x4 raw0 = __builtin_nontemporal_load((const u32x4*)(kp + r * 128u + kchunk));   // streamed once
            const u32x4 raw1 = __builtin_nontemporal_load((const u32x4*)(kp + r * 128u + kchunk + 64u));
            const uint32_t E0 = kep[r * NB + keb0];
            const uint32_t E1 = (N == 128) ? E0 : (uint32_t)kep[r * NB + keb1];
            const float sh0 = scale_hi(E0), sl0 = scale_lo(E0);
            const float sh1 = scale_hi(E1), sl1 = scale_lo(E1);
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) s_acc[hg][u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int d = 0; d < 8; ++d) {
                const Pieces kk = d < 4 ? unpack4(raw0[d & 3], sh0, sl0) : unpack4(raw1[d & 3], sh1, sl1);
                const bf16x8 bk = join(kk.h01, kk.h23, kk.l01, kk.l23);
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
            // Rescale the running output only when some head's maximum moved (alpha == 1 otherwise).
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
            const uint8_t* __restrict__ vp = v_mant + tile_base(u) * 128;
            const uint8_t* __restrict__ vep = v_exp + tile_base(u) * NB;
            Pieces va[4], vb[4];   // channels 8j..8j+3 and 8j+4..8j+7 of tokens 16u + 4kg + i
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t r = FULL ? (uint32_t)(16 * u + 4 * kg + i) : (uint32_t)min(16 * u + 4 * kg + i, left - 1);
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 wv = __builtin_nontemporal_load((const u32x2*)(vp + r * 128u + 8u * (uint32_t)j));   // streamed once
                const uint2 w = make_uint2(wv[0], wv[1]);
                const uint32_t E = vep[r * NB + veb];
                const float sh = scale_hi(E), sl = scale_lo(E);
                va[i] = unpack4(w.x, sh, sl);
                vb[i] = unpack4(w.y, sh, sl);
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
                // MFMA m: channel pair (8j + 2m, 8j + 2m + 1), hi pieces then lo pieces
                o_acc[hg][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(va[0].h01, va[1].h01, va[2].h01, va[3].h01), o_acc[hg][0], 0, 0, 0);
                o_acc[hg][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(va[0].l01, va[1].l01, va[2].l01, va[3].l01), o_acc[hg][0], 0, 0, 0);
                o_acc[hg][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(va[0].h23, va[1].h23, va[2].h23, va[3].h23), o_acc[hg][1], 0, 0, 0);
                o_acc[hg][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(va[0].l23, va[1].l23, va[2].l23, va[3].l23), o_acc[hg][1], 0, 0, 0);
                o_acc[hg][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(vb[0].h01, vb[1].h01, vb[2].h01, vb[3].h01), o_acc[hg][2], 0, 0, 0);
                o_acc[hg][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(vb[0].l01, vb[1].l01, vb[2].l01, vb[3].l01), o_acc[hg][2], 0, 0, 0);
                o_acc[hg][3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(vb[0].h23, vb[1].h23, vb[2].h23, vb[3].h23), o_acc[hg][3], 0, 0, 0);
                o_acc[hg][3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, join(vb[0].l23, vb[1].l23, vb[2].l23, vb[3].l23), o_acc[hg][3], 0, 0, 0);
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
            // result rows (parity 0: hi, lo limb), (parity 1: hi, lo limb) of channel pair m
            o_s[wave][head][8 * j + 2 * m] = o_acc[hg][m][0] + o_acc[hg][m][1];
            o_s[wave][head][8 * j + 2 * m + 1] = o_acc[hg][m][2] + o_acc[hg][m][3];
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

template <int HG, int PL, bool PAGED>
hipError_t launch_n(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    switch (block) {
        case 16: decode_split_mfma_p8<16, HG, PL, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        case 32: decode_split_mfma_p8<32, HG, PL, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        case 64: decode_split_mfma_p8<64, HG, PL, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        default: decode_split_mfma_p8<128, HG, PL, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
    }
    return hipGetLastError();
}

// The LDS-DMA pipeline (decode_lds.h) for 8-bit mantissas: 16-bit I/O.  Its staging area is twice that of the 4-bit
// pipeline (68 KB per workgroup), so two workgroups share a compute unit.
template <int N, int HG, bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 4)))
void decode_split_lds_p8(DecodeArgs a, int dt) {
    kvbfp::lds::decode_split_lds_body<8, N, HG, PAGED>(a, dt);
}

// The same with the query cast to 8-bit BFP and blocks of 32 and wider: the score product on the integer datapath
// (v_mfma_i32_16x16x64_i8 on the codes, block exponents added afterwards; Sec. II-B).
template <int N, int HG, bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 4)))
void decode_split_lds_p8_qi8(DecodeArgs a, int dt) {
    kvbfp::lds::decode_split_lds_body<8, N, HG, PAGED, true>(a, dt);
}

template <int HG, bool PAGED>
hipError_t launch_lds_qi8(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    switch (block) {
        case 32: decode_split_lds_p8_qi8<32, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        case 64: decode_split_lds_p8_qi8<64, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        default: decode_split_lds_p8_qi8<128, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
    }
    return hipGetLastError();
}

template <int HG, bool PAGED>
hipError_t launch_lds(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    switch (block) {
        case 16: decode_split_lds_p8<16, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        case 32: decode_split_lds_p8<32, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        case 64: decode_split_lds_p8<64, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
        default: decode_split_lds_p8<128, HG, PAGED><<<grid, 256, 0, s>>>(a, dt); break;
    }
    return hipGetLastError();
}

template <int HG, int PL>
hipError_t launch_p(const DecodeArgs& a, int dt, int block, dim3 grid, hipStream_t s) {
    return a.block_table ? launch_n<HG, PL, true>(a, dt, block, grid, s) : launch_n<HG, PL, false>(a, dt, block, grid, s);
}

}  // namespace

namespace kvbfp {

hipError_t launch_decode_split_mfma_p8(const DecodeArgs& a, int dtype, int block, int batch, hipStream_t s) {
    const dim3 grid((unsigned)a.n_splits, (unsigned)a.H_kv, (unsigned)batch);
    // fp32 outputs take three probability limbs (24 bits), 16-bit outputs two
    if (dtype == KVBFP_F32) return a.g_cnt <= 4 ? launch_p<1, 3>(a, dtype, block, grid, s) : launch_p<2, 3>(a, dtype, block, grid, s);
    if (a.q_mant_bits == 8 && block >= 32) {      // 8-bit query codes x 8-bit key codes: integer matrix product
        if (a.block_table) return a.g_cnt <= 4 ? launch_lds_qi8<1, true>(a, dtype, block, grid, s) : launch_lds_qi8<2, true>(a, dtype, block, grid, s);
        return a.g_cnt <= 4 ? launch_lds_qi8<1, false>(a, dtype, block, grid, s) : launch_lds_qi8<2, false>(a, dtype, block, grid, s);
    }
    if (a.block_table) return a.g_cnt <= 4 ? launch_lds<1, true>(a, dtype, block, grid, s) : launch_lds<2, true>(a, dtype, block, grid, s);
    return a.g_cnt <= 4 ? launch_lds<1, false>(a, dtype, block, grid, s) : launch_lds<2, false>(a, dtype, block, grid, s);
}

}  // namespace kvbfp
