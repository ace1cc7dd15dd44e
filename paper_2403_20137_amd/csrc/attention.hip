// Decode attention over the packed BFP cache for gfx950 (Sec. III run-time flow: cached keys are
// read back in block format and multiplied with the permuted query; the rest is ordinary softmax
// attention; values are handled the same way).
//
// Split-K over the sequence: pass 1 gives every (batch, kv-head, split) its own workgroup, which
// streams its token range once, keeps an online softmax (running maximum m, normaliser l,
// unnormalised output o) for the query heads that share the KV head, and writes (m, l, o) to the
// workspace; pass 2 merges the splits with the usual log-sum-exp weights, normalises, restores the
// original channel order of the values and rounds once to the output type.
//
// All softmax arithmetic is done in base 2: the query is pre-multiplied by softmax_scale*log2(e),
// so exp(x) becomes the native 2^x.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

#include "decode_args.h"
#include "decode_dev.h"
#include "kvbfp_internal.h"

using kvbfp::DecodeArgs;

namespace {

constexpr int kD = 128;
constexpr int kTile = kvbfp::kTokenTile;   // tokens per tile = threads per workgroup
constexpr int kHeadsPerWg = 4;             // query heads handled by one workgroup of the generic kernel


__device__ __forceinline__ float load_as_float(const void* p, int dt, int64_t i) {
    if (dt == KVBFP_F32) return ((const float*)p)[i];
    const uint32_t h = ((const uint16_t*)p)[i];
    if (dt == KVBFP_F16) return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
    return __uint_as_float(h << 16);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Signed integer value of a sign-magnitude code as a float.
template <int P>
__device__ __forceinline__ float code_value(uint32_t c) {
    const float m = (float)(c & ((1u << (P - 1)) - 1u));
    return (c >> (P - 1)) ? -m : m;
}

// Generic split pass: fp32 FMAs everywhere, any block size, any group size (query heads are processed
// four per workgroup; larger groups re-read the cache).  The fallback for what the matrix-core passes
// do not take: more than 32 (virtual) heads per kv-head, planes that are not 16-byte aligned.
// grid = (n_splits, H_kv * ceil(G/4), B), block = 256.
//
// ROPE: the keys were cached before the rotary embedding and are rotated here, at token index m = their
// position in the cache (Sec. III; Alg. 1 step 5 for the reordered parameters Theta', i', s').  With
// k_rot[j] = k'[j] cos(m Theta'[j]) + s'[j] k'[i'[j]] sin(m Theta'[j]) and the structure of the three
// vectors (i' an involution, equal Theta' and opposite s' within a pair) the score is
//     q'.k_rot = sum_j k'[j] ( q'[j] cos(m Theta'[j]) + q''[j] sin(m Theta'[j]) ),  q''[j] = -s'[j] q'[i'[j]],
// so no cached element has to meet its partner.  m = tile0 + r: the tile's angle is folded into the two
// query vectors once per tile (A = q' ch + q'' sh, B = q'' ch - q' sh), and the phasor of the offset r
// = 16 a + b inside the tile is the product of two 16-entry tables per channel.  Tables and the tile
// phasor are built in double precision from the fp32 frequencies (one sincos of Theta'[j], one of
// t_begin Theta'[j] and of the tile step, then complex products), so that angles of 10^5 radians keep
// fp32 accuracy.
template <int P, bool ROPE>
__global__ __launch_bounds__(kTile) void decode_split_generic(DecodeArgs a, int dt) {
    constexpr int kRowBytes = kD * P / 8;
    constexpr int kRowVec = kRowBytes / 16;
    __shared__ float qs[kHeadsPerWg][kD];                      // ROPE: A of the current tile
    __shared__ float qb[ROPE ? kHeadsPerWg : 1][kD];           // B of the current tile
    __shared__ float q1[ROPE ? kHeadsPerWg : 1][kD];           // q'
    __shared__ float q2[ROPE ? kHeadsPerWg : 1][kD];           // q''
    __shared__ float2 ph_lo[ROPE ? kD : 1][16];                // (cos, sin)(b Theta'[j]),    b < 16
    __shared__ float2 ph_mid[ROPE ? kD : 1][16];               // (cos, sin)(16 a Theta'[j]), a < 16
    __shared__ float sc[kHeadsPerWg][kTile];
    __shared__ float alpha_s[kHeadsPerWg];
    __shared__ float ored[4][kHeadsPerWg][kD];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int split = blockIdx.x;
    const int gg_count = (a.G + kHeadsPerWg - 1) / kHeadsPerWg;
    const int kvh = blockIdx.y / gg_count;
    const int g0 = (blockIdx.y % gg_count) * kHeadsPerWg;
    const int n_act = min(kHeadsPerWg, a.G - g0);
    const int b = blockIdx.z;
    const int h0 = kvh * a.G + g0;   // first query head of this workgroup

    int64_t L = a.seq_len ? (int64_t)a.seq_len[b] : a.max_len;
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    // 256-token tiles are dealt out round-robin: split s takes tiles s, s + n_splits, s + 2 n_splits, ...
    const int64_t t_begin = (int64_t)split * kTile;
    const int64_t t_end = L;
    const int64_t tile_step = (int64_t)a.n_splits * kTile;
    const int nb = kD >> a.log2_block;

    if (t_begin >= t_end) {   // nothing cached in this split
        for (int i = tid; i < n_act * kD; i += kTile) {
            const int g = i / kD, j = i % kD;
            a.part_o[(((int64_t)b * a.H_q + h0 + g) * a.n_splits + split) * kD + j] = 0.f;
        }
        if (tid < n_act) {
            float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + tid) * a.n_splits + split) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        return;
    }

    // q' = permuted query (optionally cast to BFP) times softmax_scale*log2(e); unused head slots are zero
    for (int i = tid; i < kHeadsPerWg * kD; i += kTile) {
        const int g = i / kD, j = i % kD;
        float v = 0.f;
        if (g < n_act) {
            const int c = a.perm_k ? (a.perm_k[kvh * kD + j] & (kD - 1)) : j;   // masked: device data the host cannot check
            v = load_as_float(a.q, dt, kvbfp::query_row(a, b, kvh, g0 + g) * kD + c);
        }
        qs[g][j] = a.q_mant_bits ? v : v * a.scale_log2e;
    }
    __syncthreads();
    if (a.q_mant_bits) {
        kvbfp::dev::bfp_round_queries(&qs[0][0], (uint32_t*)&sc[0][0], kHeadsPerWg, a.log2_block, a.q_mant_bits);
        for (int i = tid; i < kHeadsPerWg * kD; i += kTile) (&qs[0][0])[i] *= a.scale_log2e;
        __syncthreads();
    }

    double hi_c = 1.0, hi_s = 0.0, step_c = 1.0, step_s = 0.0;   // thread j < D: phasor of tile0 Theta'[j], of the tile step
    if (ROPE) {
        for (int i = tid; i < kHeadsPerWg * kD; i += kTile) (&q1[0][0])[i] = (&qs[0][0])[i];
        __syncthreads();
        for (int i = tid; i < kHeadsPerWg * kD; i += kTile) {
            const int g = i / kD, j = i % kD;
            q2[g][j] = -a.rope_sign[kvh * kD + j] * q1[g][a.rope_partner[kvh * kD + j] & (kD - 1)];
        }
        if (tid < kD) {
            const double th = (double)a.rope_theta[kvh * kD + tid];
            double c1, s1;
            sincos(th, &s1, &c1);
            double pc = 1.0, ps = 0.0;
            for (int k = 0; k < 16; ++k) {
                ph_lo[tid][k] = make_float2((float)pc, (float)ps);
                const double nc = pc * c1 - ps * s1;
                ps = ps * c1 + pc * s1;
                pc = nc;
            }
            const double c16 = pc, s16 = ps;
            pc = 1.0;
            ps = 0.0;
            for (int k = 0; k < 16; ++k) {
                ph_mid[tid][k] = make_float2((float)pc, (float)ps);
                const double nc = pc * c16 - ps * s16;
                ps = ps * c16 + pc * s16;
                pc = nc;
            }
            sincos((double)tile_step * th, &step_s, &step_c);     // from one of this workgroup's tiles to its next
            sincos((double)t_begin * th, &hi_s, &hi_c);
        }
        __syncthreads();
    }

    float m_run = -INFINITY, l_run = 0.f;          // wave g owns head g0+g (uniform per wave)
    float o[kHeadsPerWg][2];
#pragma unroll
    for (int g = 0; g < kHeadsPerWg; ++g) o[g][0] = o[g][1] = 0.f;
    const int cp = lane;                            // V phase: channels 2cp, 2cp+1

    for (int64_t tile0 = t_begin; tile0 < t_end; tile0 += tile_step) {
        if (ROPE) {   // the queries of this tile (nobody reads qs / qb between the end of a tile and here)
            if (tid < kD) {
                const float ch = (float)hi_c, sh = (float)hi_s;
#pragma unroll
                for (int g = 0; g < kHeadsPerWg; ++g) {
                    const float x = q1[g][tid], y = q2[g][tid];
                    qs[g][tid] = x * ch + y * sh;
                    qb[g][tid] = y * ch - x * sh;
                }
                const double nc = hi_c * step_c - hi_s * step_s;
                hi_s = hi_s * step_c + hi_c * step_s;
                hi_c = nc;
            }
            __syncthreads();
        }
        // rows of the planes are addressed as base + token; a paged cache with pages of 64 tokens or more has one
        // base per 64 tokens, the share of a wavefront in both phases below; with smaller pages every token looks
        // up its own row
        const int64_t tw = tile0 + wave * 64;
        const bool per_token = a.block_table != nullptr && a.log2_page < 6;
        const int64_t base = (tw < t_end && !per_token) ? kvbfp::cache_row(a, b, kvh, tw) - tw : 0;
        // ---- scores: one cached token per thread
        const int64_t t = tile0 + tid;
        float s[kHeadsPerWg];
#pragma unroll
        for (int g = 0; g < kHeadsPerWg; ++g) s[g] = -INFINITY;
        if (t < t_end) {
            uint4 raw[kRowVec];
            const int64_t krow = per_token ? kvbfp::cache_row(a, b, kvh, t) : base + t;
            const uint4* rp = (const uint4*)(a.k_mant + krow * kRowBytes);
#pragma unroll
            for (int i = 0; i < kRowVec; ++i) raw[i] = rp[i];
            const uint8_t* ep = a.k_exp + krow * nb;
#pragma unroll
            for (int g = 0; g < kHeadsPerWg; ++g) s[g] = 0.f;
#pragma unroll
            for (int c = 0; c < kD / 16; ++c) {      // 16 channels at a time (never straddles a block)
                const int E = ep[(c * 16) >> a.log2_block];
                const float scale = ldexpf(1.0f, E - 127 - (P - 2));
                float v[16];
                if (P == 4) {
                    const uint4 r = raw[c / 2];
                    const uint32_t w0 = (c & 1) ? r.z : r.x, w1 = (c & 1) ? r.w : r.y;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        v[i] = code_value<4>((w0 >> (4 * i)) & 0xFu);
                        v[8 + i] = code_value<4>((w1 >> (4 * i)) & 0xFu);
                    }
                } else {
                    const uint4 r = raw[c];
                    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                    for (int i = 0; i < 16; ++i) v[i] = code_value<8>((w[i / 4] >> (8 * (i % 4))) & 0xFFu);
                }
                if (ROPE) {
                    float acc[kHeadsPerWg];
#pragma unroll
                    for (int g = 0; g < kHeadsPerWg; ++g) acc[g] = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int j = c * 16 + i;
                        const float2 pm = ph_mid[j][tid >> 4], pl = ph_lo[j][tid & 15];
                        const float kc = v[i] * (pm.x * pl.x - pm.y * pl.y);     // k' cos((16a + b) Theta')
                        const float ks = v[i] * (pm.y * pl.x + pm.x * pl.y);     // k' sin(...)
#pragma unroll
                        for (int g = 0; g < kHeadsPerWg; ++g) acc[g] = fmaf(qs[g][j], kc, fmaf(qb[g][j], ks, acc[g]));
                    }
#pragma unroll
                    for (int g = 0; g < kHeadsPerWg; ++g) s[g] = fmaf(scale, acc[g], s[g]);
                } else {
#pragma unroll
                    for (int g = 0; g < kHeadsPerWg; ++g) {
                        float acc = 0.f;
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc = fmaf(qs[g][c * 16 + i], v[i], acc);
                        s[g] = fmaf(scale, acc, s[g]);
                    }
                }
            }
        }
#pragma unroll
        for (int g = 0; g < kHeadsPerWg; ++g)        // several query tokens: head slot g0+g does not see the last few tokens
            sc[g][tid] = t < L - kvbfp::hidden_tokens(a, g0 + g) ? s[g] : -INFINITY;
        __syncthreads();

        // ---- online softmax: wave g updates head g
        {
            const int g = wave;
            float sv[kTile / 64];
            float tmax = -INFINITY;
#pragma unroll
            for (int k = 0; k < kTile / 64; ++k) {
                sv[k] = sc[g][lane + 64 * k];
                tmax = fmaxf(tmax, sv[k]);
            }
            tmax = wave_max(tmax);                  // -inf only if this head sees none of the tile (several query tokens)
            const float m_new = fmaxf(m_run, tmax);
            const float m_ref = m_new == -INFINITY ? 0.f : m_new;
            float tsum = 0.f;
#pragma unroll
            for (int k = 0; k < kTile / 64; ++k) {
                const float pw = exp2f(sv[k] - m_ref);   // 2^-inf = 0 for padding
                sc[g][lane + 64 * k] = pw;
                tsum += pw;
            }
            tsum = wave_sum(tsum);
            const float al = exp2f(m_run - m_ref);       // 0 on the first tile
            l_run = l_run * al + tsum;
            m_run = m_new;
            if (lane == 0) alpha_s[g] = al;
        }
        __syncthreads();

        // ---- values: wave w takes tokens [64w, 64w+64) of the tile, lane = channel pair
#pragma unroll
        for (int g = 0; g < kHeadsPerWg; ++g) {
            const float al = alpha_s[g];
            o[g][0] *= al;
            o[g][1] *= al;
        }
        const int64_t tw0 = tile0 + wave * 64;
        const int cnt = (int)max((int64_t)0, min((int64_t)64, t_end - tw0));
        auto add_value_row = [&](const int k, const int64_t vrow) {
            const int E = a.v_exp[vrow * nb + ((2 * cp) >> a.log2_block)];
            const float scale = ldexpf(1.0f, E - 127 - (P - 2));
            float v0, v1;
            if (P == 4) {
                const uint32_t byte = a.v_mant[vrow * kRowBytes + cp];
                v0 = code_value<4>(byte & 0xFu) * scale;
                v1 = code_value<4>(byte >> 4) * scale;
            } else {
                const uint32_t two = ((const uint16_t*)(a.v_mant + vrow * kRowBytes))[cp];
                v0 = code_value<8>(two & 0xFFu) * scale;
                v1 = code_value<8>(two >> 8) * scale;
            }
#pragma unroll
            for (int g = 0; g < kHeadsPerWg; ++g) {
                const float pw = sc[g][wave * 64 + k];
                o[g][0] = fmaf(pw, v0, o[g][0]);
                o[g][1] = fmaf(pw, v1, o[g][1]);
            }
        };
        if (per_token) {      // its own loop: the look-up stays out of the common one
            for (int k = 0; k < cnt; ++k) add_value_row(k, kvbfp::cache_row(a, b, kvh, tw0 + k));
        } else {
            for (int k = 0; k < cnt; ++k) add_value_row(k, base + tw0 + k);
        }
        __syncthreads();   // sc and alpha_s are rewritten by the next tile
    }

    // ---- merge the four token slices and write the partial result of this split
#pragma unroll
    for (int g = 0; g < kHeadsPerWg; ++g) {
        ored[wave][g][2 * cp] = o[g][0];
        ored[wave][g][2 * cp + 1] = o[g][1];
    }
    __syncthreads();
    for (int i = tid; i < n_act * kD; i += kTile) {
        const int g = i / kD, j = i % kD;
        const float v = ored[0][g][j] + ored[1][g][j] + ored[2][g][j] + ored[3][g][j];
        a.part_o[(((int64_t)b * a.H_q + h0 + g) * a.n_splits + split) * kD + j] = v;
    }
    if (lane == 0 && wave < n_act) {
        float* ml = a.part_ml + (((int64_t)b * a.H_q + h0 + wave) * a.n_splits + split) * 2;
        ml[0] = m_run;
        ml[1] = l_run;
    }
}

__device__ __forceinline__ uint16_t narrow_bf16(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Pass 2: merge the splits of one (batch, query head).  block = 512 threads: kChan channels times 512 / kChan
// slices of the splits; grid = (H_q, B, 128 / kChan).  A round trip to memory costs far more than anything computed
// here, so every thread first puts kCombineBatch partial-output loads in flight (enough for all splits in one go
// up to kCombineBatch * slices of them), then the (m, l) pairs go through LDS, and the slices are added through LDS
// at the end.  Few (batch, head) pairs with many splits -- one long sequence -- take the 32-channel form: four
// times the workgroups, a quarter of the bytes through each compute unit.
constexpr int kCombineThreads = 512;
template <int kCombineBatch, int kChan>
__global__ __launch_bounds__(kCombineThreads) void decode_combine(DecodeArgs a, int dt) {
    constexpr int kSlices = kCombineThreads / kChan;
    constexpr int kMaxLds = 1024;
    __shared__ float m_s[kMaxLds];
    __shared__ float l_s[kMaxLds];
    __shared__ float red[kSlices][2][kChan];
    __shared__ float red_m[kSlices];
    const int jl = threadIdx.x % kChan, sl = threadIdx.x / kChan;
    const int j = blockIdx.z * kChan + jl;      // channel (cache order)
    const int h = blockIdx.x, b = blockIdx.y;
    const int64_t bh = (int64_t)b * a.H_q + h;
    const float* ml = a.part_ml + bh * a.n_splits * 2;
    const float* po = a.part_o + bh * a.n_splits * kD;
    const int n = a.n_splits;
    const bool staged = n <= kMaxLds;           // otherwise (m, l) are read from global memory each time

    // where this channel goes in the output row: requested with the partial outputs, not after the sums (a load here
    // costs nothing, at the end it is one more round trip to memory)
    const int kvh = h / a.G;
    const int c_raw = a.perm_v ? a.perm_v[kvh * kD + j] : j;
    float v[kCombineBatch];                     // first batch of this thread's partial outputs: splits sl + kSlices k
#pragma unroll
    for (int k = 0; k < kCombineBatch; ++k) {
        const int i = sl + k * kSlices;
        v[k] = i < n ? po[(int64_t)i * kD + j] : 0.f;
    }
    if (staged) {
        for (int i = threadIdx.x; i < n; i += kCombineThreads) {
            const float2 t = *(const float2*)(ml + 2 * i);
            m_s[i] = t.x;
            l_s[i] = t.y;
        }
        __syncthreads();
    }
    auto m_of = [&](int i) { return staged ? m_s[i] : ml[2 * i]; };
    auto l_of = [&](int i) { return staged ? l_s[i] : ml[2 * i + 1]; };
    // Each slice works relative to the maximum of its own splits (a short, unrolled scan instead of
    // one long serial loop over all of them); the slices are brought to the common maximum at the end.
    float mk[kCombineBatch];
    float Ms = -INFINITY;
#pragma unroll
    for (int k = 0; k < kCombineBatch; ++k) {
        const int i = sl + k * kSlices;
        mk[k] = i < n ? m_of(i) : -INFINITY;
        Ms = fmaxf(Ms, mk[k]);
    }
    for (int i = sl + kCombineBatch * kSlices; i < n; i += kSlices) Ms = fmaxf(Ms, m_of(i));
    float num = 0.f, den = 0.f;
    if (Ms > -INFINITY) {                       // empty splits carry m = -inf -> weight 0
#pragma unroll
        for (int k = 0; k < kCombineBatch; ++k) {
            const int i = sl + k * kSlices;
            if (i < n) {
                const float w = exp2f(mk[k] - Ms);
                num = fmaf(w, v[k], num);
                den = fmaf(w, l_of(i), den);
            }
        }
        for (int i = sl + kCombineBatch * kSlices; i < n; i += kSlices) {
            const float w = exp2f(m_of(i) - Ms);
            num = fmaf(w, po[(int64_t)i * kD + j], num);
            den = fmaf(w, l_of(i), den);
        }
    }
    red[sl][0][jl] = num;
    red[sl][1][jl] = den;
    if (jl == 0) red_m[sl] = Ms;
    __syncthreads();
    if (sl != 0) return;
    float M = -INFINITY;
#pragma unroll
    for (int k = 0; k < kSlices; ++k) M = fmaxf(M, red_m[k]);
    num = 0.f;
    den = 0.f;
    if (M > -INFINITY) {
#pragma unroll
        for (int k = 0; k < kSlices; ++k) {
            const float w = exp2f(red_m[k] - M);        // 0 for a slice without cached tokens
            num = fmaf(w, red[k][0][jl], num);
            den = fmaf(w, red[k][1][jl], den);
        }
    }
    const float r = den > 0.f ? num / den : 0.f;
    const int c = c_raw & (kD - 1);             // masked: the store stays inside the row
    const int64_t oi = kvbfp::query_row(a, b, kvh, h % a.G) * kD + c;
    if (dt == KVBFP_F32) ((float*)a.out)[oi] = r;
    else if (dt == KVBFP_F16) ((uint16_t*)a.out)[oi] = __builtin_bit_cast(unsigned short, (_Float16)r);
    else ((uint16_t*)a.out)[oi] = narrow_bf16(r);
}

int log2_exact(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

}  // namespace

using namespace kvbfp;

extern "C" {

size_t kvbfp_decode_workspace_bytes(const kvbfp_layout* L, int32_t n_q_heads, int64_t max_len) {
    clear_error();
    if (check_device_layout(L) != KVBFP_OK) return 0;
    if (n_q_heads <= 0 || n_q_heads % L->n_kv_heads != 0 || max_len <= 0 || max_len > L->max_seq) {
        fail(KVBFP_ERR_INVALID_ARG, "decode_workspace_bytes: bad n_q_heads/max_len");
        return 0;
    }
    const SplitPlan sp = plan_splits(L, n_q_heads, max_len);
    return (size_t)L->batch * (size_t)n_q_heads * (size_t)sp.n_splits * (size_t)(kD + 2) * sizeof(float);
}

// What the variants of the decode call add to the plain one; the defaults are the plain call.
struct DecodeExtras {
    int32_t q_mant_bits = 0;                 // query cast to BFP first (kvbfp_decode_attention_qbfp)
    float* kernel_ms = nullptr;              // HOST float[2]: wait and return the two kernel durations
    const void* k_new = nullptr;             // the current token, appended first (kvbfp_append_decode_attention)
    const void* v_new = nullptr;
    int64_t new_stride_b = 0, new_stride_h = 0;
    int32_t n_q_tokens = 1;                  // kvbfp_decode_attention_multi
    const float* rope_theta = nullptr;       // rotation at read (kvbfp_decode_attention_rope)
    const int32_t* rope_partner = nullptr;
    const float* rope_sign = nullptr;
    const Paging* paging = nullptr;          // L is a pool of pages (kvbfp_decode_attention_paged)
    // kvbfp_decode_attention_profile_ring: with kernel_ms, the split pass is launched `reps` times back to back over
    // the caches ring[0], ring[1], ... (cyclically) between the first two events, then the combine pass `reps`
    // times between the last two; the durations returned are per launch.
    const kvbfp_cache* ring = nullptr;
    int32_t ring_len = 0, reps = 1;
};

static int decode_impl(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                       const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                       int64_t max_len, float softmax_scale, const int32_t* perm_k,
                       const int32_t* perm_v, void* out, void* workspace, size_t workspace_bytes,
                       void* hip_stream, const DecodeExtras& x = DecodeExtras{}) {
    const int32_t q_mant_bits = x.q_mant_bits, n_q_tokens = x.n_q_tokens;
    float* const kernel_ms = x.kernel_ms;
    const void* const k_new = x.k_new;
    const void* const v_new = x.v_new;
    const int64_t new_stride_b = x.new_stride_b, new_stride_h = x.new_stride_h;
    const float* const rope_theta = x.rope_theta;
    const int32_t* const rope_partner = x.rope_partner;
    const float* const rope_sign = x.rope_sign;
    const Paging* const paging = x.paging;
    clear_error();
    kvbfp_layout logical;
    const kvbfp_layout* pool = L;
    if (paging) {
        if (int rc = check_paging(pool, *paging, &logical)) return rc;
        L = &logical;             // from here on: what the sequences look like
    }
    const bool rope = rope_theta || rope_partner || rope_sign;
    if (rope && !(rope_theta && rope_partner && rope_sign))
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention_rope: rope_theta, rope_partner and rope_sign are all needed");
    if (rope && (q_mant_bits != 0 || n_q_tokens != 1 || k_new || v_new))
        return fail(KVBFP_ERR_UNSUPPORTED, "decode_attention_rope: plain single-token decode only");
    if (n_q_tokens < 1 || n_q_tokens > 64)
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: n_q_tokens = %d (1..64)", n_q_tokens);
    if (q_mant_bits != 0 && q_mant_bits != 4 && q_mant_bits != 8)
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: q_mant_bits = %d (0, 4 or 8)", q_mant_bits);
    if (int rc = check_device_layout(L)) return rc;
    if (int rc = check_cache(cache, true, true)) return rc;
    if (!q || !out) return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: q/out is NULL");
    if (dtype_size(dtype) == 0) return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: unknown dtype %d", (int)dtype);
    if (n_q_heads <= 0 || n_q_heads % L->n_kv_heads != 0)
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: n_q_heads %d not a multiple of n_kv_heads %d",
                    n_q_heads, L->n_kv_heads);
    if (max_len <= 0 || max_len > L->max_seq)
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: max_len %lld outside (0, max_seq=%lld]",
                    (long long)max_len, (long long)L->max_seq);
    if (!std::isfinite(softmax_scale))
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention: softmax_scale is not finite");
    // from here on "heads" are virtual heads: every query token brings its own set (see DecodeArgs)
    const int32_t real_heads = n_q_heads;
    n_q_heads *= n_q_tokens;
    const size_t need = kvbfp_decode_workspace_bytes(L, n_q_heads, max_len);
    if (!workspace || workspace_bytes < need)
        return fail(KVBFP_ERR_WORKSPACE, "decode_attention: workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : (size_t)0);
    if ((uintptr_t)workspace % 256 != 0)
        return fail(KVBFP_ERR_WORKSPACE, "decode_attention: workspace must be 256-byte aligned");
    if ((int64_t)L->batch > 65535 || (int64_t)n_q_heads > 65535)
        return fail(KVBFP_ERR_UNSUPPORTED, "decode_attention: batch/heads exceed the grid limits");

    SplitPlan sp = plan_splits(L, n_q_heads, max_len);       // what the workspace is sized for
    DecodeArgs a{};
    a.k_mant = cache->k_mant; a.k_exp = cache->k_exp; a.v_mant = cache->v_mant; a.v_exp = cache->v_exp;
    a.q = q; a.out = out; a.seq_len = seq_len_dev; a.perm_k = perm_k; a.perm_v = perm_v;
    a.part_o = (float*)workspace;
    a.max_seq = L->max_seq; a.max_len = max_len;
    a.H_kv = L->n_kv_heads; a.H_q = n_q_heads; a.G = n_q_heads / L->n_kv_heads;
    a.log2_block = log2_exact(L->block);
    a.n_q_tokens = n_q_tokens; a.real_Hq = real_heads; a.real_G = real_heads / L->n_kv_heads;
    a.q_mant_bits = q_mant_bits;
    a.scale_log2e = softmax_scale * 1.4426950408889634f;
    a.rope_theta = rope_theta; a.rope_partner = rope_partner; a.rope_sign = rope_sign;
    if (paging) {
        a.block_table = paging->block_table; a.table_stride = paging->table_stride;
        a.n_pages = pool->batch;
        a.log2_page = log2_exact((int)pool->max_seq);
    }

    hipStream_t s = (hipStream_t)hip_stream;
    const int gg = (a.G + kHeadsPerWg - 1) / kHeadsPerWg;
    if ((int64_t)a.H_kv * gg > 65535)
        return fail(KVBFP_ERR_UNSUPPORTED, "decode_attention: too many heads for the grid");
    auto aligned16 = [](const void* p) { return ((uintptr_t)p & 15u) == 0; };
    // Matrix-core passes (not with the rotation at read): up to 8 (virtual) heads of a kv-head per launch; larger groups take
    // several launches over head subsets (the cache is then read once per subset), up to 4 of them.
    // (mantissa planes are 16-byte aligned, checked above; exponent planes that are not go to the general
    // pass, which reads them byte by byte)
    const bool fast = !rope && a.G <= 32 && aligned16(a.k_exp) && aligned16(a.v_exp);
    // rotation at read: the matrix-core pass takes 4-bit mantissas with 16-bit I/O, four heads per launch
    const bool rope_fast = rope && !paging && dtype != KVBFP_F32 && L->mant_bits == 4 && a.G <= 32 &&
                           aligned16(a.k_exp) && aligned16(a.v_exp);
    // (its workgroups hold a 64 KB table in LDS, two fit a compute unit: fewer splits, one resident round)
    if (rope_fast) {
        const int64_t units = (int64_t)L->batch * L->n_kv_heads;
        const int64_t two_per_cu = (512 + units - 1) / units;
        if (sp.n_splits > two_per_cu) sp.n_splits = (int32_t)two_per_cu;
    }
    a.n_splits = sp.n_splits;
    a.part_ml = a.part_o + (size_t)L->batch * n_q_heads * sp.n_splits * kD;
    const dim3 grid1((unsigned)sp.n_splits, (unsigned)(a.H_kv * gg), (unsigned)L->batch);
    a.g_base = 0;
    a.g_cnt = a.G < 8 ? a.G : 8;
    // The current token (kvbfp_append_decode_attention): cast inside the LDS split pass, else by the
    // cache-write kernel ahead of the split pass.  Either way it lands at position seq_len - 1.
    if (k_new || v_new) {
        if (!k_new || !v_new) return fail(KVBFP_ERR_INVALID_ARG, "append_decode_attention: k_new and v_new are both needed");
        if (n_q_tokens != 1) return fail(KVBFP_ERR_UNSUPPORTED, "append_decode_attention: one query token only");
        if (new_stride_b < 0 || new_stride_h < 0)
            return fail(KVBFP_ERR_INVALID_ARG, "append_decode_attention: negative stride");
        // Inside the LDS split pass the cast is done by the one wavefront that reads the new row, off
        // the path of everybody else; elsewhere the cache-write kernel goes first, as in the two calls.
        const bool in_kernel = fast && dtype != KVBFP_F32;      // the LDS pipeline: every block size, both mantissa widths
        if (in_kernel) {
            a.k_new = k_new; a.v_new = v_new; a.new_stride_b = new_stride_b; a.new_stride_h = new_stride_h;
        } else {
            if (int rc = kvbfp::quantize_append_impl(pool, cache, k_new, v_new, dtype, 1, new_stride_b, 0, new_stride_h,
                                                     max_len - 1, seq_len_dev, max_len, perm_k, perm_v, hip_stream,
                                                     paging))
                return rc;
        }
    }
    // Optional timing of the two launches (kvbfp_decode_attention_profile): events on the same stream.
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    if (kernel_ms) {
        for (auto& e : ev)
            if (hipEventCreate(&e) != hipSuccess) {
                for (auto& made : ev)
                    if (made) (void)hipEventDestroy(made);
                return fail(KVBFP_ERR_HIP, "decode_attention_profile: hipEventCreate failed");
            }
        (void)hipEventRecord(ev[0], s);
    }
    hipError_t err = hipSuccess;
    auto launch_split = [&]() {
        if (fast) {
            // heads per launch: 8, or 16 where the LDS pipeline applies and more than 8 are left (its
            // sixteen-head variant keeps two workgroups per CU resident instead of three)
            const bool lds_path = dtype != KVBFP_F32 && L->mant_bits == 4 && L->block <= 32;
            for (int g0 = 0; g0 < a.G && err == hipSuccess; g0 += a.g_cnt) {
                const int left = a.G - g0;
                a.g_base = g0;
                a.g_cnt = (lds_path && left > 8) ? (left < 16 ? left : 16) : (left < 8 ? left : 8);
                err = L->mant_bits == 4 ? launch_decode_split_mfma(a, (int)dtype, L->block, L->batch, s)
                                        : launch_decode_split_mfma_p8(a, (int)dtype, L->block, L->batch, s);
                a.k_new = a.v_new = nullptr;       // the current token is cast by the first launch only
            }
        } else if (rope_fast) {
            for (int g0 = 0; g0 < a.G && err == hipSuccess; g0 += 4) {
                a.g_base = g0;
                a.g_cnt = a.G - g0 < 4 ? a.G - g0 : 4;
                err = launch_decode_split_rope(a, (int)dtype, L->block, L->batch, s);
            }
        } else {
            if (rope) {
                if (L->mant_bits == 4) decode_split_generic<4, true><<<grid1, kTile, 0, s>>>(a, (int)dtype);
                else decode_split_generic<8, true><<<grid1, kTile, 0, s>>>(a, (int)dtype);
            } else {
                if (L->mant_bits == 4) decode_split_generic<4, false><<<grid1, kTile, 0, s>>>(a, (int)dtype);
                else decode_split_generic<8, false><<<grid1, kTile, 0, s>>>(a, (int)dtype);
            }
            err = hipGetLastError();
        }
    };
    const int reps = (kernel_ms && x.ring && x.ring_len > 0 && x.reps > 1) ? x.reps : 1;
    for (int r = 0; r < reps && err == hipSuccess; ++r) {
        if (reps > 1) {
            const kvbfp_cache& c = x.ring[r % x.ring_len];
            a.k_mant = c.k_mant; a.k_exp = c.k_exp; a.v_mant = c.v_mant; a.v_exp = c.v_exp;
        }
        launch_split();
    }
    if (kernel_ms) (void)hipEventRecord(ev[1], s);
    for (int r = 0; r < reps && err == hipSuccess; ++r) {
        // few (batch, head) pairs with many splits: 32 channels per workgroup (16 slices x 8 loads cover 128 splits)
        if (sp.n_splits > 32 && (int64_t)n_q_heads * L->batch < 256) {
            const dim3 grid2((unsigned)n_q_heads, (unsigned)L->batch, kD / 32);
            decode_combine<8, 32><<<grid2, kCombineThreads, 0, s>>>(a, (int)dtype);
        } else {
            const dim3 grid2((unsigned)n_q_heads, (unsigned)L->batch, 1);
            if (sp.n_splits <= 32) decode_combine<8, kD><<<grid2, kCombineThreads, 0, s>>>(a, (int)dtype);
            else decode_combine<32, kD><<<grid2, kCombineThreads, 0, s>>>(a, (int)dtype);
        }
        err = hipGetLastError();
    }
    if (kernel_ms) {
        (void)hipEventRecord(ev[2], s);
        hipError_t e2 = hipEventSynchronize(ev[2]);
        if (e2 == hipSuccess) e2 = hipEventElapsedTime(&kernel_ms[0], ev[0], ev[1]);
        if (e2 == hipSuccess) e2 = hipEventElapsedTime(&kernel_ms[1], ev[1], ev[2]);
        kernel_ms[0] /= (float)reps;
        kernel_ms[1] /= (float)reps;
        for (auto& e : ev) (void)hipEventDestroy(e);
        if (err == hipSuccess) err = e2;
    }
    if (err != hipSuccess) return fail(KVBFP_ERR_HIP, "decode_attention: %s", hipGetErrorString(err));
    return KVBFP_OK;
}

int kvbfp_decode_attention(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                           const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                           int64_t max_len, float softmax_scale, const int32_t* perm_k,
                           const int32_t* perm_v, void* out, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream);
}

int kvbfp_decode_attention_qbfp(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                                const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                                int64_t max_len, float softmax_scale, const int32_t* perm_k,
                                const int32_t* perm_v, int32_t q_mant_bits, void* out, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

int kvbfp_append_decode_attention(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                                  const void* k_new, const void* v_new, int64_t new_stride_b,
                                  int64_t new_stride_h, const void* q, kvbfp_dtype dtype,
                                  const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                  const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits,
                                  void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!k_new || !v_new) {
        clear_error();
        return fail(KVBFP_ERR_INVALID_ARG, "append_decode_attention: k_new/v_new is NULL");
    }
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.k_new = k_new; x.v_new = v_new; x.new_stride_b = new_stride_b; x.new_stride_h = new_stride_h;
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

int kvbfp_decode_attention_multi(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                                 int32_t n_q_tokens, const void* q, kvbfp_dtype dtype,
                                 const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                 const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits, void* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.n_q_tokens = n_q_tokens;
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

int kvbfp_decode_attention_rope(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                                const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                                int64_t max_len, float softmax_scale, const int32_t* perm_k,
                                const int32_t* perm_v, const float* rope_theta, const int32_t* rope_partner,
                                const float* rope_sign, void* out, void* workspace, size_t workspace_bytes,
                                void* hip_stream, float* kernel_ms) {
    if (!rope_theta || !rope_partner || !rope_sign) {
        clear_error();
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention_rope: rope_theta/rope_partner/rope_sign is NULL");
    }
    DecodeExtras x;
    x.kernel_ms = kernel_ms;
    x.rope_theta = rope_theta; x.rope_partner = rope_partner; x.rope_sign = rope_sign;
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

size_t kvbfp_decode_workspace_bytes_paged(const kvbfp_layout* pool, int64_t table_stride, int32_t batch,
                                          int32_t n_q_heads, int64_t max_len) {
    clear_error();
    static const int32_t placeholder = 0;      // only its address is looked at here
    const Paging pg{&placeholder, table_stride, batch};
    kvbfp_layout logical;
    if (check_paging(pool, pg, &logical) != KVBFP_OK) return 0;
    return kvbfp_decode_workspace_bytes(&logical, n_q_heads, max_len);
}

int kvbfp_decode_attention_paged(const kvbfp_layout* pool, const kvbfp_cache* cache, const int32_t* block_table,
                                 int64_t table_stride, int32_t batch, int32_t n_q_heads, const void* q,
                                 kvbfp_dtype dtype, const int32_t* seq_len_dev, int64_t max_len,
                                 float softmax_scale, const int32_t* perm_k, const int32_t* perm_v,
                                 int32_t q_mant_bits, void* out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, float* kernel_ms) {
    const Paging pg{block_table, table_stride, batch};
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.kernel_ms = kernel_ms;
    x.paging = &pg;
    return decode_impl(pool, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

int kvbfp_append_decode_attention_paged(const kvbfp_layout* pool, const kvbfp_cache* cache,
                                        const int32_t* block_table, int64_t table_stride, int32_t batch,
                                        int32_t n_q_heads, const void* k_new, const void* v_new,
                                        int64_t new_stride_b, int64_t new_stride_h, const void* q, kvbfp_dtype dtype,
                                        const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                        const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits, void* out,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!k_new || !v_new) {
        clear_error();
        return fail(KVBFP_ERR_INVALID_ARG, "append_decode_attention_paged: k_new/v_new is NULL");
    }
    const Paging pg{block_table, table_stride, batch};
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.k_new = k_new; x.v_new = v_new; x.new_stride_b = new_stride_b; x.new_stride_h = new_stride_h;
    x.paging = &pg;
    return decode_impl(pool, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

int kvbfp_decode_attention_multi_paged(const kvbfp_layout* pool, const kvbfp_cache* cache,
                                       const int32_t* block_table, int64_t table_stride, int32_t batch,
                                       int32_t n_q_heads, int32_t n_q_tokens, const void* q, kvbfp_dtype dtype,
                                       const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                       const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits, void* out,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    const Paging pg{block_table, table_stride, batch};
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.n_q_tokens = n_q_tokens;
    x.paging = &pg;
    return decode_impl(pool, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

// ---- kvbfp_decode_attention_noalloc: the partial results of the splits live in a file-scope device
// array instead of a caller's workspace.  Every GPU holds its own copy of the array; its address on a
// device is asked for once, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[KVBFP_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (nullptr + recorded error on failure).
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(KVBFP_ERR_HIP, "decode_attention_noalloc: cannot identify the current device");
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            fail(KVBFP_ERR_HIP, "decode_attention_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int kvbfp_decode_attention_noalloc(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                                   const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                                   int64_t max_len, float softmax_scale, const int32_t* perm_k,
                                   const int32_t* perm_v, int32_t q_mant_bits, void* out, void* hip_stream) {
    clear_error();
    // the size check comes first: a geometry that does not fit is refused before anything else happens
    const size_t need = kvbfp_decode_workspace_bytes(L, n_q_heads, max_len);
    if (need == 0) return fail(KVBFP_ERR_INVALID_ARG, "decode_attention_noalloc: bad layout, n_q_heads or max_len");
    if (need > (size_t)KVBFP_NOALLOC_SCRATCH_BYTES)
        return fail(KVBFP_ERR_WORKSPACE,
                    "decode_attention_noalloc: this geometry needs %zu bytes of split partials, the built-in "
                    "scratch holds %zu; use kvbfp_decode_attention with a workspace",
                    need, (size_t)KVBFP_NOALLOC_SCRATCH_BYTES);
    void* const ws = scratch_on_current_device();
    if (!ws) return KVBFP_ERR_HIP;
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out, ws,
                       (size_t)KVBFP_NOALLOC_SCRATCH_BYTES, hip_stream, x);
}

int kvbfp_decode_attention_profile(const kvbfp_layout* L, const kvbfp_cache* cache, int32_t n_q_heads,
                                   const void* q, kvbfp_dtype dtype, const int32_t* seq_len_dev,
                                   int64_t max_len, float softmax_scale, const int32_t* perm_k,
                                   const int32_t* perm_v, int32_t q_mant_bits, void* out, void* workspace,
                                   size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
    if (!kernel_ms) {
        clear_error();
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention_profile: kernel_ms is NULL");
    }
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.kernel_ms = kernel_ms;
    return decode_impl(L, cache, n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

int kvbfp_decode_attention_profile_ring(const kvbfp_layout* L, const kvbfp_cache* caches, int32_t n_caches,
                                        int32_t n_launches, int32_t n_q_heads, const void* q, kvbfp_dtype dtype,
                                        const int32_t* seq_len_dev, int64_t max_len, float softmax_scale,
                                        const int32_t* perm_k, const int32_t* perm_v, int32_t q_mant_bits, void* out,
                                        void* workspace, size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
    clear_error();
    if (!kernel_ms) return fail(KVBFP_ERR_INVALID_ARG, "decode_attention_profile_ring: kernel_ms is NULL");
    if (!caches || n_caches <= 0 || n_launches <= 0 || n_launches > 4096)
        return fail(KVBFP_ERR_INVALID_ARG, "decode_attention_profile_ring: caches / n_caches / n_launches (1..4096)");
    for (int i = 0; i < n_caches; ++i)
        if (int rc = check_cache(&caches[i], true, true)) return rc;
    DecodeExtras x;
    x.q_mant_bits = q_mant_bits;
    x.kernel_ms = kernel_ms;
    x.ring = caches; x.ring_len = n_caches; x.reps = n_launches;
    return decode_impl(L, &caches[0], n_q_heads, q, dtype, seq_len_dev, max_len, softmax_scale, perm_k, perm_v, out,
                       workspace, workspace_bytes, hip_stream, x);
}

}  // extern "C"
