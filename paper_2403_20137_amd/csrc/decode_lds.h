// LDS-DMA pipeline of the decode split pass (internal; included by the translation units that instantiate it).
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>
#include <utility>

#include "decode_args.h"
#include "decode_dev.h"
#include "kvbfp_internal.h"
#include "quantize_dev.h"

namespace kvbfp {
namespace lds {

using kvbfp::DecodeArgs;
using namespace kvbfp::dev;

// scale operand of the conversions: only the exponent field is looked at, and it is the stored exponent byte
__device__ __forceinline__ float scale_operand(uint32_t E) { return __uint_as_float(E << 23); }
// 8 sign-magnitude nibbles -> 8 bf16 values in slot order [c0,c2,c4,c6,c1,c3,c5,c7] (the nibble s|mmm widened to
// the byte s0000mmm is the FP8-E4M3 subnormal (-1)^s m 2^-9)
struct Unpacked4 { bf16x2 p[4]; };
__device__ __forceinline__ Unpacked4 unpack8_p4(uint32_t w, float scale) {
    const uint32_t lo = ((w << 4) & 0x80808080u) | (w & 0x07070707u);          // even nibbles as FP8 bytes
    const uint32_t hi = (w & 0x80808080u) | ((w >> 4) & 0x07070707u);          // odd nibbles
    Unpacked4 u;
    u.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, false);      // (c0, c2)
    u.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, scale, true);       // (c4, c6)
    u.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, false);      // (c1, c3)
    u.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, scale, true);       // (c5, c7)
    return u;
}
// 8-bit mantissas: the byte s mmmm lll is split into s000mmmm and s0000lll, both valid FP8-E4M3 numbers (the
// subnormals and the first binade share one spacing: s000xxxx reads as +-x 2^-9 for x = 0..15).  4 bytes ->
// hi pieces (c0,c1), (c2,c3) and lo pieces (c0,c1), (c2,c3) as bf16 pairs; the hi piece takes 8 times the scale.
struct Pieces8 { bf16x2 h01, h23, l01, l23; };
__device__ __forceinline__ Pieces8 unpack4_p8(uint32_t w, float s_hi, float s_lo) {
    const uint32_t hi = ((w >> 3) & 0x0F0F0F0Fu) | (w & 0x80808080u);
    const uint32_t lo = w & 0x87878787u;
    Pieces8 r;
    r.h01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, s_hi, false);
    r.h23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, s_hi, true);
    r.l01 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, s_lo, false);
    r.l23 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, s_lo, true);
    return r;
}
typedef int v4i __attribute__((ext_vector_type(4)));
// four sign-magnitude bytes -> four two's-complement bytes (a stored code is never "minus zero", so no carry
// crosses a byte)
__device__ __forceinline__ int twos_complement4(uint32_t w) {
    const uint32_t mag = w & 0x7F7F7F7Fu, sgn = (w >> 7) & 0x01010101u;
    const uint32_t ones = (sgn << 8) - sgn;             // 0xFF in every negative byte
    return (int)((mag ^ ones) + sgn);
}
// channel offset inside a dword of MFMA slot x
__device__ __forceinline__ int slot_channel(int x) { return (x < 4) ? 2 * x : 2 * (x - 4) + 1; }

// ------------------------------------------------------------------------------------------------
// LDS-staged split pass (Sec. III run-time flow; every block size, 4- and 8-bit mantissas, fp16/bf16 I/O):
// the packed rows travel global -> LDS by DMA (global_load_lds) instead of through registers, so every
// wavefront keeps most of a 64-token tile in flight without holding registers for it.
//   * Keys are not unpacked at all.  4-bit: the raw nibbles are the FP4 operand of the scaled FP8 x FP4 MFMA
//     (v_mfma_scale_f32_16x16x128_f8f6f4) and the block exponent byte is its E8M0 scale.  8-bit: the two
//     pieces s000mmmm and s0000lll of every byte are FP8 operands as they are (two masks and a shift per
//     dword), the high piece with the block's exponent byte + 3 as its scale.  The query is four FP8 limbs
//     with a power-of-two scale per 32 channels.
//   * Values are converted to bf16 (one instruction per two codes, the exponent byte as its scale operand)
//     and go through v_mfma_f32_16x16x32_bf16 with the probabilities as the other operand.
//
// Each wavefront owns a private staging area of four 16-token stages for keys and four for values
// (1 KB of 4-bit or 2 KB of 8-bit mantissas per stage = one or two DMA instructions) plus the exponent
// bytes of the whole tile per plane.  A stage is re-filled for the wavefront's next tile right after its
// last read, in the fixed order K0, key exponents, K1..K3, V0, value exponents, V1..V3.  DMA completes in
// issue order, so when a stage is about to be read, everything issued after it may still be outstanding
// and nothing else: one s_waitcnt vmcnt(constant) per stage is the whole synchronisation.  The compiler
// does not model the DMA -> ds_read dependency, hence the explicit waits and scheduling barriers; the
// main loop contains no other vector-memory instruction.
//
// 4-bit key stage: DMA lane 4r+c fetches chunk c ^ (r/4 % 4) of row r (four neighbouring lanes cover one
// 64-byte row, so the global access coalesces like a linear copy); lane (j, kg) then reads slot
// 4j + (kg ^ (j/4 % 4)), which spreads every group of 16 lanes over all banks.  4-bit value stage: the 16
// rows are stored in the order 4*(row%4) + row/4, which makes the dword reads of lanes (j, kg) -> row 4kg+i,
// dword j hit 64 different banks.  8-bit stages: eight lanes per 128-byte row; key chunks swizzled with
// row/2 % 8, value rows in the same 4*(row%4) + row/4 order, read eight bytes at a time.
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
// four dword reads, STRIDE apart
template <int OFF, int STRIDE>
__device__ __forceinline__ void lds_issue_4w(uint32_t addr, uint32_t (&e)[4]) {
    asm volatile("ds_read_b32 %0, %4 offset:%5\n\tds_read_b32 %1, %4 offset:%6\n\tds_read_b32 %2, %4 offset:%7\n\tds_read_b32 %3, %4 offset:%8"
                 : "=&v"(e[0]), "=&v"(e[1]), "=&v"(e[2]), "=&v"(e[3])
                 : "v"(addr), "n"(OFF), "n"(OFF + STRIDE), "n"(OFF + 2 * STRIDE), "n"(OFF + 3 * STRIDE) : "memory");
}
// value mantissas of stage U: dwords at m_addr + 256 * (4U + i), i = 0..3
template <int U>
__device__ __forceinline__ void lds_issue_val_mant(uint32_t m_addr, uint64_t& w01, uint64_t& w23) {
    asm volatile("ds_read2st64_b32 %0, %2 offset0:%3 offset1:%4\n\tds_read2st64_b32 %1, %2 offset0:%5 offset1:%6"
                 : "=&v"(w01), "=&v"(w23) : "v"(m_addr), "n"(4 * U), "n"(4 * U + 1), "n"(4 * U + 2), "n"(4 * U + 3) : "memory");
}
// 8-bit mantissas: the 8 bytes at m_addr + 512 * (4U + i), i = 0..3 (two per register quad)
template <int U>
__device__ __forceinline__ void lds_issue_val_mant8(uint32_t m_addr, u32x4& w01, u32x4& w23) {
    asm volatile("ds_read2st64_b64 %0, %2 offset0:%3 offset1:%4\n\tds_read2st64_b64 %1, %2 offset0:%5 offset1:%6"
                 : "=&v"(w01), "=&v"(w23) : "v"(m_addr), "n"(4 * U), "n"(4 * U + 1), "n"(4 * U + 2), "n"(4 * U + 3) : "memory");
}
__device__ __forceinline__ void lds_wait(u32x4& a) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a) : : "memory"); }
__device__ __forceinline__ void lds_wait(u32x4& a, u32x4& b) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b) : : "memory"); }
__device__ __forceinline__ void lds_wait(u32x4& a, u32x4& b, uint32_t (&e)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]) : : "memory");
}
template <int HG>
__device__ __forceinline__ void lds_wait(u32x4& w01, u32x4& w23, uint64_t (&pp)[HG]) {
    if constexpr (HG == 1) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w01), "+v"(w23), "+v"(pp[0]) : : "memory");
    else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w01), "+v"(w23), "+v"(pp[0]), "+v"(pp[1]) : : "memory");
}
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

// PAGED: the planes are a pool of pages and every 16-token stage of a 64-token tile looks up its page (scalar
// loads, issued a tile ahead of the requests that need them); a separate instantiation, so the contiguous case
// is untouched.
// QI8 (8-bit mantissas, blocks of 32 and wider, query cast to 8-bit BFP): the score product on the integer
// datapath of Sec. II-B -- v_mfma_i32_16x16x64_i8 on the signed codes of query and keys, one accumulator per 32
// channels, and the two block exponents added and applied to the integer sums afterwards.
template <int P, int N, int HG, bool PAGED, bool QI8 = false>
__device__ __forceinline__ void decode_split_lds_body(const DecodeArgs& a, const int dt) {
    static_assert(P == 4 || P == 8, "mantissa widths of the format");
    static_assert(!QI8 || (P == 8 && N >= 32), "integer score product: 8-bit codes, one key exponent per 32 channels");
    static_assert(P == 4 || HG <= 2, "8-bit mantissas: one or two groups of four heads");
    // value conversions produce value * 2^-kShift (the stored exponent byte is their scale operand); the
    // probabilities carry the inverse
    constexpr int kShift = P == 4 ? 7 : 3;
    constexpr int kRowB = kD * P / 8;              // bytes of a packed row
    constexpr int kStageB = 16 * kRowB;            // bytes of a 16-token stage: 1 KB / 2 KB
    constexpr int kM = kStageB / 1024;             // DMA instructions per stage (64 lanes x 16 bytes each)
    static_assert(N == 16 || N == 32 || N == 64 || N == 128, "block sizes of the format");
    static_assert(HG < 4 || N <= 32, "the sixteen-head variant is built for blocks of 16 and 32");
    constexpr int NB = kD / N;
    constexpr int NH = HG * 4;
    constexpr int kTileTok = 64;
    // per-wavefront staging area
    constexpr int kKm = 0;                         // 4 stages of key mantissas
    constexpr int kVm = kKm + 4 * kStageB;         // 4 stages of value mantissas
    // Exponents of a whole 64-token tile: [64 tokens][kExpRow bytes] in LDS.  Blocks of 16 / 32: the 8 / 4 bytes of a
    // token as they lie in the plane, fetched as dwords (two DMA instructions / one).  Blocks of 64 / 128: a token has
    // 2 / 1 bytes, the plane's rows are not dword-aligned, so each lane fetches its token's bytes with a 2- / 1-byte
    // DMA element, which lands zero-extended in the lane's own dword.
    constexpr int kExpRow = NB >= 4 ? NB : 4;
    constexpr int kExpElt = NB >= 4 ? 4 : NB;      // bytes per lane and DMA instruction
    constexpr int kEt = kTileTok * kExpRow;
    constexpr int kKe = kVm + 4 * kStageB;
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
    // sixteen heads: the query operand (4 x 8 registers) does not stay in registers between tiles; it lives in LDS,
    // [NH * 4 limb rows][128], and every tile reads it back for its score phase
    constexpr bool kQueryInLds = HG == 4 || (HG == 2 && PAGED && ((P == 4 && N == 32) || (P == 8 && N == 16)));   // (and where paging would push a three-wavefront variant over its registers)
    // One small LDS object either way: the limbs' scale bytes [NH * 4][4] of the set-up, or -- where the query
    // operand lives in LDS -- that operand; the scale bytes then sit at the end of the query staging area, whose
    // second half the limbs do not need in that case.
    __shared__ __align__(16) uint8_t qaux_lds[kQueryInLds ? NH * 4 * kD : NH * 16];
    uint8_t* const qop_lds = qaux_lds;
    uint8_t* const qsc_lds = kQueryInLds ? (uint8_t*)&p_lds[0][0] + sizeof(p_lds) - NH * 16 : qaux_lds;

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

    // The page numbers of a wavefront's tiles do not come from look-ups inside the main loop: a load there shares a
    // counter with the requests the loop keeps in flight and waits for one by one, and every wait then also waits for
    // the table (over 16-token pages the pass took 61.5 us with a look-up per tile and 54.7 us in an experiment
    // without any).  They are fetched in bulk by the 64 lanes (tile lane/4, stage lane%4, as quotients like q[u] below)
    // into a list of kPreTiles tiles in LDS, slot = tile index % kPreTiles: all of it at kernel start, and one half of
    // it, for the tiles 32..63 ahead, whenever the loop enters the other half.  (One variant's 80 KB of LDS leave no
    // room for the list: it looks its pages up tile by tile.)
    constexpr int kPreTiles = !PAGED || (P == 8 && HG == 2 && N == 16) ? 0 : 64;      // 4 KB of LDS per workgroup
    __shared__ __align__(16) int32_t pt_lds[kPreTiles > 0 ? kWaves * kPreTiles * 4 : 4];
    const int64_t tile_step = (int64_t)a.n_splits * kWaves * kTileTok;
    auto fetch_pages = [&](auto n_tag, const int first_tile) {    // tiles first_tile .. first_tile + n - 1, n = 32 or 64
        constexpr int n = decltype(n_tag)::value;
        int32_t got[n / 16];
#pragma unroll
        for (int pass = 0; pass < n / 16; ++pass) {               // all loads first, then the stores
            const int tile = first_tile + 16 * pass + (lane >> 2);
            int64_t t = t_begin + wave * kTileTok + (int64_t)tile * tile_step + 16 * (lane & 3);
            if (t >= t_end) t = (t_end - 1) & ~(int64_t)15;
            got[pass] = (int32_t)(kvbfp::cache_row(a, b, kvh, t) >> 4);
        }
#pragma unroll
        for (int pass = 0; pass < n / 16; ++pass) {
            const int tile = first_tile + 16 * pass + (lane >> 2);
            pt_lds[(wave * (kPreTiles > 0 ? kPreTiles : 1) + (tile & (kPreTiles > 0 ? kPreTiles - 1 : 0))) * 4 + (lane & 3)] = got[pass];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    if constexpr (kPreTiles > 0) fetch_pages(std::integral_constant<int, 64>{}, 0);

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
        kvbfp::cast::encode_store<P, N>(x, nr_sub, nr_live, const_cast<uint8_t*>(nr_which ? a.v_mant : a.k_mant),
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
    // Where the 64-token tile that starts at token T of the split lies in the planes.  One region per sequence,
    // and pages of 64 tokens or more (a tile has one page): r0 = first row of the tile relative to the bases below.
    // Pages of 16 or 32 tokens: one entry per 16-token stage, q[u] = (first plane row of stage u) / 16 -- a stage
    // starts at a multiple of 16 rows, and the quotient fits 32 bits.  A stage that starts beyond the last cached
    // token takes the entry of the stage that holds that token.
    const bool small_pages = PAGED && a.log2_page < 6;          // wave-uniform
    struct TileRows { int64_t r0; int32_t q[PAGED ? 4 : 1]; };
    // (ti: index of the tile in this wavefront's sequence of tiles)
    auto tile_rows = [&](const int T, const bool live, const int ti) -> TileRows {
        TileRows tr;
        tr.r0 = 0;
#pragma unroll
        for (int u = 0; u < (PAGED ? 4 : 1); ++u) tr.q[u] = 0;
        if constexpr (PAGED) {
            if (kPreTiles > 0 && live) {
                const int4 e = *(const int4*)&pt_lds[(wave * kPreTiles + (ti & (kPreTiles - 1))) * 4];
                tr.q[0] = __builtin_amdgcn_readfirstlane(e.x);
                tr.q[1] = __builtin_amdgcn_readfirstlane(e.y);
                tr.q[2] = __builtin_amdgcn_readfirstlane(e.z);
                tr.q[3] = __builtin_amdgcn_readfirstlane(e.w);
                tr.r0 = (int64_t)tr.q[0] << 4;
            } else if (live && !small_pages) {
                tr.r0 = kvbfp::cache_row(a, b, kvh, t_begin + T);
            } else if (live) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    int64_t t = t_begin + T + 16 * u;
                    if (t >= t_end) t = (t_end - 1) & ~(int64_t)15;
                    tr.q[u] = (int32_t)(kvbfp::cache_row(a, b, kvh, t) >> 4);
                }
            }
        } else {
            tr.r0 = live ? (int64_t)T : 0;
        }
        return tr;
    };
    const uint8_t* __restrict__ k_mant = a.k_mant + base * kRowB;
    const uint8_t* __restrict__ v_mant = a.v_mant + base * kRowB;
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
    // 8-bit mantissas: a row is eight 16-byte chunks, a stage takes two DMA instructions; lane L of instruction i
    // fills LDS slot L + 64 i = (row position L/8 + 8i, chunk slot L%8).  Keys: row = position, and the slot holds
    // chunk (L%8) ^ (row/2 % 8), which lets lane (j, kg) read the chunks kg and 4 + kg of row j without bank
    // conflicts.  Values: position q holds row 4 (q%4) + q/4, chunks in order.
    const int k8_row[2] = {lane >> 3, (lane >> 3) + 8};
    const int k8_chunk[2] = {(lane & 7) ^ ((k8_row[0] >> 1) & 7), (lane & 7) ^ ((k8_row[1] >> 1) & 7)};
    const int v8_row[2] = {4 * ((lane >> 3) & 3) + (lane >> 5), 4 * ((lane >> 3) & 3) + (lane >> 5) + 2};
    const uint32_t e_src = (uint32_t)lane * kExpElt;   // exponents: element `lane` (+64 per further instruction) of the tile's rows

    // Re-fills of the staging area.  Mantissas: stage u of a tile that starts at token t of the split = plane
    // row `row` (tile_row of the tile).  A full tile takes the immediate-offset form (the offset applies to the
    // global and to the LDS address alike, 1024 bytes per stage in both); in a ragged one rows past the last
    // cached token re-read that token.  `left` values are wave-uniform, so these are scalar branches.
    auto fill_mant = [&](auto U, const bool keys, const bool tile_full, const int t, const TileRows& rows) {
        constexpr int u = decltype(U)::value;
        uint8_t* const lm = wbase + (keys ? kKm : kVm);
        if (PAGED && small_pages) {
            // the stage's own page: first row of the stage, then (row of the stage, chunk) of this lane
            const uint8_t* __restrict__ sp = (keys ? k_mant : v_mant) + ((int64_t)rows.q[u] << 4) * kRowB;
            // rows of the stage past the last cached token re-read a cached row of the stage that holds that token
            const int last = (n_tok - (t + 16 * u) >= 16) ? 15 : ((n_tok - 1) & 15);
#pragma unroll
            for (int i = 0; i < kM; ++i) {
                int r, c;
                if constexpr (P == 8) {
                    r = keys ? k8_row[i] : v8_row[i];
                    c = keys ? k8_chunk[i] : (lane & 7);
                } else {
                    r = keys ? kd_row : vrow_of_slot;
                    c = keys ? kd_chunk : vp_c;
                }
                if (!tile_full) r = min(r, last);
                // (an unsigned 32-bit lane offset from a wave-uniform base: no 64-bit address arithmetic per lane)
                __builtin_amdgcn_global_load_lds(KVBFP_GPTR(sp + (uint32_t)(r * kRowB + c * 16)), KVBFP_LPTR(lm + u * kStageB + i * 1024), 16, 0, kStreamAux);
            }
            return;
        }
        const uint8_t* __restrict__ mp = (keys ? k_mant : v_mant) + rows.r0 * kRowB;
        if constexpr (P == 8) {
            const int left = n_tok - (t + 16 * u);       // may be <= 0: then every lane re-reads the last cached token
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                int r = keys ? k8_row[i] : v8_row[i];
                const int c = keys ? k8_chunk[i] : (lane & 7);
                if (!tile_full) r = min(r, left - 1);
                const int mo = (16 * u + r) * 128 + c * 16;
                __builtin_amdgcn_global_load_lds(KVBFP_GPTR(mp + mo), KVBFP_LPTR(lm + u * kStageB + i * 1024), 16, 0, kStreamAux);
            }
        } else if (tile_full) {
            __builtin_amdgcn_global_load_lds(KVBFP_GPTR(mp + (keys ? k_src : v_src)), KVBFP_LPTR(lm), 16, u * 1024, kStreamAux);
        } else {
            const int left = n_tok - (t + 16 * u);       // may be <= 0: then every lane re-reads the last cached token
            const int r = keys ? kd_row : vrow_of_slot, c = keys ? kd_chunk : vp_c;
            const int mo = (16 * u + min(r, left - 1)) * 64 + c * 16;
            __builtin_amdgcn_global_load_lds(KVBFP_GPTR(mp + mo), KVBFP_LPTR(lm + u * 1024), 16, 0, kStreamAux);
        }
    };
    // Exponents of a whole tile, [64 tokens][NB] as they lie in the plane.
    auto fill_exp = [&](const bool keys, const bool tile_full, const int t, const TileRows& rows) {
        uint8_t* const le = wbase + (keys ? kKe : kVe);
        if (PAGED && small_pages) {
            const uint8_t* __restrict__ pp = keys ? k_exp : v_exp;
            const int left = n_tok - t;                    // >= 1
#pragma unroll
            for (int x = 0; x < kExpDma; ++x) {
                const int byte = (int)e_src + 256 * x;      // offset in the tile's exponent rows: this lane's token and byte
                int tk = byte / NB;
                if (!tile_full) tk = min(tk, left - 1);
                const int st = tk >> 4;
                const int32_t lo = (st & 1) ? rows.q[1] : rows.q[0], hi = (st & 1) ? rows.q[3] : rows.q[2];
                const int64_t row = ((int64_t)((st & 2) ? hi : lo) << 4) + (tk & 15);
                const uint8_t* __restrict__ src = pp + (row * NB + byte % NB);
                if constexpr (NB >= 4) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(src), KVBFP_LPTR(le + 256 * x), 4, 0, kStreamAux);
                else if constexpr (NB == 2) __builtin_amdgcn_global_load_lds(KVBFP_GPTR(src), KVBFP_LPTR(le + 256 * x), 2, 0, kStreamAux);
                else __builtin_amdgcn_global_load_lds(KVBFP_GPTR(src), KVBFP_LPTR(le + 256 * x), 1, 0, kStreamAux);
            }
            return;
        }
        const uint8_t* __restrict__ ep = (keys ? k_exp : v_exp) + rows.r0 * NB;
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
        const TileRows row0 = tile_rows(T_first, true, 0);
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
    // 8-bit keys in blocks of 16: a 32-channel MX block of the key operand holds two blocks, so each product is
    // issued twice, once with the query's odd blocks of 16 zeroed and once with the even ones (a block of 16 of the
    // FP8 operand lies in one lane group: even blocks in even groups)
    v8i aq8e[(P == 8 && N == 16) ? HG : 1], aq8o[(P == 8 && N == 16) ? HG : 1];
    // QI8: the query's signed 8-bit codes, row 4*head (the other rows zero), channels 64m + 16kg ..+15 for the
    // MFMA m of a stage, once with the lane groups of the upper 32 channels zeroed and once with the lower ones;
    // qei = the power of two of each 32-channel group of this lane's head, minus the 6 of the keys' code scale
    v4i aqi[QI8 ? HG : 1][2][2];
    int qei[QI8 ? HG : 1][4];
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
        uint8_t* q8 = kQueryInLds ? qop_lds : (uint8_t*)(qr + NH * kD);   // [NH * 4 limb rows][kD positions], beside the fp32 values
        uint8_t* qsc = qsc_lds;
        const int kb = qchan >> 5;
        if constexpr (QI8) {
            // the cast query (cache order, unscaled) is code * 2^e per block; per 32 channels the codes are taken
            // relative to that group's own largest magnitude, which keeps them integers of at most 7 bits
            int* const qexp = (int*)qsc_lds;              // [NH][4]
            const int c = tid & (kD - 1);
#pragma unroll
            for (int k = 0; k < kQPerThread; ++k) {
                const int g = (tid + 256 * k) / kD;
                const float v = qr[g * kD + c];
                float mx = row_max(fabsf(v));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                int e = 0;
                if (mx > 0.f) (void)frexpf(mx, &e);        // mx = f * 2^e, f in [0.5, 1): codes below 2^7 at scale 2^(e - 7)
                e -= 7;
                q8[g * kD + c] = (uint8_t)(int8_t)(int)ldexpf(v, -e);
                if ((c & 31) == 0) qexp[g * 4 + (c >> 5)] = mx > 0.f ? e : 0;
            }
            lds_barrier();
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) {
                const bool carries = (j & 3) == 0;        // row 4*head: the codes; rows of the other limbs: zero
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const u32x4 cw = *(const u32x4*)(q8 + (hg * 4 + (j >> 2)) * kD + 64 * m + 16 * kg);
                    const v4i codes = carries ? v4i{(int)cw[0], (int)cw[1], (int)cw[2], (int)cw[3]} : v4i{0, 0, 0, 0};
                    aqi[hg][m][0] = kg < 2 ? codes : v4i{0, 0, 0, 0};
                    aqi[hg][m][1] = kg < 2 ? v4i{0, 0, 0, 0} : codes;
                }
#pragma unroll
                for (int grp = 0; grp < 4; ++grp) qei[hg][grp] = qexp[(hg * 4 + kg) * 4 + grp] - 6;
            }
            lds_barrier();                                // the buffer goes over to the probabilities
        } else {
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
            // 4-bit keys: - 1, the key operand below is magnitude / 2 at the block's own exponent byte;
            // 8-bit keys: + 3, the low piece reads as lo 2^-9 and stands for lo 2^-6 at the block's exponent byte
            sa8[hg] = qsc[(hg * 16 + j) * 4 + kg] + (P == 4 ? -1 : 3);
            if constexpr (P == 8 && N == 16) {
                const v8i zero = {0, 0, 0, 0, 0, 0, 0, 0};
                aq8e[hg] = (kg & 1) ? zero : aq8[hg];
                aq8o[hg] = (kg & 1) ? aq8[hg] : zero;
            }
        }
        lds_barrier();                                    // the buffer goes over to the probabilities
        }
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
    // (QI8: all exponent bytes of token j, the lane scales the sums of every 32-channel group itself)
    const uint32_t keq = lds_addr(wbase + kKe + j * kExpRow + (QI8 ? 0 : (N == 16 ? 2 * kg : (32 * kg) / N)));   // + 16 kExpRow per stage
    const uint32_t vq = lds_addr(wbase + kVm + kg * 64 + j * 4);                           // + i*256: row 4kg+i sits at position 4i+kg
    // 8-bit mantissas: chunks kg and 4 + kg of row j (slots swizzled with row/2 % 8); bytes 8j..8j+7 of position 4i + kg
    const int k8_slot = kg ^ ((j >> 1) & 7);
    const uint32_t kq8a = lds_addr(wbase + kKm + (8 * j + k8_slot) * 16);
    const uint32_t kq8b = lds_addr(wbase + kKm + (8 * j + (k8_slot ^ 4)) * 16);
    const uint32_t vq8 = lds_addr(wbase + kVm + kg * 128 + j * 8);
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
        u32x4 rawk8[kPipe ? 2 : 1][2], vw8a[kPipe ? 2 : 1], vw8b[kPipe ? 2 : 1];     // 8-bit mantissas
        uint32_t kexp[4];
        uint64_t vw01[kPipe ? 2 : 1], vw23[kPipe ? 2 : 1], ppv[kPipeP ? 2 : 1][HG];
        u32x4 vexp32[4];          // blocks of 32: per stage the exponent dwords of tokens 4kg..4kg+3
        uint32_t vexp16[16];      // blocks of 16: per (stage, token) this lane's exponent byte
        // sixteen heads: the sixteen exponent bytes this lane needs of a tile, packed into four registers right after
        // they arrive (blocks of 32: register i = token 4kg + i, byte u = stage; blocks of 16: register u, byte i)
        constexpr bool kPackVexp = HG == 4 || (HG == 2 && N == 32 && PAGED && P == 4);   // (and where paging would push a three-wavefront variant over its registers)
        uint32_t vexp_pk[4];
        const uint32_t pk_sel01 = (uint32_t)(j >> 2) | ((4u + (uint32_t)(j >> 2)) << 8) | 0x0c0c0000u;
        const uint32_t pk_sel23 = ((uint32_t)(j >> 2) << 16) | ((4u + (uint32_t)(j >> 2)) << 24) | 0x00000c0cu;
        // DMA completes in issue order; per tile that is K0, key exponents, K1..K3, V0, value exponents, V1..V3.
        // "The oldest stage still outstanding has landed" = at most (instructions issued after it) outstanding:
        // with kM instructions per stage, 7 kM + kExpDma after the first stage of a plane (it ends with the exponents),
        // 7 kM + 2 kExpDma after any other,
        // while the next tile is being requested; on the last tile only what is left of the tile itself.
        auto wait_dma = [&](const bool refilling, auto steady_tag, auto tail_tag) {
            __builtin_amdgcn_sched_barrier(0);
            if (refilling) __builtin_amdgcn_s_waitcnt(vmcnt_imm(decltype(steady_tag)::value));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(decltype(tail_tag)::value));
            __builtin_amdgcn_sched_barrier(0);
        };
        constexpr int kAfterFirst = 7 * kM + kExpDma, kAfterOther = 7 * kM + 2 * kExpDma;
        auto issue_k0 = [&] {
            if constexpr (P == 8) {
                lds_issue_b128<0>(kq8a, rawk8[0][0]);
                lds_issue_b128<0>(kq8b, rawk8[0][1]);
            } else {
                lds_issue_b128<0>(kq, rawk[0]);
            }
            if constexpr (QI8 && N == 32) lds_issue_4w<0, 16 * kExpRow>(keq, kexp);
            else lds_issue_4<0, 16 * kExpRow, N == 16 || (QI8 && N == 64)>(keq, kexp);
        };
        // wait for the DMA of a stage and issue its LDS reads (`more`: the next tile is being requested meanwhile)
        auto start_k = [&](auto U, const bool more) {             // key stage U >= 1
            constexpr int u = decltype(U)::value;
            wait_dma(more, std::integral_constant<int, kAfterOther>{}, std::integral_constant<int, (7 - u) * kM + kExpDma>{});
            if constexpr (P == 8) {
                lds_issue_b128<u * kStageB>(kq8a, rawk8[kPipe ? (u & 1) : 0][0]);
                lds_issue_b128<u * kStageB>(kq8b, rawk8[kPipe ? (u & 1) : 0][1]);
            } else {
                lds_issue_b128<u * 1024>(kq, rawk[kPipe ? (u & 1) : 0]);
            }
        };
        auto start_v0 = [&](const bool more) {                    // value stage 0 and the tile's value exponents
            wait_dma(more, std::integral_constant<int, kAfterFirst>{}, std::integral_constant<int, 3 * kM>{});
            if constexpr (P == 8) lds_issue_val_mant8<0>(vq8, vw8a[0], vw8b[0]);
            else lds_issue_val_mant<0>(vq, vw01[0], vw23[0]);
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
            wait_dma(more, std::integral_constant<int, kAfterOther>{}, std::integral_constant<int, (3 - u) * kM>{});
            if constexpr (P == 8) lds_issue_val_mant8<u>(vq8, vw8a[kPipe ? (u & 1) : 0], vw8b[kPipe ? (u & 1) : 0]);
            else lds_issue_val_mant<u>(vq, vw01[kPipe ? (u & 1) : 0], vw23[kPipe ? (u & 1) : 0]);
            if constexpr (kPipeP) issue_p(U, std::integral_constant<int, u & 1>{});
        };
        // One tile.  STEADY: this tile is complete and seen whole by every head, and a complete next tile is being
        // requested -- the common case, compiled without the ragged-tile branches, clamps and masks.
        auto tile_body = [&](auto steady_tag, const int T0, const int T1, const bool more_rt, const bool full1_rt,
                             const bool masked_rt, const TileRows& row1) {
            constexpr bool STEADY = decltype(steady_tag)::value;
            const bool more = STEADY ? true : more_rt;
            const bool full1 = STEADY ? true : full1_rt;
            const bool masked = STEADY ? false : masked_rt;
            const int left = n_tok - T0;
            // the first stage of a tile is read here and not ahead, at the end of the tile before: a register with a
            // read pending must not be live across the loop's back edge (the compiler may copy it there)
            wait_dma(true, std::integral_constant<int, kAfterFirst>{}, std::integral_constant<int, 0>{});
            issue_k0();
            if constexpr (kQueryInLds) {
                asm volatile("" ::: "memory");            // a fresh read every tile: the values must not stay live in between
#pragma unroll
                for (int hg = 0; hg < HG; ++hg) {
                    const u32x4 lo = *(const u32x4*)(qop_lds + (hg * 16 + j) * kD + kg * 32);
                    const u32x4 hi = *(const u32x4*)(qop_lds + (hg * 16 + j) * kD + kg * 32 + 16);
                    aq8[hg] = v8i{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
                    if constexpr (P == 8 && N == 16) {
                        const v8i zero = {0, 0, 0, 0, 0, 0, 0, 0};
                        aq8e[hg] = (kg & 1) ? zero : aq8[hg];
                        aq8o[hg] = (kg & 1) ? aq8[hg] : zero;
                    }
                }
            }

            // ---------------- scores
            f32x4 s_acc[HG][4];
            // sixteen heads: the four limb rows of a stage are added up while the next stage's products run, so that
            // one stage of accumulators is live at a time instead of four (64 registers less at the peak)
            constexpr bool kEarlySum = HG == 4;
            float s_sum[kEarlySum ? HG : 1][4];
            static_for<4>([&](auto U) {
                constexpr int u = decltype(U)::value;
                constexpr int cur = kPipe ? (u & 1) : 0;
                if constexpr (!kPipe && u > 0) start_k(U, more);
                if constexpr (P == 8) {
                    if (u == 0) lds_wait(rawk8[0][0], rawk8[0][1], kexp); else lds_wait(rawk8[cur][0], rawk8[cur][1]);
                } else {
                    if (u == 0) lds_wait(rawk[0], kexp); else lds_wait(rawk[cur]);
                }
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
                if constexpr (QI8) {
                    // integer datapath (Sec. II-B): signed codes x signed codes into i32, one accumulator per 32
                    // channels (the lane groups of the other 32 channels of a 64-wide product are zero in the query
                    // operand), then one exponent addition and one scaling per group
                    v4i kb2[2];
#pragma unroll
                    for (int m = 0; m < 2; ++m)
                        kb2[m] = v4i{twos_complement4(rawk8[cur][m][0]), twos_complement4(rawk8[cur][m][1]),
                                     twos_complement4(rawk8[cur][m][2]), twos_complement4(rawk8[cur][m][3])};
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg) {
                        float sc = 0.f;
#pragma unroll
                        for (int grp = 0; grp < 4; ++grp) {
                            const v4i sum = __builtin_amdgcn_mfma_i32_16x16x64_i8(aqi[hg][grp >> 1][grp & 1], kb2[grp >> 1],
                                                                                   v4i{0, 0, 0, 0}, 0, 0, 0);
                            const int Ek = (int)((kexp[u] >> (N == 32 ? 8 * grp : (N == 64 ? 8 * (grp >> 1) : 0))) & 0xFFu);
                            const int field = min(max(Ek + qei[hg][grp], 0), 254);     // key code scale 2^(Ek - 133), query 2^(qei + 6)
                            sc = fmaf((float)sum[0], __uint_as_float((uint32_t)field << 23), sc);
                        }
                        s_acc[hg][u] = f32x4{sc * a.scale_log2e, 0.f, 0.f, 0.f};
                    }
                } else if constexpr (P == 8) {
                    // the two FP8 pieces of every byte are the B operands as they are (no conversion): magnitude =
                    // 8 hi + lo, so the high piece takes the block's exponent byte + 3 as its E8M0 scale
                    v8i bh, bl;
#pragma unroll
                    for (int d = 0; d < 8; ++d) {
                        const uint32_t w = rawk8[cur][d >> 2][d & 3];
                        bh[d] = (int)(((w >> 3) & 0x0F0F0F0Fu) | (w & 0x80808080u));
                        bl[d] = (int)(w & 0x87878787u);
                    }
                    if (N >= 32) {
                        const int sb = (int)kexp[u];
#pragma unroll
                        for (int hg = 0; hg < HG; ++hg) {
                            s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], bh, s_acc[hg][u], 0, 0, 0, sa8[hg], 0, sb + 3);
                            s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], bl, s_acc[hg][u], 0, 0, 0, sa8[hg], 0, sb);
                        }
                    } else {
                        const int sb0 = (int)(kexp[u] & 0xFFu), sb1 = (int)(kexp[u] >> 8);
#pragma unroll
                        for (int hg = 0; hg < HG; ++hg) {
                            s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8e[hg], bh, s_acc[hg][u], 0, 0, 0, sa8[hg], 0, sb0 + 3);
                            s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8e[hg], bl, s_acc[hg][u], 0, 0, 0, sa8[hg], 0, sb0);
                            s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8o[hg], bh, s_acc[hg][u], 0, 0, 0, sa8[hg], 0, sb1 + 3);
                            s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8o[hg], bl, s_acc[hg][u], 0, 0, 0, sa8[hg], 0, sb1);
                        }
                    }
                } else
                // magnitude/2 = FP4(s,0,m1,m0) + FP4(s,m2,0,0): two masked copies of the raw nibbles are the B
                // operands and the block's exponent byte is their E8M0 scale (the halving sits in the query's scale).
                if (N >= 32) {                 // one exponent byte per 32 channels (the same byte for wider blocks)
                    const int sb = (int)kexp[u];
                    const v8i b1 = {(int)(raw[0] & 0xBBBBBBBBu), (int)(raw[1] & 0xBBBBBBBBu), (int)(raw[2] & 0xBBBBBBBBu),
                                    (int)(raw[3] & 0xBBBBBBBBu), 0, 0, 0, 0};
                    const v8i b2 = {(int)(raw[0] & 0xCCCCCCCCu), (int)(raw[1] & 0xCCCCCCCCu), (int)(raw[2] & 0xCCCCCCCCu),
                                    (int)(raw[3] & 0xCCCCCCCCu), 0, 0, 0, 0};
                    // (operand by operand over the head groups: one key operand is live at a time, and consecutive
                    // products go to different accumulators)
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], b1, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb);
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], b2, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb);
                } else {
                    // the lane's 32 nibbles are two blocks of 16 (dwords 0-1 and 2-3) with an exponent each
                    const int sb0 = (int)(kexp[u] & 0xFFu), sb1 = (int)(kexp[u] >> 8);
                    const v8i lo1 = {(int)(raw[0] & 0xBBBBBBBBu), (int)(raw[1] & 0xBBBBBBBBu), 0, 0, 0, 0, 0, 0};
                    const v8i lo2 = {(int)(raw[0] & 0xCCCCCCCCu), (int)(raw[1] & 0xCCCCCCCCu), 0, 0, 0, 0, 0, 0};
                    const v8i hi1 = {0, 0, (int)(raw[2] & 0xBBBBBBBBu), (int)(raw[3] & 0xBBBBBBBBu), 0, 0, 0, 0};
                    const v8i hi2 = {0, 0, (int)(raw[2] & 0xCCCCCCCCu), (int)(raw[3] & 0xCCCCCCCCu), 0, 0, 0, 0};
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], lo1, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb0);
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], lo2, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb0);
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], hi1, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb1);
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_acc[hg][u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(aq8[hg], hi2, s_acc[hg][u], 0, 4, 0, sa8[hg], 0, sb1);
                }
                if constexpr (kEarlySum && u > 0) {
#pragma unroll
                    for (int hg = 0; hg < HG; ++hg)
                        s_sum[hg][u - 1] = (s_acc[hg][u - 1][0] + s_acc[hg][u - 1][1]) + (s_acc[hg][u - 1][2] + s_acc[hg][u - 1][3]);
                }
            });
            if constexpr (kEarlySum) {
#pragma unroll
                for (int hg = 0; hg < HG; ++hg) s_sum[hg][3] = (s_acc[hg][3][0] + s_acc[hg][3][1]) + (s_acc[hg][3][2] + s_acc[hg][3][3]);
            }

            // ---------------- online softmax; lane (j, kg) owns head kg of each group, tokens 16u + j
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) {
                float s[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)      // the limb rows
                    s[u] = kEarlySum ? s_sum[kEarlySum ? hg : 0][u] : (s_acc[hg][u][0] + s_acc[hg][u][1]) + (s_acc[hg][u][2] + s_acc[hg][u][3]);
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
                if constexpr (P == 8) lds_wait<HG>(vw8a[cur], vw8b[cur], ppv[pc]);
                else lds_wait<HG>(vw01[cur], vw23[cur], ppv[pc]);
                if (u == 0) { if (N == 32) lds_wait(vexp32); else lds_wait(vexp16); }
                if constexpr (kPackVexp && u == 0) {
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        if (N == 32)
                            vexp_pk[x] = __builtin_amdgcn_perm(vexp32[1][x], vexp32[0][x], pk_sel01) |
                                         __builtin_amdgcn_perm(vexp32[3][x], vexp32[2][x], pk_sel23);
                        else
                            vexp_pk[x] = vexp16[4 * x] | (vexp16[4 * x + 1] << 8) | (vexp16[4 * x + 2] << 16) | (vexp16[4 * x + 3] << 24);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (more) {
                    fill_mant(U, false, full1, T1, row1);
                    if (u == 0) fill_exp(false, full1, T1, row1);
                }
                if constexpr (kPipe && u < 3) start_v(std::integral_constant<int, u + 1>{}, more);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (P == 8) {
                    // bytes 8j..8j+7 of the rows 4kg + i: two dwords per row; both pieces of every code enter the
                    // reduction next to the same probability
                    const uint32_t wx[4] = {vw8a[cur][0], vw8a[cur][2], vw8b[cur][0], vw8b[cur][2]};
                    const uint32_t wy[4] = {vw8a[cur][1], vw8a[cur][3], vw8b[cur][1], vw8b[cur][3]};
                    Pieces8 va[4], vb[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t sl = N == 32 ? __builtin_amdgcn_alignbit(vexp32[u][i], vexp32[u][i], ve_rot) : (vexp16[4 * u + i] << 23);
                        const float s_lo = __uint_as_float(sl), s_hi = __uint_as_float(sl + (3u << 23));
                        va[i] = unpack4_p8(wx[i], s_hi, s_lo);
                        vb[i] = unpack4_p8(wy[i], s_hi, s_lo);
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
                } else {
                const uint32_t vw[4] = {(uint32_t)vw01[cur], (uint32_t)(vw01[cur] >> 32), (uint32_t)vw23[cur], (uint32_t)(vw23[cur] >> 32)};
                Unpacked4 vv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // scale operand: the exponent byte in the exponent field (the conversion looks at nothing else:
                    // for blocks of 32 the other bytes of the dword stay where the rotation leaves them)
                    float sc;
                    if constexpr (kPackVexp) {
                        constexpr int reg = N == 32 ? 0 : u;            // + i for blocks of 32 (not a constant expression there)
                        const uint32_t pk = vexp_pk[N == 32 ? i : reg];
                        sc = __uint_as_float(__builtin_amdgcn_alignbit(pk, pk, (uint32_t)((8 * (N == 32 ? u : i) + 9) & 31)));
                    } else {
                        sc = N == 32 ? __uint_as_float(__builtin_amdgcn_alignbit(vexp32[u][i], vexp32[u][i], ve_rot))
                                     : scale_operand(vexp16[4 * u + i]);
                    }
                    vv[i] = unpack8_p4(vw[i], sc);
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
                }
            });
            // (the next tile writes its probabilities after its score phase; every read of this tile's has returned)
        };
        int ti = 0;
        for (int T0 = T_first; T0 < n_tok; T0 += kStep, ++ti) {
            const int T1 = T0 + kStep;
            const bool more = T1 < n_tok;            // wave-uniform
            if constexpr (kPreTiles > 0) {
                // entering a half of the page list: the other half takes the tiles 32..63 ahead (rare: its loads are
                // ordinary ones, waited for right here)
                if (ti > 0 && (ti & 31) == 0 && more) fetch_pages(std::integral_constant<int, 32>{}, ti + 32);
            }
            const TileRows row1 = tile_rows(T1, more, ti + 1);
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
            // 4-bit: MFMA m holds slots 2m, 2m + 1 of the dword; 8-bit: the channel pair (8j + 2m, 8j + 2m + 1)
            const int c_even = 8 * j + (P == 4 ? slot_channel(2 * m) : 2 * m);
            const int c_odd = 8 * j + (P == 4 ? slot_channel(2 * m + 1) : 2 * m + 1);
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


}  // namespace lds
}  // namespace kvbfp
