// Streaming kernel for both selectors of Sec. 3.2: the paper's online rule (Qerror
// summed over group-wise maxima; default 8 groups, all dialects, block 32) and
// the exhaustive squared-error search (group count 0 in the template), with
// the two-stage filter, SeDA candidate lists (Sec. 3.4) and the second plane
// of the activation decomposition (Sec. 3.3): in one pass with the first
// plane, or alone from a first plane already in memory.
//
// One lane owns 32 consecutive elements of a row -- one block of 32 or two
// blocks of 16: it loads the 64 bytes with four 16-byte loads, keeps the
// elements as 16 packed bf16 pairs and runs every per-element step on both
// halves of a register at once (packed 16-bit integer instructions).  Nothing
// crosses lanes (but the exhaustive selector's scores).  A wavefront therefore covers 64 consecutive 32-element
// chunks (4 KiB of input) and writes 1 KiB of codes and 128 (block 16: 256)
// bytes of metadata, all contiguous.  In the code below "chunk" indices (gb)
// count these 32-element pieces.
//
// LDS tables, built once per workgroup:
//   * Qerror rows (32 bytes per bin, one byte per dialect) in 16 copies laid
//     out so that lane l always reads banks 4*(l%16)..4*(l%16)+3: the 16-byte
//     row reads of a wavefront never collide whatever bins the lanes ask for;
//   * a pair table: (bin of element 2m, bin of element 2m+1, dialect) -> the
//     finished code byte without sign bits, so one lookup emits two elements;
//   * exhaustive selector (instead of the Qerror rows): the dialect matrices and
//     one histogram per block -- its scores are a matrix product, taken on the
//     matrix cores (select_sse_matrix).
//
// A block whose largest magnitude is NaN/Inf-sized or below 2^-122 (and not
// zero) leaves the packed path: the wavefront then redoes its tile with a
// plain per-element routine that covers every input.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fb4_tables.hpp"

namespace fb4 {

#ifndef FB4_FAST_THREADS
#define FB4_FAST_THREADS 512
#endif

constexpr int kFastThreads = FB4_FAST_THREADS;
constexpr int kFastWaves = kFastThreads / 64;

struct FastParams {
    const uint16_t* x;
    long long row_stride;   // elements
    uint32_t nb;            // 32-element chunks per row
    uint32_t n_blocks;      // rows * nb
    uint32_t n_tiles;       // ceil(n_blocks / 64)
    uint32_t div_mul;       // row = (gb * div_mul) >> div_shift   (gb < 2^31)
    uint32_t div_shift;
    uint8_t* codes;
    uint16_t* meta;
    const uint8_t* blob;
    const int32_t* token_group;   // SeDA: [rows] or null
    const uint8_t* sub;           // SeDA: [n_groups][8] DIDs
    uint32_t n_groups;            // SeDA: <= kMaxFastGroups
    uint32_t n_dialects;
    // fused second plane of the salient rows (Sec. 3.3)
    const int32_t* salient;       // [n_sal] ascending, unique
    uint32_t n_sal;
    uint32_t rows;                // <= kMaxFusedRows
    uint8_t* codes2;              // [n_sal][nb * 16]
    uint16_t* meta2;              // [n_sal][nb * 32 / block]
    // second plane only (mode 2): the first plane of the whole tensor; x is read at the rows `salient` lists and
    // codes / meta are the compact second plane
    const uint8_t* codes1;        // [rows][nb * 16]
    const uint16_t* meta1;        // [rows][nb * 32 / block]
};

constexpr uint32_t kMaxFastGroups = 1023;   // SeDA groups whose exclusion rows fit the workgroup's LDS

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_sub(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, a) - __builtin_bit_cast(u16x2, b));
}
// max(a - b, 0) in both halves
__device__ __forceinline__ uint32_t pk_sub_sat(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, a),
                                                                      __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_shl(uint32_t a, uint32_t n)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, a) << __builtin_bit_cast(u16x2, n));
}
__device__ __forceinline__ uint32_t pk_shr(uint32_t v, uint32_t s)   // per half: v >> s, s <= 15
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, v) >> __builtin_bit_cast(u16x2, s));
}
__device__ __forceinline__ uint32_t halves_max(uint32_t v) { return max(v & 0xFFFFu, v >> 16); }
__device__ __forceinline__ uint32_t halves_min(uint32_t v) { return min(v & 0xFFFFu, v >> 16); }
// a.lo*b.lo + a.hi*b.hi + c
__device__ __forceinline__ uint32_t dot2_u16(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_udot2(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b), c, false);
}
// A constant the optimizer cannot fold back into an instruction literal: keeps
// three-operand instructions encodable with the constant in a register.
__device__ __forceinline__ uint32_t sgpr_const(uint32_t v)
{
    uint32_t r;
    asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "i"(v));
    return r;
}
__device__ __forceinline__ uint32_t vgpr_const(uint32_t v)
{
    uint32_t r;
    asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "i"(v));
    return r;
}

// LDS layout of the fast kernel (bytes)
// Qerror rows in 16 bank-disjoint copies, piece (bin, half, copy) = 16 bytes of row `bin`: an LDS pass serves
// 16 lanes, and lane l reads copy l % 16, so a row read never conflicts whatever the lanes' bins (8 groups:
// 23.85 -> 23.6 us on the 16384x3072 workload against 8 copies, 16 groups 25.4 -> 24.6, 32 groups 36.1 -> 31.5).
constexpr int kRowCopies = 16;
constexpr int kLdsRows = 0;              // [32 bins][2 halves][16 copies][16 B]  16 KiB
constexpr int kLdsPair = 16384;          // [32 hi bins][32 lo bins][32 dialects] 32 KiB
constexpr int kLdsNibT = 16384 + 32768;  // [32 bins][32 dialects]                1 KiB
constexpr int kLdsRange = kLdsNibT + 1024;   // two-stage: [8 ranges][32 B] 0xFF = dialect excluded
// fused decomposition only: decode table, bitmap of salient rows, salient rows before each bitmap word
constexpr uint32_t kMaxFusedRows = 65536;
constexpr int kLdsDecode = kLdsRange + 256;              // [32 dialects][8] bf16 patterns      512 B
constexpr int kLdsMagNib = kLdsDecode + 512;             // [32 dialects] eight 4-bit magnitudes 128 B
constexpr int kLdsSalBits = kLdsMagNib + 128;            // one bit per row                     8 KiB
constexpr int kLdsSalRank = kLdsSalBits + kMaxFusedRows / 8;   // uint16 per bitmap word         4 KiB
constexpr int kLdsDecompBytes = 512 + 128 + kMaxFusedRows / 8 + kMaxFusedRows / 32 * 2;
// SeDA: [n_groups + 1][32 B] 0xFF = dialect excluded; last row: none.  Placed after everything else.
constexpr int lds_seda_offset(bool decomp) { return kLdsRange + 256 + (decomp ? kLdsDecompBytes : 0); }
// Exhaustive selector only (it runs on the matrix cores: select_sse_matrix), placed last:
//   * per bin the (gain, magnitude) byte pairs of the 32 dialects, 64 B: [32 bins][32 dialects][2] = 2 KiB (read by
//     the prologue and the plain routine);
//   * the lanes' pieces of the dialect matrices, [8 pieces][64 lanes][16 B] = 8 KiB;
//   * per wavefront the histograms of its 64 blocks, one per lane: dword (bin b, lane l) at (64 b + l) * 4 =
//     (elements of the lane's block in bin b) << 24 | 128 + (sum of their 7-bit fractions).  Bin-major, so that
//     the 64 lanes of an instruction always touch 64 different banks, whatever their bins (block-major rows: a
//     third of the LDS time went to bank conflicts of the additions).  The first two wavefronts' histograms lie
//     in the 16 KiB of the Qerror rows, which this selector does not use.
constexpr int kGmBytes = 32 * 4 * 16;
constexpr int kMatrixTableBytes = 8 * 64 * 16;
constexpr int kHistWaveBytes = 32 * 64 * 4;
constexpr int lds_gm_offset(bool seda, bool decomp)
{
    return lds_seda_offset(decomp) + (seda ? (int)(kMaxFastGroups + 1) * 32 : 0);
}
constexpr int lds_matrix_offset(bool seda, bool decomp) { return lds_gm_offset(seda, decomp) + kGmBytes; }
// LDS offset of wavefront w's histograms
__host__ __device__ constexpr int lds_hist_offset(bool seda, bool decomp, int w)
{
    return w < 2 ? kLdsRows + w * kHistWaveBytes
                 : lds_matrix_offset(seda, decomp) + kMatrixTableBytes + (w - 2) * kHistWaveBytes;
}
// Online selector with 32 groups (every element its own group): its score sum_elements Qerror[bin][d] is the block's
// bin counts times the Qerror matrix, taken on the matrix cores as well (select_lut32_matrix).  Placed last: per
// wavefront the counts of its 64 blocks, dword (bin b, lane l) at (64 b + l) * 4 (the Qerror rows stay: the plain
// routine reads them).
constexpr int lds_count_offset(bool seda, bool decomp, int w) { return lds_gm_offset(seda, decomp) + w * kHistWaveBytes; }
// sse_waves: wavefronts of a workgroup that runs the exhaustive selector, else 0; count_waves: the same for the
// online selector with 32 groups
constexpr int lds_fast_bytes(bool seda, bool decomp, int sse_waves = 0, int count_waves = 0)
{
    return sse_waves     ? lds_hist_offset(seda, decomp, sse_waves > 2 ? sse_waves : 2)
           : count_waves ? lds_count_offset(seda, decomp, count_waves)
                         : lds_gm_offset(seda, decomp);
}

struct BlockCodes {
    uint32_t code[4];
    uint32_t meta;
};

// Sec. 3.3 residual of one element: x - y, exact in fp32, rounded once to bf16 (nearest even), where y is
// the decoded first-plane value of the element.  An Inf / NaN element is its own residual.
//   xh: bf16 pattern of x; nib: its first-plane code; did, eoff: dialect and (exponent byte - 130) << 7 of
//   its block; dec: decode table [dialect][index] of bf16 magnitude patterns.
__device__ __forceinline__ uint32_t residual_elem(uint32_t xh, uint32_t nib, uint32_t did, uint32_t eoff,
                                                  const uint16_t* dec)
{
    const uint32_t mb = did < 32u ? (uint32_t)dec[did * 8 + (nib & 7u)] : 0u;
    uint32_t yb = mb ? ((mb + eoff) & 0x7FFFu) : 0u;
    yb |= (nib & 8u) << 12;
    const float d = __uint_as_float(xh << 16) - __uint_as_float(yb << 16);
    uint32_t u = __float_as_uint(d);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (((xh >> 7) & 0xFFu) == 0xFFu) ? xh : (u >> 16);
}

// Plain per-element routine for one block of kBlock elements with G groups, any input (Sec. 3.1-3.2); reads
// the block again from global memory.  Same arithmetic as the generic kernel.  Kept out of line on purpose:
// inlined, its global loads make the compiler wait for every outstanding load where the two paths join,
// which serializes the prefetch of the next tile (36 us instead of 25 us on the 16384x3072 workload).
// excl_a / excl_b: LDS offsets of 32-byte exclusion rows (0xFF = excluded), or 0xFFFFFFFF for none.  A dialect
// excluded by excl_a never wins; excl_b (the two-stage range filter) applies only if it leaves a candidate.
// kResidual: quantize the residual of the first plane (c1 = the block's first-plane code words, m1 = its
// metadata word) instead of x itself.
// G == 0: the exhaustive selector (gm_off: LDS offset of its (gain, magnitude) table).
template <int kBlock, int G, bool kResidual>
__device__ __noinline__ BlockCodes quantize_block_plain(const uint16_t* xb, const uint8_t* lds, uint32_t excl_a,
                                                        bool two_stage, uint4 c1, uint32_t m1, uint32_t gm_off)
{
    constexpr bool kSse = G == 0;
    constexpr int GG = kSse ? kBlock : G;   // the exhaustive selector looks at every element
    constexpr int PER = kBlock / GG;
    BlockCodes out;
    auto elem = [&](int i) -> uint32_t {
        const uint32_t h = xb[i];
        if (!kResidual) return h;
        const uint32_t cw = i < 8 ? c1.x : i < 16 ? c1.y : i < 24 ? c1.z : c1.w;
        return residual_elem(h, (cw >> (4 * (i & 7))) & 0xFu, m1 & 0xFFu, ((m1 >> 8) - 130u) << 7,
                             reinterpret_cast<const uint16_t*>(lds + kLdsDecode));
    };
    uint32_t amax = 0;
#pragma unroll 1
    for (int i = 0; i < kBlock; ++i) {
        uint32_t m = elem(i) & 0x7FFFu;
        amax = max(amax, (m > 0x7F80u) ? 0u : m);
    }
    const uint32_t eb = min(max(amax >> 7, 4u), 254u);
    // X = 256 * xhat (exact whenever xhat >= 0.5)
    auto x256_of = [&](uint32_t h) -> uint32_t {
        uint32_t m = h & 0x7FFFu;
        if (m > 0x7F80u) m = 0;
        uint32_t ef = m >> 7;
        uint32_t sig = (m & 0x7Fu) | (ef ? 0x80u : 0u);
        uint32_t sh = eb + 3u - max(ef, 1u);
        return (sh <= 7u) ? (sig << (7u - sh)) : (sig >> min(sh - 7u, 31u));
    };
    auto bin_of = [&](uint32_t h) -> uint32_t { return min(x256_of(h) >> 7, 31u); };
    uint32_t gbin[GG];
#pragma unroll
    for (int j = 0; j < GG; ++j) {
        uint32_t g = 0;
#pragma unroll 1
        for (int i = 0; i < PER; ++i) g = max(g, bin_of(elem(PER * j + i)));
        gbin[j] = g;
    }
    uint32_t bmax = 0;
#pragma unroll
    for (int j = 0; j < GG; ++j) bmax = max(bmax, gbin[j]);
    const uint32_t excl_b = kLdsRange + (min(max(bmax >> 1, 8u), 15u) - 8u) * 32u;
    uint32_t best = 0xFFFFFFFFu, best_b = 0xFFFFFFFFu;
#pragma unroll 1
    for (uint32_t d = 0; d < 32; ++d) {
        if (excl_a != 0xFFFFFFFFu && lds[excl_a + d]) continue;
        uint32_t s = 0;
        if (kSse) {
            // Z_d = sum of 128 * gain + frac * magnitude: the largest Z is the smallest squared error
            uint32_t z = 0;
#pragma unroll 1
            for (int i = 0; i < kBlock; ++i) {
                const uint32_t X = x256_of(elem(i));
                const uint32_t b = min(X >> 7, 31u), f = X - (b << 7);
                const uint8_t* e = lds + gm_off + b * 64u + d * 2u;
                z += ((uint32_t)e[0] << 7) + (uint32_t)e[1] * f;
            }
            s = 0xFFFFFu - z;
        } else {
#pragma unroll
            for (int j = 0; j < GG; ++j) s += lds[kLdsRows + gbin[j] * (32 * kRowCopies) + (d >> 4) * (16 * kRowCopies) + (d & 15)];
        }
        best = min(best, (s << 5) | d);
        if (two_stage && !lds[excl_b + d]) best_b = min(best_b, (s << 5) | d);
    }
    if (best_b != 0xFFFFFFFFu) best = best_b;
    const uint32_t did = best & 31u;
    out.code[0] = out.code[1] = out.code[2] = out.code[3] = 0;
#pragma unroll 1
    for (int c = 0; c < kBlock / 8; ++c) {
        uint32_t v = 0;
#pragma unroll 1
        for (int i = 0; i < 8; ++i) {
            uint32_t h = elem(8 * c + i);
            uint32_t nib = lds[kLdsNibT + bin_of(h) * 32 + did] | ((h >> 15) << 3);
            v |= nib << (4 * i);
        }
        out.code[c] = v;
    }
    out.meta = did | (eb << 8);
    return out;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

// Exhaustive selector on the matrix cores: what a lane keeps for the whole launch (make_matrix_consts).
struct MatrixConsts {
    uint32_t wtab;        // LDS offset of this lane's pieces of the two dialect matrices: piece (c, which) at
                          // wtab + (2 c + which) * 1024, 16 bytes (kept in LDS, not in 32 registers: the kernel
                          // then fits three wavefronts per SIMD)
    uint32_t row;         // LDS offset of the histogram row of this lane's own block
    uint32_t rd[2];       // LDS offsets of the 64 bytes it reads of block 32 t + lane % 32, t = 0, 1
    uint32_t half4;       // 4 * (lane / 32)
    i32x4 w3;             // candidate restrictions: byte j = 64 where 16 (lane / 32) + j == lane % 32, else 0
    i32x4 wq[4];          // online selector with 32 groups: this lane's pieces of the (negated) Qerror matrix
};

struct TileConsts {
    uint32_t k7f, k80, kpair, row_base;
    uint32_t kdid[16];   // DID pairs of the 16 key registers: (4i, 4i+2) and (4i+1, 4i+3)
    uint32_t gm_off;     // exhaustive selector: LDS offset of its table
    MatrixConsts mx;     // only set by a kernel that runs the exhaustive selector on the matrix cores
};

__device__ __forceinline__ TileConsts make_tile_consts(uint32_t lane, uint32_t gm_off)
{
    TileConsts K;
    K.gm_off = gm_off;
    K.row_base = kLdsRows + (lane & (kRowCopies - 1u)) * 16u;
    K.k7f = sgpr_const(0x007F007Fu);
    K.k80 = vgpr_const(0x00800080u);
    K.kpair = sgpr_const(32u | (1024u << 16));   // lo bin * 32 + hi bin * 1024
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        K.kdid[2 * i] = sgpr_const((4u * i) | ((4u * i + 2u) << 16));
        K.kdid[2 * i + 1] = sgpr_const((4u * i + 1u) | ((4u * i + 3u) << 16));
    }
    return K;
}

// Sec. 3.2 online selection for one block from the bins of its R group maxima: sum the Qerror rows, drop the
// excluded candidates, argmin with the lowest DID on ties.  Rows hold one byte per dialect; eight of them
// (8 x 31 = 248) still fit the byte, so rows are summed eight at a time and widened to 16 bits in between.
// excl_a: LDS offset of this block's SeDA exclusion row (kSeda only).
template <int R, bool kTwoStage, bool kSeda>
__device__ __forceinline__ uint32_t select_lut_rows(const uint32_t (&gbin)[R], const uint8_t* lds,
                                                    const TileConsts& K, uint32_t excl_a)
{
    static_assert(R % 8 == 0, "rows are summed eight at a time");
    uint32_t ev[8], od[8];   // 16-bit sums of dialects (4i, 4i+2) and (4i+1, 4i+3); R == 8 keeps bytes in ev
    // ---- candidate restrictions (Sec. 3.4 SeDA, Sec. 3.2 two-stage) as rows of bytes, 0xFF = excluded.  Their
    // reads go out together with the first batch of Qerror rows.
    uint4 xa0 = make_uint4(0, 0, 0, 0), xa1 = xa0, xr0 = xa0, xr1 = xa0;
    if (kSeda) {
        xa0 = *reinterpret_cast<const uint4*>(lds + excl_a);
        xa1 = *reinterpret_cast<const uint4*>(lds + excl_a + 16);
    }
    if (kTwoStage) {
        // first stage: keep the dialects whose top magnitude is the integer part of the block maximum
        uint32_t binmax = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) binmax = max(binmax, gbin[r]);
        const uint32_t roff = kLdsRange + (min(max(binmax >> 1, 8u), 15u) - 8u) * 32u;
        xr0 = *reinterpret_cast<const uint4*>(lds + roff);
        xr1 = *reinterpret_cast<const uint4*>(lds + roff + 16);
    }
#pragma unroll
    for (int c = 0; c < R / 8; ++c) {
        uint32_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        // all row reads are issued before the first sum: with two wavefronts per SIMD their latency shows
        uint4 r0[8], r1[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint8_t* row = lds + K.row_base + gbin[8 * c + j] * (32u * kRowCopies);
            r0[j] = *reinterpret_cast<const uint4*>(row);
            r1[j] = *reinterpret_cast<const uint4*>(row + 16 * kRowCopies);
        }
        asm volatile("" ::: "memory");
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            acc[0] += r0[j].x; acc[1] += r0[j].y; acc[2] += r0[j].z; acc[3] += r0[j].w;
            acc[4] += r1[j].x; acc[5] += r1[j].y; acc[6] += r1[j].z; acc[7] += r1[j].w;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (R == 8) {
                ev[i] = acc[i];
            } else {
                const uint32_t e = acc[i] & 0x00FF00FFu;
                const uint32_t o = __builtin_amdgcn_perm(0u, acc[i], 0x0C030C01u);
                ev[i] = c ? ev[i] + e : e;
                od[i] = c ? od[i] + o : o;
            }
        }
    }
    uint32_t ea[8] = {xa0.x, xa0.y, xa0.z, xa0.w, xa1.x, xa1.y, xa1.z, xa1.w};
    if (kTwoStage) {
        const uint32_t eb2[8] = {ea[0] | xr0.x, ea[1] | xr0.y, ea[2] | xr0.z, ea[3] | xr0.w,
                                 ea[4] | xr1.x, ea[5] | xr1.y, ea[6] | xr1.z, ea[7] | xr1.w};
        // ... unless that leaves nothing (possible only together with a SeDA list)
        const bool none = kSeda && ((eb2[0] & eb2[1] & eb2[2] & eb2[3] & eb2[4] & eb2[5] & eb2[6] & eb2[7]) == 0xFFFFFFFFu);
#pragma unroll
        for (int i = 0; i < 8; ++i) ea[i] = none ? ea[i] : eb2[i];
    }
    // ---- argmin with lowest DID on ties: 16-bit keys (sum << 5 | DID), 32 of them in 16 registers.  An
    // excluded dialect gets a key no real sum reaches.
    uint32_t best = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t e, o;
        if (R == 8) {
            const uint32_t a = (kSeda || kTwoStage) ? (ev[i] | ea[i]) : ev[i];   // 0xFF > 248 >= any real sum
            e = a & 0x00FF00FFu;                                  // dialects 4i, 4i+2
            o = __builtin_amdgcn_perm(0u, a, 0x0C030C01u);        // dialects 4i+1, 4i+3
        } else {
            e = ev[i];
            o = od[i];
        }
        uint32_t ke = (e << 5) | K.kdid[2 * i];
        uint32_t ko = (o << 5) | K.kdid[2 * i + 1];
        if (R != 8 && (kSeda || kTwoStage)) {
            const uint32_t xe = ea[i] & 0x00FF00FFu;
            const uint32_t xo = __builtin_amdgcn_perm(0u, ea[i], 0x0C030C01u);
            ke |= xe | (xe << 8);                                 // 0xFFFF > (992 << 5 | 31)
            ko |= xo | (xo << 8);
        }
        best = pk_min(best, pk_min(ke, ko));
    }
    return halves_min(best) & 31u;
}

// Exhaustive selection (Sec. 3.2, first paragraph) for the blocks of a wavefront, whose elements sit in registers
// b2[first .. first + RB) (bins, two per register) and x2 (256 * xhat, two per register).  With X = 256 * xhat =
// 128 * bin + frac and m the nearest magnitude of a dialect, (X - 256 m)^2 = X^2 - 512 Z with
// Z = 128 * m * (bin - m) + frac * m: the smallest error is the largest Z_d = sum over the elements of
// 128 * gain[bin][d] + frac * mag[bin][d] (< 2^20, every quantity an exact integer).
// As a matrix product: Z_d depends on a block only through, per bin b, the number
// of its elements in the bin, n_b, and the sum of their fractions, F_b: Z_d = sum_b 128 n_b gain[b][d] +
// F_b mag[b][d] -- a [blocks x 64] by [64 x 32 dialects] product of small integers, which the matrix cores do
// exactly (8-bit operands, 32-bit sums) in 16 instructions per 64 blocks where the vector ALU needs 1024.
//   * Histogram: every lane adds its block's elements into its own LDS column, one ds_add_u32 per element:
//     dword (bin, lane) += 1 << 24 | frac.  Dwords start at 0x80.
//   * Operands: a matrix instruction takes 32 blocks; lane l reads the dwords of bins 16 h .. 16 h + 15
//     (h = l / 32) of block l % 32, puts 0x80 back and flips bit 7 of what it read.  The four bytes of a dword
//     are then: the low byte of F_b as a SIGNED number s_b; (F_b + 128) >> 8 = h_b, so that F_b = 256 h_b + s_b;
//     zero; n_b -- all within the signed 8-bit range (n_b <= 32, h_b <= 16), and they go into the instruction as
//     they lie: the reduction index of a piece of 16 bytes is (bin, byte), the same in both operands.
//   * Dialect matrices (make_matrix_consts), for the same (bin, byte) positions: w1 = (mag, 0, 0, 0) gives
//     P3 = sum s_b mag; w2 = (0, 2 mag, 0, gain - 120) gives P12 = sum 2 h_b mag + n_b (gain - 120), and
//     Z_d = 128 P12 + P3 + 128 * 120 * (elements of the block); the last term is the same for all dialects and
//     is left out (gain <= 240 would not fit a signed byte), so keys are signed.
//   * The product is taken as dialects x blocks, so a lane ends up with 16 dialects of ONE block (dialect
//     8 (i / 4) + 4 h + i % 4 in accumulator i): keys Z * 32 + 31 - DID, the largest wins, the two half-wavefronts
//     meet through a lane swap, and lane l < 32 holds the choice for block l of the first 32 blocks,
//     lane l >= 32 that for block l of the second 32: every lane ends up with its own block's dialect.
// The LDS unit works a wavefront's instructions off in order, so the reads see the additions without any wait in
// between.  Call from all 64 lanes (full EXEC).
//   * Candidate restrictions (two-stage range filter, SeDA lists): the exclusion rows in LDS hold a byte per
//     dialect, 0xFF = -1 where excluded.  The lane that owns a block knows where its rows are (range_row, seda_row:
//     LDS offsets); a lane swap hands them to the two lanes that hold the block's dialects, which read their 16
//     bytes and send them through one more matrix instruction each, against a matrix with 64 (SeDA) or 16 (range)
//     on the diagonal: the result, -64 or -16 or their sum for an excluded dialect, is added to the key shifted
//     up by 23 bits -- a SeDA-excluded dialect loses to every other one, a range-excluded one to every one that is
//     not, and if the range excludes all candidates the best of them still wins, which is the rule
//     ("unless it leaves no candidate").  |key| < 2^25 before that.
template <int RB, bool kTwoStage, bool kSeda>
__device__ __forceinline__ uint32_t select_sse_matrix(const uint32_t (&b2)[16], const uint32_t (&x2)[16], int first,
                                                      uint8_t* lds, const MatrixConsts& M, uint32_t lane,
                                                      uint32_t range_row, uint32_t seda_row)
{
    const uint32_t k_lo = sgpr_const(256u), k_hi = sgpr_const(256u << 16);   // 256 * bin from either half
    const uint32_t one_lo = sgpr_const(1u), one_hi = sgpr_const(1u << 16);   // the fraction of either half
    const uint32_t k_cnt = vgpr_const(0x01000000u);
#pragma unroll
    for (int k = first; k < first + RB; ++k) {
        const uint32_t f2 = x2[k] & 0x007F007Fu;
        uint32_t* a0 = reinterpret_cast<uint32_t*>(lds + dot2_u16(b2[k], k_lo, M.row));
        uint32_t* a1 = reinterpret_cast<uint32_t*>(lds + dot2_u16(b2[k], k_hi, M.row));
        __hip_atomic_fetch_add(a0, dot2_u16(f2, one_lo, k_cnt), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        __hip_atomic_fetch_add(a1, dot2_u16(f2, one_hi, k_cnt), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t r[2][16];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        uint32_t* col = reinterpret_cast<uint32_t*>(lds + M.rd[t]);
#pragma unroll
        for (int j = 0; j < 16; ++j) r[t][j] = col[64 * j];
#pragma unroll
        for (int j = 0; j < 16; ++j) col[64 * j] = 0x80u;
    }
    // exclusion rows of the blocks this lane works for: element t of a swapped pair is the owner's value for
    // group t (lane % 32 of the first 32 lanes, of the second 32)
    i32x4 xr[2], xa[2];
    if (kTwoStage) {
        const auto sw = __builtin_amdgcn_permlane32_swap(range_row, range_row, false, false);
#pragma unroll
        for (int t = 0; t < 2; ++t) xr[t] = *reinterpret_cast<const i32x4*>(lds + sw[t] + 4u * M.half4);
    }
    if (kSeda) {
        const auto sw = __builtin_amdgcn_permlane32_swap(seda_row, seda_row, false, false);
#pragma unroll
        for (int t = 0; t < 2; ++t) xa[t] = *reinterpret_cast<const i32x4*>(lds + sw[t] + 4u * M.half4);
    }
    int res[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        i32x16 p12 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        i32x16 p3 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        i32x16 pen = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        if (kSeda) pen = __builtin_amdgcn_mfma_i32_32x32x32_i8(M.w3, xa[t], pen, 0, 0, 0);
        if (kTwoStage) {
            const i32x4 w3r = {M.w3.x >> 2, M.w3.y >> 2, M.w3.z >> 2, M.w3.w >> 2};   // 16 on the diagonal
            pen = __builtin_amdgcn_mfma_i32_32x32x32_i8(w3r, xr[t], pen, 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const i32x4 b = {(int)(r[t][4 * c] ^ 0x80u), (int)(r[t][4 * c + 1] ^ 0x80u), (int)(r[t][4 * c + 2] ^ 0x80u),
                             (int)(r[t][4 * c + 3] ^ 0x80u)};
            const i32x4 w1 = *reinterpret_cast<const i32x4*>(lds + M.wtab + (2 * c) * 1024);
            const i32x4 w2 = *reinterpret_cast<const i32x4*>(lds + M.wtab + (2 * c + 1) * 1024);
            p3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, b, p3, 0, 0, 0);
            p12 = __builtin_amdgcn_mfma_i32_32x32x32_i8(w2, b, p12, 0, 0, 0);
        }
        int best = (int)0x80000000;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            // (the tie-break constant sits in a scalar register the optimizer cannot see through: shift-and-or,
            // then shift-and-add, two instructions per key instead of three)
            const uint32_t low = ((uint32_t)p3[i] << 5) | sgpr_const((uint32_t)(31 - 8 * (i >> 2) - (i & 3)));
            uint32_t key = ((uint32_t)p12[i] << 12) + low;
            if (kSeda || kTwoStage) key += (uint32_t)pen[i] << 23;
            best = max(best, (int)key);
        }
        best -= (int)M.half4;   // this half's dialects are 4 * (lane / 32) further up
        // (the other half-wavefront's best through a lane swap in the vector ALU: no LDS round trip)
        const auto sw = __builtin_amdgcn_permlane32_swap((uint32_t)best, (uint32_t)best, false, false);
        res[t] = max((int)sw[0], (int)sw[1]);
    }
    return 31u - ((uint32_t)(lane < 32u ? res[0] : res[1]) & 31u);
}

// The lane's pieces of the dialect matrices (written to lds + matrix_off), from the (gain, magnitude) table at
// lds + gm_off (which must be complete), and its places in the wavefront's histograms at lds + hist_off, which it
// initializes.
__device__ __forceinline__ MatrixConsts make_matrix_consts(uint8_t* lds, uint32_t gm_off, uint32_t matrix_off,
                                                           uint32_t hist_off, uint32_t lane)
{
    MatrixConsts M;
    const uint32_t d = lane & 31u, h = lane >> 5;
    M.wtab = matrix_off + lane * 16u;
    const uint32_t base = hist_off;
    M.row = base + lane * 4u;
    M.rd[0] = base + d * 4u + h * (16u * 256u);
    M.rd[1] = M.rd[0] + 32u * 4u;
    M.half4 = 4u * h;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        uint32_t a[4], b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t bin = 16u * h + 4u * c + j;
            const uint32_t gm = *reinterpret_cast<const uint16_t*>(lds + gm_off + bin * 64u + d * 2u);   // gain | mag << 8
            const uint32_t mag = gm >> 8, gain = gm & 0xFFu;
            a[j] = mag;
            b[j] = (mag << 9) | (((gain - 120u) & 0xFFu) << 24);
        }
        // (every wavefront writes the same values: no barrier needed before its own reads)
        *reinterpret_cast<uint4*>(lds + M.wtab + (2 * c) * 1024) = make_uint4(a[0], a[1], a[2], a[3]);
        *reinterpret_cast<uint4*>(lds + M.wtab + (2 * c + 1) * 1024) = make_uint4(b[0], b[1], b[2], b[3]);
    }
    {
        const uint32_t j = d - 16u * h;   // the byte of this lane's own dialect, if it lies in this half
        const uint32_t v = 64u << (8u * (j & 3u));
        M.w3 = i32x4{(int)((j >> 2) == 0u ? v : 0u), (int)((j >> 2) == 1u ? v : 0u), (int)((j >> 2) == 2u ? v : 0u),
                     (int)((j >> 2) == 3u ? v : 0u)};
    }
#pragma unroll
    for (int b = 0; b < 32; ++b) reinterpret_cast<uint32_t*>(lds + M.row)[64 * b] = 0x80u;
    return M;
}

// Sec. 3.2 online selection with 32 groups: every element is its own group, so the score of dialect d is
// sum_elements Qerror[bin][d] = sum_b n_b Qerror[b][d] with n_b the block's elements in bin b -- the same matrix
// product as the exhaustive selector's, with counts alone (32 row reads of 32 bytes per block otherwise, the LDS
// pipe's bound: 30.7 us on 16384x3072).  A lane adds 1 to dword (bin, lane) per element; the lanes that hold a
// block's dialects read its 32 dwords (byte 0 = n_b <= 32, the other bytes zero), put zero back, and four matrix
// instructions against (-Qerror, 0, 0, 0) give minus the score: keys -S * 32 + 31 - DID, the largest wins (smallest
// score, lowest DID on ties); candidate restrictions as in select_sse_matrix.  Block size 32, full EXEC.
template <bool kTwoStage, bool kSeda>
__device__ __forceinline__ uint32_t select_lut32_matrix(const uint32_t (&b2)[16], uint8_t* lds, const MatrixConsts& M,
                                                        uint32_t lane, uint32_t range_row, uint32_t seda_row)
{
    const uint32_t k_lo = sgpr_const(256u), k_hi = sgpr_const(256u << 16);   // 256 * bin from either half
    const uint32_t one = vgpr_const(1u);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        uint32_t* a0 = reinterpret_cast<uint32_t*>(lds + dot2_u16(b2[k], k_lo, M.row));
        uint32_t* a1 = reinterpret_cast<uint32_t*>(lds + dot2_u16(b2[k], k_hi, M.row));
        __hip_atomic_fetch_add(a0, one, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        __hip_atomic_fetch_add(a1, one, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t r[2][16];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        uint32_t* col = reinterpret_cast<uint32_t*>(lds + M.rd[t]);
#pragma unroll
        for (int j = 0; j < 16; ++j) r[t][j] = col[64 * j];
#pragma unroll
        for (int j = 0; j < 16; ++j) col[64 * j] = 0u;
    }
    i32x4 xr[2], xa[2];
    if (kTwoStage) {
        const auto sw = __builtin_amdgcn_permlane32_swap(range_row, range_row, false, false);
#pragma unroll
        for (int t = 0; t < 2; ++t) xr[t] = *reinterpret_cast<const i32x4*>(lds + sw[t] + 4u * M.half4);
    }
    if (kSeda) {
        const auto sw = __builtin_amdgcn_permlane32_swap(seda_row, seda_row, false, false);
#pragma unroll
        for (int t = 0; t < 2; ++t) xa[t] = *reinterpret_cast<const i32x4*>(lds + sw[t] + 4u * M.half4);
    }
    int res[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        i32x16 ps = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        i32x16 pen = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        if (kSeda) pen = __builtin_amdgcn_mfma_i32_32x32x32_i8(M.w3, xa[t], pen, 0, 0, 0);
        if (kTwoStage) {
            const i32x4 w3r = {M.w3.x >> 2, M.w3.y >> 2, M.w3.z >> 2, M.w3.w >> 2};   // 16 on the diagonal
            pen = __builtin_amdgcn_mfma_i32_32x32x32_i8(w3r, xr[t], pen, 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const i32x4 b = {(int)r[t][4 * c], (int)r[t][4 * c + 1], (int)r[t][4 * c + 2], (int)r[t][4 * c + 3]};
            ps = __builtin_amdgcn_mfma_i32_32x32x32_i8(M.wq[c], b, ps, 0, 0, 0);
        }
        int best = (int)0x80000000;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            uint32_t key = ((uint32_t)ps[i] << 5) | sgpr_const((uint32_t)(31 - 8 * (i >> 2) - (i & 3)));
            if (kSeda || kTwoStage) key += (uint32_t)pen[i] << 23;
            best = max(best, (int)key);
        }
        best -= (int)M.half4;
        const auto sw = __builtin_amdgcn_permlane32_swap((uint32_t)best, (uint32_t)best, false, false);
        res[t] = max((int)sw[0], (int)sw[1]);
    }
    return 31u - ((uint32_t)(lane < 32u ? res[0] : res[1]) & 31u);
}

// What select_lut32_matrix keeps per lane: the pieces of the negated Qerror matrix, from the Qerror rows at
// lds + kLdsRows (copy 0; they must be complete), and its places in the wavefront's counts at lds + count_off,
// which it clears.
__device__ __forceinline__ MatrixConsts make_count_consts(uint8_t* lds, uint32_t count_off, uint32_t lane)
{
    MatrixConsts M;
    const uint32_t d = lane & 31u, h = lane >> 5;
    M.wtab = 0;
    M.row = count_off + lane * 4u;
    M.rd[0] = count_off + d * 4u + h * (16u * 256u);
    M.rd[1] = M.rd[0] + 32u * 4u;
    M.half4 = 4u * h;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        uint32_t a[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t bin = 16u * h + 4u * c + j;
            const uint32_t q = lds[kLdsRows + bin * (32 * kRowCopies) + (d >> 4) * (16 * kRowCopies) + (d & 15u)];
            a[j] = (0u - q) & 0xFFu;
        }
        M.wq[c] = i32x4{(int)a[0], (int)a[1], (int)a[2], (int)a[3]};
    }
    {
        const uint32_t j = d - 16u * h;
        const uint32_t v = 64u << (8u * (j & 3u));
        M.w3 = i32x4{(int)((j >> 2) == 0u ? v : 0u), (int)((j >> 2) == 1u ? v : 0u), (int)((j >> 2) == 2u ? v : 0u),
                     (int)((j >> 2) == 3u ? v : 0u)};
    }
#pragma unroll
    for (int b = 0; b < 32; ++b) reinterpret_cast<uint32_t*>(lds + M.row)[64 * b] = 0u;
    return M;
}

// One lane owns 32 consecutive elements of a row: w = its 32 bf16 as 16 packed pairs, holding one block of
// 32 or two blocks of 16.  Produces the four code words and the metadata (one 16-bit word, or two for block
// size 16 with the first block in the low half).  xb / in_range are only used by the plain per-element
// routine of a tile with special values (tile_special reports that this route was taken).  kResidual: w holds the Sec. 3.3 residual of the first plane
// (code1, meta1), which the plain routine recomputes from x.  stage: 16 words of the lane's private memory when w
// is not in global memory at all (xb is then ignored).
// kCounts: the calling kernel has the LDS counts that select_lut32_matrix needs (32 groups only).
template <int kBlock, int G, bool kTwoStage, bool kSeda, bool kResidual = false, bool kCounts = false>
__device__ __forceinline__ void compute_tile(const uint32_t (&w)[16], const uint8_t* lds, const TileConsts& K,
                                             const uint16_t* xb, bool in_range, uint32_t excl_a,
                                             uint32_t (&code)[4], uint32_t& meta,
                                             const uint32_t (&code1)[4], uint32_t meta1, bool& tile_special,
                                             uint32_t* stage = nullptr)
{
    constexpr int NB = 32 / kBlock;     // blocks per lane
    constexpr int RB = 16 / NB;         // packed registers per block
    constexpr bool kSse = G == 0;       // exhaustive selector: every element, no groups
    constexpr int GG = kSse ? kBlock : G;
    constexpr int PER = kBlock / GG;    // elements per group
    static_assert((kBlock == 32 || kBlock == 16) && (PER == 4 || PER == 2 || PER == 1), "supported shapes");
    // ---- magnitudes and maxima (bf16 bit patterns order like the values)
    uint32_t a[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) a[k] = w[k] & 0x7FFF7FFFu;
    uint32_t gm[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) gm[j] = pk_max(a[2 * j], a[2 * j + 1]);
    uint32_t bm[NB];
    if (NB == 1) {
        bm[0] = halves_max(pk_max(pk_max(pk_max(gm[0], gm[1]), pk_max(gm[2], gm[3])),
                                  pk_max(pk_max(gm[4], gm[5]), pk_max(gm[6], gm[7]))));
    } else {
        bm[0] = halves_max(pk_max(pk_max(gm[0], gm[1]), pk_max(gm[2], gm[3])));
        bm[NB - 1] = halves_max(pk_max(pk_max(gm[4], gm[5]), pk_max(gm[6], gm[7])));
    }
    bool special = false;
#pragma unroll
    for (int b = 0; b < NB; ++b) special = special || !(bm[b] == 0u || (bm[b] - 0x0280u) < (0x7F80u - 0x0280u));

    tile_special = __builtin_amdgcn_ballot_w64(special) != 0;   // wave-uniform
    if (tile_special) {
        // rare: some block of this tile holds NaN / Inf or is tiny
        code[0] = code[1] = code[2] = code[3] = 0;
        meta = 0;
        if (stage) {
            // the elements exist in registers only (a fused producer made them): the plain routine gets them
            // through this lane's private memory, NaNs as the canonical quiet NaN.  (The zero below is opaque to
            // the optimizer: without it the 160 instructions of this loop are hoisted out of the rare branch
            // and run for every tile.)
            uint32_t zero;
            asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                uint32_t v = w[k] | zero;
                if ((v & 0x7FFFu) > 0x7F80u) v = (v & 0xFFFF0000u) | 0x7FC0u;
                if ((v & 0x7FFF0000u) > 0x7F800000u) v = (v & 0xFFFFu) | 0x7FC00000u;
                stage[k] = v;
            }
            xb = reinterpret_cast<const uint16_t*>(stage);
        }
        if (in_range) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint4 c1 = NB == 1 ? make_uint4(code1[0], code1[1], code1[2], code1[3])
                                         : make_uint4(code1[2 * b], code1[2 * b + 1], 0u, 0u);
                const BlockCodes r = quantize_block_plain<kBlock, G, kResidual>(
                    xb + b * kBlock, lds, kSeda ? excl_a : 0xFFFFFFFFu, kTwoStage, c1, (meta1 >> (16 * b)) & 0xFFFFu,
                    K.gm_off);
#pragma unroll
                for (int c = 0; c < 4 / NB; ++c) code[b * (4 / NB) + c] = r.code[c];
                meta |= r.meta << (16 * b);
            }
        }
    } else {
        uint32_t b2[16];
        uint32_t x2[16];   // exhaustive selector: 256 * xhat
        uint32_t did[NB];
        meta = 0;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            // ---- shared exponent (Sec. 3.1) and bins (Sec. 3.2), two elements per instruction
            const uint32_t ebm = bm[b] >> 7;
            const uint32_t eb = max(ebm, 4u);                       // stored exponent byte
            const uint32_t ec = (max(ebm, 5u) + 3u) * 0x00010001u;  // shift base in both halves
#pragma unroll
            for (int k = b * RB; k < (b + 1) * RB; ++k) {
                const uint32_t ef = pk_shr(a[k], 0x00070007u);                 // exponent fields
                const uint32_t sh = pk_min(pk_sub(ec, ef), 0x000F000Fu);       // >= 3; >= 8 means bin 0
                const uint32_t sig = (a[k] & K.k7f) | K.k80;                   // 1.m as 8-bit integers
                b2[k] = pk_shr(sig, sh);                                       // floor(2*xhat), 0..31
                // 256 * xhat = sig << (7 - sh); an element with sh > 7 is in bin 0 and its value is not used
                if (kSse) x2[k] = pk_shl(sig, pk_sub_sat(0x00070007u, sh));
            }
            if (kSse) {
                // the block's range row: its largest element has bin 16 + (top three mantissa bits), range = bin / 2
                // (an all-zero block: range row 0, as from its bins)
                const uint32_t range_row = kLdsRange + ((bm[b] >> 4) & 7u) * 32u;
                did[b] = select_sse_matrix<RB, kTwoStage, kSeda>(b2, x2, b * RB, const_cast<uint8_t*>(lds), K.mx,
                                                                 threadIdx.x & 63u, range_row, excl_a);
            } else if (kCounts && G == 32) {
                const uint32_t range_row = kLdsRange + ((bm[b] >> 4) & 7u) * 32u;
                did[b] = select_lut32_matrix<kTwoStage, kSeda>(b2, const_cast<uint8_t*>(lds), K.mx, threadIdx.x & 63u,
                                                               range_row, excl_a);
            } else {
                // ---- group-wise maxima: groups are runs of PER elements
                uint32_t gbin[GG];
#pragma unroll
                for (int r = 0; r < GG; ++r) {
                    if (PER == 4) gbin[r] = halves_max(pk_max(b2[b * RB + 2 * r], b2[b * RB + 2 * r + 1]));
                    else if (PER == 2) gbin[r] = halves_max(b2[b * RB + r]);
                    else gbin[r] = (r & 1) ? (b2[b * RB + r / 2] >> 16) : (b2[b * RB + r / 2] & 0xFFFFu);
                }
                did[b] = select_lut_rows<GG, kTwoStage, kSeda>(gbin, lds, K, excl_a);
            }
            meta |= (did[b] | (eb << 8)) << (16 * b);
        }
        // ---- emit: every element through Qvalue of the chosen dialect, two elements per pair-table lookup
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t pbase = kLdsPair + did[c / (4 / NB)];
            uint32_t byte[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) byte[m] = lds[dot2_u16(b2[4 * c + m], K.kpair, pbase)];
            uint32_t v = byte[0] | (byte[1] << 8) | (byte[2] << 16) | (byte[3] << 24);
            // sign bits: element 2m -> bit 8m+3, element 2m+1 -> bit 8m+7
            const uint32_t x01 = __builtin_amdgcn_perm(w[4 * c + 1], w[4 * c + 0], 0x07030501u);  // b1(w0) b1(w1) b3(w0) b3(w1)
            const uint32_t x23 = __builtin_amdgcn_perm(w[4 * c + 3], w[4 * c + 2], 0x07030501u);
            const uint32_t lo = __builtin_amdgcn_perm(x23, x01, 0x05040100u);   // b1 of w0..w3
            const uint32_t hi = __builtin_amdgcn_perm(x23, x01, 0x07060302u);   // b3 of w0..w3
            v |= ((lo >> 4) & 0x08080808u) | (hi & 0x80808080u);
            code[c] = v;
        }
    }
}

// Address of block gb's first element, in elements from p.x.
template <bool kFlat>
__device__ __forceinline__ long long block_offset(const FastParams& p, uint32_t gb)
{
    if (kFlat) return (long long)gb * 32;
    const uint32_t row = (uint32_t)(((unsigned long long)gb * p.div_mul) >> p.div_shift);
    return (long long)row * p.row_stride + (long long)(gb - row * p.nb) * 32;
}

struct Block64 {   // one block: 32 bf16 = four 16-byte loads, plus its row's SeDA group
    uint4 q0, q1, q2, q3;
    int32_t grp;
    // second plane only: the block's first-plane code words and metadata, and its source row (-1: none)
    uint4 c1;
    uint32_t m1;
    int32_t row;
};

// Requests block gb.  There is no branch: a lane past the end reads the last block (its result is never
// stored, and data that a valid lane holds too cannot send the tile down another route), so that the loads
// sit in straight-line code and the waits that follow can be counted exactly.
// kGather: gb counts the blocks of the compact second plane; `row` is the tensor row of gb's list entry (a
// row outside the tensor reads row 0 and is marked).
template <int kBlock, bool kFlat, bool kSeda, bool kGather>
__device__ __forceinline__ Block64 load_block(const FastParams& p, uint32_t gb, int32_t row = 0)
{
    Block64 b;
    const uint32_t gbc = min(gb, p.n_blocks - 1u);
    b.grp = -1;
    b.c1 = make_uint4(0, 0, 0, 0);
    b.m1 = 0;
    b.row = 0;
    if (kGather) {
        const uint32_t pos = (uint32_t)(((unsigned long long)gbc * p.div_mul) >> p.div_shift);
        const uint32_t j = gbc - pos * p.nb;
        const bool ok = (uint32_t)row < p.rows;
        const size_t rowc = ok ? (size_t)row : 0;
        b.row = ok ? row : -1;
        const uint4* px = reinterpret_cast<const uint4*>(p.x + (long long)rowc * p.row_stride + (long long)j * 32);
        b.q0 = px[0]; b.q1 = px[1]; b.q2 = px[2]; b.q3 = px[3];
        const size_t blk = rowc * p.nb + j;
        b.c1 = *reinterpret_cast<const uint4*>(p.codes1 + blk * 16);
        b.m1 = kBlock == 16 ? reinterpret_cast<const uint32_t*>(p.meta1)[blk] : (uint32_t)p.meta1[blk];
        if (kSeda) b.grp = p.token_group[rowc];
        return b;
    }
    const uint4* px = reinterpret_cast<const uint4*>(p.x + block_offset<kFlat>(p, gbc));
    b.q0 = px[0]; b.q1 = px[1]; b.q2 = px[2]; b.q3 = px[3];
    if (kSeda) b.grp = p.token_group[(uint32_t)(((unsigned long long)gbc * p.div_mul) >> p.div_shift)];
    return b;
}

// Second plane only: the tensor row that block gb of the compact plane belongs to.
__device__ __forceinline__ int32_t load_row(const FastParams& p, uint32_t gb)
{
    const uint32_t gbc = min(gb, p.n_blocks - 1u);
    return p.salient[(uint32_t)(((unsigned long long)gbc * p.div_mul) >> p.div_shift)];
}

// Writes one tile's results: 16 bytes of codes per lane and the metadata words.  When the whole tile is in
// range and the metadata array is 16-byte aligned, eight neighbouring lanes gather their 16-bit metadata
// into one 16-byte store (sub-dword stores are slow to coalesce); block size 16 has one dword per lane.
// lane_ok = false: this lane writes nothing (second plane only: its list entry names no row of the tensor).
template <int kBlock>
__device__ __forceinline__ void store_tile(const FastParams& p, uint32_t gb, uint32_t lane, const uint4& code,
                                           uint32_t meta, bool meta_aligned, bool lane_ok = true)
{
    const uint32_t tile_first = gb - lane;   // wave-uniform
    if (meta_aligned && tile_first + 64u <= p.n_blocks && __builtin_amdgcn_ballot_w64(!lane_ok) == 0) {
        // results are written once and not read again by this kernel: streaming (non-temporal) stores
        typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
        const u32x4s cv = {code.x, code.y, code.z, code.w};
        __builtin_nontemporal_store(cv, reinterpret_cast<u32x4s*>(p.codes + (size_t)gb * 16));
        if (kBlock == 16) {
            __builtin_nontemporal_store(meta, reinterpret_cast<uint32_t*>(p.meta) + gb);
        } else {
            const uint32_t m = meta & 0xFFFFu;
            const uint32_t m1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x101, 0xF, 0xF, true);    // lane i <- i+1
            const uint32_t p2 = m | (m1 << 16);
            const uint32_t q2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)p2, 0x102, 0xF, 0xF, true);   // lane i <- i+2
            const uint32_t r0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)p2, 0x104, 0xF, 0xF, true);   // lane i <- i+4
            const uint32_t r1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)q2, 0x104, 0xF, 0xF, true);
            const u32x4s mv = {p2, q2, r0, r1};
            if ((lane & 7u) == 0u) __builtin_nontemporal_store(mv, reinterpret_cast<u32x4s*>(p.meta + gb));
        }
    } else if (gb < p.n_blocks && lane_ok) {
        *reinterpret_cast<uint4*>(p.codes + (size_t)gb * 16) = code;
        if (kBlock == 16) reinterpret_cast<uint32_t*>(p.meta)[gb] = meta;   // the launcher checks 4-byte alignment
        else p.meta[gb] = (uint16_t)meta;
    }
}

// Sec. 3.3 residual of one lane's 32 elements against its first plane (code, meta): x - y in fp32 (exact),
// then one rounding to bf16.  y = copysign(magnitude * 2^(e-3), x): the code carries x's sign.  The eight
// 4-bit magnitudes of the block's dialect sit in one register; an Inf / NaN element (only possible when
// may_have_naninf) is its own residual.
template <int kBlock>
__device__ __forceinline__ void residual32(const uint32_t (&w)[16], const uint32_t (&code)[4], uint32_t meta,
                                           const uint8_t* lds, bool may_have_naninf, uint32_t (&r)[16])
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    constexpr int NB = 32 / kBlock;
    uint32_t mags[NB];
    float scale[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const uint32_t mw = (meta >> (16 * b)) & 0xFFFFu;
        const uint32_t did = mw & 0xFFu;
        mags[b] = did < 32u ? reinterpret_cast<const uint32_t*>(lds + kLdsMagNib)[did] : 0u;
        scale[b] = __uint_as_float(((mw >> 8) - 3u) << 23);          // 2^(e-3); exponent byte >= 4
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int b = k / (16 / NB);
        const uint32_t cw = code[k >> 2];
        const int j = 2 * (k & 3);                                   // nibble of the low half
        const uint32_t s0 = j ? ((cw >> (4 * j - 2)) & 0x1Cu) : ((cw << 2) & 0x1Cu);   // 4 * index
        const uint32_t s1 = (cw >> (4 * j + 2)) & 0x1Cu;
        const float m0 = (float)((mags[b] >> s0) & 0xFu), m1 = (float)((mags[b] >> s1) & 0xFu);
        const float x0 = __uint_as_float(w[k] << 16), x1 = __uint_as_float(w[k] & 0xFFFF0000u);
        const f32x2 d = {x0 - __builtin_copysignf(m0 * scale[b], x0), x1 - __builtin_copysignf(m1 * scale[b], x1)};
        uint32_t out = __builtin_bit_cast(uint32_t, __builtin_convertvector(d, bf16x2));   // round to nearest even
        if (may_have_naninf) {
            if (((w[k] >> 7) & 0xFFu) == 0xFFu) out = (out & 0xFFFF0000u) | (w[k] & 0xFFFFu);
            if (((w[k] >> 23) & 0xFFu) == 0xFFu) out = (out & 0xFFFFu) | (w[k] & 0xFFFF0000u);
        }
        r[k] = out;
    }
}

// Sec. 3.4 exclusion rows for kernels that fuse a producer in front of the quantizer: row g of
// lds[offset ..] holds 0xFF for every dialect that group g may not use, the extra row n_groups (rows outside
// any group) and a group without a valid DID exclude nothing.  Call from all threads, then synchronize.
__device__ __forceinline__ void build_seda_rows(uint8_t* lds, int offset, const uint8_t* sub, uint32_t n_groups,
                                                uint32_t n_dialects, uint32_t n_threads)
{
    for (uint32_t g = threadIdx.x; g <= n_groups; g += n_threads) {
        uint32_t keep = 0;
        if (g < n_groups) {
            const uint2 s8 = *reinterpret_cast<const uint2*>(sub + (size_t)g * 8);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t d = ((k < 4 ? s8.x : s8.y) >> (8 * (k & 3))) & 0xFFu;
                if (d < n_dialects) keep |= 1u << d;
            }
        }
        uint32_t* row = reinterpret_cast<uint32_t*>(lds + offset + g * 32);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t k4 = (keep >> (4 * i)) & 0xFu;
            const uint32_t ex = ((k4 & 1u) ? 0u : 0x000000FFu) | ((k4 & 2u) ? 0u : 0x0000FF00u) |
                                ((k4 & 4u) ? 0u : 0x00FF0000u) | ((k4 & 8u) ? 0u : 0xFF000000u);
            row[i] = keep ? ex : 0u;
        }
    }
}
constexpr uint32_t kMaxFusedProducerGroups = 255;   // SeDA groups the producer-fused kernels hold in LDS

// The leading scalar arguments repeat the fields of `p` that the first loads and the loop bound depend on:
// the library is compiled so that the leading argument registers (14 of them on this target: all of these)
// are filled by the dispatcher when the wavefront starts (the rest of the arguments come by a load, half a microsecond later), and the table and
// tile requests can then go out at once.
// kMode: 0 = the first plane, 1 = both planes in one pass (rows listed in p.salient get a second plane),
// 2 = the second plane only, of the rows p.salient lists, from x and a first plane already in memory.
template <int kBlock, int G, bool kFlat, bool kTwoStage, bool kSeda, int kMode = 0, int kThreads = kFastThreads>
__global__ __launch_bounds__(kThreads) void quantize_lut_kernel(
    const uint8_t* blob, const uint16_t* x, uint32_t n_blocks, uint32_t n_tiles, uint32_t div_mul, uint32_t div_shift,
    uint32_t nb, uint32_t n_workgroups, long long row_stride, const int32_t* salient, FastParams p)
{
    p.blob = blob; p.x = x; p.n_blocks = n_blocks; p.n_tiles = n_tiles; p.div_mul = div_mul; p.div_shift = div_shift;
    p.nb = nb; p.row_stride = row_stride; p.salient = salient;
    constexpr int kWaves = kThreads / 64;
    constexpr bool kDecomp = kMode == 1, kGather = kMode == 2;
    constexpr bool kRes = kMode != 0;   // residuals are formed: decode tables needed
    static_assert(!(kGather && kFlat), "gathered rows are addressed through their row stride");
    constexpr int kLdsSeda = lds_seda_offset(kRes);
    constexpr bool kSse = G == 0;   // the exhaustive selector
    constexpr int kLdsGm = lds_gm_offset(kSeda, kRes);
    constexpr bool kCounts = G == 32 && kBlock == 32 && !kRes;   // 32 groups: scores on the matrix cores
    __shared__ __align__(16) uint8_t lds[lds_fast_bytes(kSeda, kRes, kSse ? kThreads / 64 : 0, kCounts ? kThreads / 64 : 0)];
    __shared__ uint32_t sal_before;      // fused decomposition: list entries below row 0
    __shared__ uint32_t sal_wave[kWaves];
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Tiles of workgroup b are b, b + W, b + 2W, ... (W = number of workgroups).  The waves of a workgroup
    // take them from a shared counter as they become free, so a wave that runs ahead of its neighbours
    // keeps working instead of idling at the end.
    __shared__ uint32_t wg_next;
    const uint32_t W = n_workgroups;   // = gridDim.x, which would have to be loaded
    Block64 cur;
    uint32_t t = blockIdx.x + wave * W;                      // first tile: static
    uint32_t t_next = blockIdx.x + (kWaves + wave) * W;   // second tile: static
    if (threadIdx.x == 0) wg_next = 2 * kWaves;
    // Loads are answered in the order they were issued.  The (small, mostly cached) table and list loads
    // therefore go out first and the first tile's right behind them: the tables are then built while the
    // tile is still on its way, instead of after it.
    constexpr int kCopies = kRowCopies;
    constexpr int kRowIt = (64 * kCopies + kThreads - 1) / kThreads;
    constexpr int kNibIt = (256 + kThreads - 1) / kThreads;
    constexpr int kSalEarly = 8;
    static_assert(kRowIt <= 2, "two row pieces per thread at most");
    uint4 row_a = make_uint4(0, 0, 0, 0), row_b = make_uint4(0, 0, 0, 0);   // (scalars, not an array: an array here ends up in scratch memory)
    uint32_t nibv[kNibIt], rngv = 0, decv = 0;
    uint4 magq = make_uint4(0, 0, 0, 0);
    uint2 sub0 = make_uint2(0, 0);
    uint4 gmm[4], gmg[4];
    int32_t sal_reg[kSalEarly];
    const bool sal_early = kDecomp && p.n_sal <= (uint32_t)kSalEarly * kThreads;
    {
        // Qerror rows in their bank-disjoint copies: piece i = (bin, half, copy) is 16 bytes of row `bin`
        // (indices are clamped, not predicated: a thread past the end loads a piece it does not write)
        auto row_piece = [&](int k) {
            const int i = min((int)threadIdx.x + k * kThreads, 64 * kCopies - 1);
            const int bin = i / (2 * kCopies), half = (i / kCopies) & 1;
            return *reinterpret_cast<const uint4*>(p.blob + kOffQerror8 + bin * 32 + half * 16);
        };
        if (!kSse) {   // (the exhaustive selector does not use them: their LDS holds two wavefronts' histograms)
            row_a = row_piece(0);
            if (kRowIt > 1) row_b = row_piece(1);
        }
#pragma unroll
        for (int k = 0; k < kNibIt; ++k)
            nibv[k] = reinterpret_cast<const uint32_t*>(p.blob + kOffQvalueT)[min((int)threadIdx.x + k * kThreads, 255)];
        if (kTwoStage) rngv = reinterpret_cast<const uint32_t*>(p.blob + kOffRangeExcl)[threadIdx.x & 63u];
        if (kRes) {
            decv = reinterpret_cast<const uint32_t*>(p.blob + kOffDecode)[threadIdx.x & 127u];
            magq = *reinterpret_cast<const uint4*>(p.blob + kOffDecode + (threadIdx.x & 31u) * 16);
        }
        if (kDecomp) {
            // a short salient list is requested now and used after the pair table; a long one is read in a
            // loop later
            if (sal_early) {
#pragma unroll
                for (int k = 0; k < kSalEarly; ++k) {
                    const uint32_t i = threadIdx.x + k * kThreads;
                    sal_reg[k] = i < p.n_sal ? p.salient[i] : 0x7FFFFFFF;   // beyond any row: ignored
                }
            }
        }
        if (kSeda && p.n_groups > 0)
            sub0 = *reinterpret_cast<const uint2*>(p.sub + (size_t)min(threadIdx.x, p.n_groups - 1u) * 8);
        if (kSse) {
            // thread `bin` of the first 32: the bin's 32 magnitudes and 32 gains (16 bits each in the table blob)
            const int bin = threadIdx.x & 31u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                gmm[q] = *reinterpret_cast<const uint4*>(p.blob + kOffMag16 + bin * 64 + q * 16);
                gmg[q] = *reinterpret_cast<const uint4*>(p.blob + kOffGain16 + bin * 64 + q * 16);
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    int32_t row_next = 0;   // second plane only: source row of this lane's block in the tile after `cur`
    if (kGather) {
        const int32_t row0 = load_row(p, t * 64u + lane);
        row_next = load_row(p, t_next * 64u + lane);
        cur = load_block<kBlock, kFlat, kSeda, kGather>(p, t * 64u + lane, row0);
    } else {
        // The first tiles of all wavefronts of the chip at once are a burst of 8 MB that queues up in the memory
        // system, and everybody's first tile arrives late.  Only the first two wavefronts of a workgroup ask at
        // once; the others ask 768 cycles (about a third of a microsecond) later, which is still before the
        // tables are built: the early tiles arrive earlier and the memory pipeline is as busy as before
        // (16384x3072: 23.4-23.7 -> 23.0-23.2 us; 8 to 16 sleep units give the same, 30 and more lose again,
        // and a delay that grows with the wavefront number, or only one early wavefront, gains less).
        if (kMode == 0 && !kSse && wave >= 2) __builtin_amdgcn_s_sleep(12);
        cur = load_block<kBlock, kFlat, kSeda, kGather>(p, t * 64u + lane);
    }
    __builtin_amdgcn_sched_barrier(0);
    {
        if (!kSse) {
            if ((int)threadIdx.x < 64 * kCopies) reinterpret_cast<uint4*>(lds + kLdsRows)[threadIdx.x] = row_a;
            if (kRowIt > 1 && (int)threadIdx.x + kThreads < 64 * kCopies)
                reinterpret_cast<uint4*>(lds + kLdsRows)[threadIdx.x + kThreads] = row_b;
        }
#pragma unroll
        for (int k = 0; k < kNibIt; ++k) {
            const int i = threadIdx.x + k * kThreads;
            if (i < 256) reinterpret_cast<uint32_t*>(lds + kLdsNibT)[i] = nibv[k];
        }
        if (kTwoStage && threadIdx.x < 64) reinterpret_cast<uint32_t*>(lds + kLdsRange)[threadIdx.x] = rngv;
        if (kSse && threadIdx.x < 32) {
            const int bin = threadIdx.x;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // piece q: dialects 8q .. 8q+7; a source dword holds two dialects' 16-bit values
                const uint32_t m[4] = {gmm[q].x, gmm[q].y, gmm[q].z, gmm[q].w};
                const uint32_t g[4] = {gmg[q].x, gmg[q].y, gmg[q].z, gmg[q].w};
                uint32_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)   // bytes: gain, mag of dialect 8q+2j, then of 8q+2j+1
                    o[j] = (g[j] & 0xFFu) | ((m[j] & 0xFFu) << 8) | ((g[j] >> 16) << 16) | ((m[j] >> 16) << 24);
                *reinterpret_cast<uint4*>(lds + kLdsGm + bin * 64 + q * 16) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
        if (kRes) {
            if (threadIdx.x < 128) reinterpret_cast<uint32_t*>(lds + kLdsDecode)[threadIdx.x] = decv;
            if (threadIdx.x < 32) {
                // the dialect's eight magnitudes (integers 0..15 stored as bf16 patterns) as nibbles
                const uint32_t dv[4] = {magq.x, magq.y, magq.z, magq.w};
                uint32_t mw = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t bits = (dv[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                    mw |= ((uint32_t)(int)__uint_as_float(bits << 16) & 0xFu) << (4 * i);
                }
                reinterpret_cast<uint32_t*>(lds + kLdsMagNib)[threadIdx.x] = mw;
            }
        }
        if (kDecomp) {
            for (uint32_t i = threadIdx.x; i < kMaxFusedRows / 32; i += kThreads)
                reinterpret_cast<uint32_t*>(lds + kLdsSalBits)[i] = 0;
            if (threadIdx.x == 0) sal_before = 0;
        }
        if (kSeda) {
            // one exclusion row per group: everything excluded except the group's valid DIDs; a group without
            // a valid DID, and the extra last row (rows outside any group), exclude nothing
            for (uint32_t g = threadIdx.x; g <= p.n_groups; g += kThreads) {
                uint32_t keep = 0;
                if (g < p.n_groups) {
                    // the first round's entries were requested with the tables
                    const uint2 s8 = g < (uint32_t)kThreads ? sub0 : *reinterpret_cast<const uint2*>(p.sub + (size_t)g * 8);
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const uint32_t d = ((k < 4 ? s8.x : s8.y) >> (8 * (k & 3))) & 0xFFu;
                        if (d < p.n_dialects) keep |= 1u << d;
                    }
                }
                uint32_t* row = reinterpret_cast<uint32_t*>(lds + kLdsSeda + g * 32);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t k4 = (keep >> (4 * i)) & 0xFu;
                    // bit j of k4 set -> byte j 0x00, else 0xFF
                    const uint32_t ex = ((k4 & 1u) ? 0u : 0x000000FFu) | ((k4 & 2u) ? 0u : 0x0000FF00u) |
                                        ((k4 & 4u) ? 0u : 0x00FF0000u) | ((k4 & 8u) ? 0u : 0xFF000000u);
                    row[i] = keep ? ex : 0u;
                }
            }
        }
        __syncthreads();
        // pair table: byte(hi, lo, d) = index(d, lo) | index(d, hi) << 4
        for (int i = threadIdx.x; i < 1024; i += kThreads) {
            const int hi = i >> 5, lo = i & 31;
            const uint4* rl = reinterpret_cast<const uint4*>(lds + kLdsNibT + lo * 32);
            const uint4* rh = reinterpret_cast<const uint4*>(lds + kLdsNibT + hi * 32);
            uint4* dst = reinterpret_cast<uint4*>(lds + kLdsPair + i * 32);
            const uint4 l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
            dst[0] = make_uint4(l0.x | (h0.x << 4), l0.y | (h0.y << 4), l0.z | (h0.z << 4), l0.w | (h0.w << 4));
            dst[1] = make_uint4(l1.x | (h1.x << 4), l1.y | (h1.y << 4), l1.z | (h1.z << 4), l1.w | (h1.w << 4));
        }
        // (the salient-row tables come after the pair table: their list is still on its way from memory)
        if (kDecomp) {
            // Salient rows as a bitmap.  The list is ascending and unique, so the position of row r in it is
            // (entries below row 0) + (salient rows below r): kept as a running count per bitmap word.
            constexpr uint32_t kWords = kMaxFusedRows / 32;
            constexpr uint32_t kWpt = (kWords + kThreads - 1) / kThreads;   // bitmap words per thread
            uint32_t* bits = reinterpret_cast<uint32_t*>(lds + kLdsSalBits);
            auto mark = [&](int32_t r) {
                if (r < 0) atomicAdd(&sal_before, 1u);
                else if ((uint32_t)r < p.rows) atomicOr(bits + ((uint32_t)r >> 5), 1u << (r & 31));
            };
            if (sal_early) {
#pragma unroll
                for (int k = 0; k < kSalEarly; ++k) mark(sal_reg[k]);
            } else {
                for (uint32_t i = threadIdx.x; i < p.n_sal; i += kThreads) mark(p.salient[i]);
            }
            __syncthreads();
            uint32_t run[kWpt];   // salient rows in this thread's words before word k
            uint32_t total = 0;
#pragma unroll
            for (uint32_t k = 0; k < kWpt; ++k) {
                const uint32_t wi = threadIdx.x * kWpt + k;
                run[k] = total;
                total += wi < kWords ? (uint32_t)__builtin_popcount(bits[wi]) : 0u;
            }
            uint32_t incl = total;   // inclusive scan over the wavefront
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t v = __shfl_up(incl, off);
                if ((int)lane >= off) incl += v;
            }
            if (lane == 63) sal_wave[wave] = incl;
            __syncthreads();
            uint32_t base = sal_before + incl - total;
            for (uint32_t k = 0; k < wave; ++k) base += sal_wave[k];
#pragma unroll
            for (uint32_t k = 0; k < kWpt; ++k) {
                const uint32_t wi = threadIdx.x * kWpt + k;
                if (wi < kWords) reinterpret_cast<uint16_t*>(lds + kLdsSalRank)[wi] = (uint16_t)(base + run[k]);
            }
        }
        __syncthreads();
    }
    TileConsts K = make_tile_consts(lane, kLdsGm);
    if (kCounts) K.mx = make_count_consts(lds, lds_count_offset(kSeda, kRes, 0) + wave * kHistWaveBytes, lane);
    if (kSse)
        K.mx = make_matrix_consts(lds, kLdsGm, lds_matrix_offset(kSeda, kRes),
                                  wave < 2 ? kLdsRows + wave * kHistWaveBytes
                                           : lds_hist_offset(kSeda, kRes, 2) + (wave - 2) * kHistWaveBytes, lane);

    // Results of a tile are held in registers and written at the top of the next iteration, right after
    // that iteration's input has arrived: memory operations retire in issue order, so a store issued just
    // before the wait for the next input would stall the wavefront for the whole write latency.
    uint4 held_code = make_uint4(0, 0, 0, 0);
    uint32_t held_meta = 0, held_gb = 0;
    bool have_held = false;   // wave-uniform
    bool held_ok = true;      // second plane only: this lane's list entry names a row of the tensor
    // second plane of a salient tile: held the same way
    uint4 held2_code = make_uint4(0, 0, 0, 0);
    uint32_t held2_meta = 0;
    size_t held2_ob = 0;
    bool held2_lane = false;   // this lane has a second-plane block to write
    bool held2_any = false;    // wave-uniform
    const bool meta_aligned = (reinterpret_cast<uintptr_t>(p.meta) & 15u) == 0;

    auto store_plane2 = [&]() {
        if (held2_lane) {
            *reinterpret_cast<uint4*>(p.codes2 + held2_ob * 16) = held2_code;
            if (kBlock == 16) {
                p.meta2[held2_ob * 2] = (uint16_t)held2_meta;
                p.meta2[held2_ob * 2 + 1] = (uint16_t)(held2_meta >> 16);
            } else {
                p.meta2[held2_ob] = (uint16_t)held2_meta;
            }
        }
    };
    while (t < p.n_tiles) {
        const uint32_t gb = t * 64u + lane;
        uint32_t w[16];
        w[0] = cur.q0.x; w[1] = cur.q0.y; w[2] = cur.q0.z; w[3] = cur.q0.w;
        w[4] = cur.q1.x; w[5] = cur.q1.y; w[6] = cur.q1.z; w[7] = cur.q1.w;
        w[8] = cur.q2.x; w[9] = cur.q2.y; w[10] = cur.q2.z; w[11] = cur.q2.w;
        w[12] = cur.q3.x; w[13] = cur.q3.y; w[14] = cur.q3.z; w[15] = cur.q3.w;
        // The previous tile's stores must not be scheduled above the arrival of this tile's input, and the
        // row's SeDA group (the last load of the tile) is consumed here too: left to the compiler, the wait
        // for it lands behind the next tile's loads and waits for those as well.
        int32_t grp = kSeda ? cur.grp : -1;
        // (second plane only: the first plane's words and the rows of the next tile arrive with the tile too)
        uint32_t c1m1[5] = {cur.c1.x, cur.c1.y, cur.c1.z, cur.c1.w, cur.m1};
        const int32_t row = cur.row;
        if (kGather)
            asm volatile("" : "+v"(row_next), "+v"(c1m1[0]), "+v"(c1m1[1]), "+v"(c1m1[2]), "+v"(c1m1[3]), "+v"(c1m1[4]));
        asm volatile("" : "+v"(held_meta), "+v"(grp) : "v"(w[0]), "v"(w[15]));
        const uint32_t excl_a = kLdsSeda + 32u * ((grp >= 0 && (uint32_t)grp < p.n_groups) ? (uint32_t)grp : p.n_groups);
        if (have_held) store_tile<kBlock>(p, held_gb, lane, held_code, held_meta, meta_aligned, held_ok);
        have_held = true;
        if (kDecomp && held2_any) store_plane2();
        held2_any = false;
        // the next tile's loads go out before this tile's arithmetic
        cur = load_block<kBlock, kFlat, kSeda, kGather>(p, t_next * 64u + lane, row_next);
        uint32_t claim = 0;
        if (lane == 0) claim = atomicAdd(&wg_next, 1u);
        const uint32_t t_after = blockIdx.x + (uint32_t)__builtin_amdgcn_readfirstlane(claim) * W;
        if (kGather) row_next = load_row(p, t_after * 64u + lane);
        uint32_t code[4], meta;
        bool tile_special;
        if (kGather) {
            // Sec. 3.3: residual of the first plane (exact, rounded once to bf16), then the same routine on it
            const bool ok = gb < p.n_blocks && row >= 0;
            const uint32_t gbc = min(gb, p.n_blocks - 1u);
            const uint32_t pos = (uint32_t)(((unsigned long long)gbc * p.div_mul) >> p.div_shift);
            const uint16_t* xb = p.x + (long long)(ok ? row : 0) * p.row_stride + (long long)(gbc - pos * p.nb) * 32;
            const uint32_t code1[4] = {c1m1[0], c1m1[1], c1m1[2], c1m1[3]};
            uint32_t w2[16];
            residual32<kBlock>(w, code1, c1m1[4], lds, true, w2);
            // a lane without a row runs the arithmetic on zeros and stores nothing
#pragma unroll
            for (int k = 0; k < 16; ++k) w2[k] = ok ? w2[k] : 0u;
            compute_tile<kBlock, G, kTwoStage, kSeda, true>(w2, lds, K, xb, ok, excl_a, code, meta, code1, c1m1[4],
                                                            tile_special);
            held_ok = ok;
        } else {
            const uint16_t* xb = p.x + block_offset<kFlat>(p, gb < p.n_blocks ? gb : 0u);
            const uint32_t no_code[4] = {0, 0, 0, 0};
            compute_tile<kBlock, G, kTwoStage, kSeda, false, kCounts>(w, lds, K, xb, gb < p.n_blocks, excl_a, code, meta,
                                                                      no_code, 0u, tile_special);
            if (kDecomp) {
                // second plane of the salient rows, from the registers that still hold the tile
                const uint32_t gbc = gb < p.n_blocks ? gb : 0u;
                const uint32_t row = (uint32_t)(((unsigned long long)gbc * p.div_mul) >> p.div_shift);
                const bool sal = gb < p.n_blocks &&
                                 ((reinterpret_cast<const uint32_t*>(lds + kLdsSalBits)[row >> 5] >> (row & 31)) & 1u);
                if (__builtin_amdgcn_ballot_w64(sal) != 0) {
                    // position of the row in the salient list
                    const uint32_t wbits = reinterpret_cast<const uint32_t*>(lds + kLdsSalBits)[row >> 5];
                    const uint32_t lo = reinterpret_cast<const uint16_t*>(lds + kLdsSalRank)[row >> 5] +
                                        __builtin_popcount(wbits & ((1u << (row & 31)) - 1u));
                    uint32_t w2[16], code2[4], meta2;
                    residual32<kBlock>(w, code, meta, lds, tile_special, w2);
                    // a lane that is not salient runs the arithmetic on zeros and stores nothing
#pragma unroll
                    for (int k = 0; k < 16; ++k) w2[k] = sal ? w2[k] : 0u;
                    bool special2;
                    compute_tile<kBlock, G, kTwoStage, kSeda, true>(w2, lds, K, xb, sal, excl_a, code2, meta2, code, meta,
                                                                    special2);
                    held2_any = true;
                    held2_lane = sal;
                    held2_ob = (size_t)lo * p.nb + (gb - row * p.nb);
                    held2_code = make_uint4(code2[0], code2[1], code2[2], code2[3]);
                    held2_meta = meta2;
                }
            }
        }
        held_code = make_uint4(code[0], code[1], code[2], code[3]);
        held_meta = meta;
        held_gb = gb;
        t = t_next;
        t_next = t_after;
    }
    if (have_held) store_tile<kBlock>(p, held_gb, lane, held_code, held_meta, meta_aligned, held_ok);
    if (kDecomp && held2_any) store_plane2();
}

}  // namespace fb4
