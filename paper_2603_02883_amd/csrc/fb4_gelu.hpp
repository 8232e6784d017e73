// The online quantizer fused behind a GeLU (App. E.2: quantization runs inside
// the operation that produces the activation; GeLU is one of the two the paper
// names).  One pass: x is read once, GeLU(x) never reaches memory.
//
// GeLU on bf16 is a function of 65536 bit patterns, and its result rounded to
// bf16 is what the quantizer sees, so the kernel looks it up instead of
// evaluating it: the host evaluates x Phi(x) (or the tanh form) in double
// for every pattern once, rounds once to bf16 (nearest even), and the kernel
// keeps the table in LDS.  Indexed by the bit pattern itself, clamped with one
// unsigned 16-bit minimum: patterns 0x0000..0x7FFF are the positive values
// (identity from 16 upwards, +Inf -> +Inf, +NaN -> 0x7FC0), 0x8000..0xC180 the
// negative values down to -16, and everything beyond -16 (-Inf included: the
// limit) is -0 like -16 itself.  Only a negative NaN needs a second look: the
// largest pattern of a tile is tracked and such a tile is patched.
#pragma once

#include <cmath>
#include <cstring>

#include "fb4_fast.hpp"

namespace fb4 {

constexpr uint32_t kGeluClamp = 0xC180u;                          // -16.0
constexpr uint32_t kGeluEntries = kGeluClamp + 1u;                // 49537
constexpr uint32_t kGeluTableBytes = ((kGeluEntries * 2u + 15u) / 16u) * 16u;   // 99088
// Runs of the table that follow from the bit pattern alone (both forms of GeLU; multiples of 8 entries):
// magnitudes [kGeluSubnormalEnd, kGeluHalfEnd) of either sign map to pattern - 0x80 (x / 2), positive
// patterns from kGeluIdentityBegin to +Inf map to themselves.
constexpr int kGeluSubnormalEnd = 0x0100, kGeluHalfEnd = 0x3B00, kGeluIdentityBegin = 0x4038;

// ---- host: the table
// double -> bf16 bits, one rounding to nearest even, from the bits of the double.
inline uint16_t bf16_from_double(double v)
{
    uint64_t b;
    std::memcpy(&b, &v, 8);
    const uint16_t sign = (uint16_t)((b >> 48) & 0x8000u);
    const int ef = (int)((b >> 52) & 0x7FF);
    const uint64_t frac = b & ((1ull << 52) - 1);
    if (ef == 0x7FF) return frac ? (uint16_t)0x7FC0 : (uint16_t)(sign | 0x7F80);
    if (ef == 0) return sign;   // zero or a double subnormal: far below the bf16 range
    int E = ef - 1023;
    const uint64_t sig = (1ull << 52) | frac;   // value = sig * 2^(E - 52)
    int shift = 45;                             // keep 8 significant bits
    if (E < -126) shift += -126 - E;            // subnormal result: fixed step 2^-133
    if (shift > 62) return sign;
    uint64_t q = sig >> shift;
    const uint64_t rem = sig & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (q & 1))) ++q;
    if (E < -126) return (uint16_t)(sign | q);  // q == 128 is the smallest normal
    if (q == 256) { q = 128; ++E; }
    if (E + 127 >= 255) return (uint16_t)(sign | 0x7F80);
    return (uint16_t)(sign | ((E + 127) << 7) | (q - 128));
}

// GeLU of the value with bit pattern h.  approximate: false = x Phi(x), true = the tanh form.
inline uint16_t gelu_entry(uint16_t h, bool approximate)
{
    const uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    if ((h & 0x7FFFu) > 0x7F80u) return 0x7FC0;
    if ((h & 0x7FFFu) == 0x7F80u) return (h & 0x8000u) ? 0x8000 : 0x7F80;
    if ((h & 0x7FFFu) == 0) return h;
    const double x = (double)f;
    if (!approximate) return bf16_from_double(0.5 * x * std::erfc(-x * 0.70710678118654752440));
    const double t = 0.79788456080286535588 * (x + 0.044715 * x * x * x);
    return bf16_from_double(x / (1.0 + std::exp(-2.0 * t)));
}

// table[k] for k = 0 .. kGeluClamp (see the head of this file); `table` holds kGeluTableBytes.
inline void build_gelu_table(bool approximate, uint16_t* table)
{
    std::memset(table, 0, kGeluTableBytes);
    for (uint32_t k = 0; k < kGeluEntries; ++k) table[k] = gelu_entry((uint16_t)k, approximate);
}

// ---- device
struct GeluParams {
    uint8_t* codes;
    uint16_t* meta;
    // Sec. 3.4 (optional): candidate lists per token group
    const int32_t* token_group;   // [rows] or null
    const uint8_t* sub;           // [n_groups][8] DIDs
    uint32_t n_groups;            // <= kMaxFusedProducerGroups
    uint32_t n_dialects;
};

// 16 wavefronts per CU (the kernel needs about 100 vector registers): 27.6 us on a 16384x3072 tensor against
// 29.8 with 12 and 34.1 with 8 -- the lookups' LDS latency wants more wavefronts than the plain quantizer's 8.
#ifndef FB4_GELU_THREADS
#define FB4_GELU_THREADS 1024
#endif
constexpr int kGeluThreads = FB4_GELU_THREADS;
constexpr int kLdsGelu = lds_fast_bytes(false, false, false);

// kBlock, G: block size (32 or 16) and number of groups of the online selector (Sec. 3.2, Sec. 4.1).
template <int kBlock, int G, bool kTwoStage, bool kSeda>
__global__ __launch_bounds__(kGeluThreads) void gelu_quantize_kernel(
    const uint8_t* blob, const uint16_t* x, const uint16_t* table, uint32_t n_blocks, uint32_t n_tiles, uint32_t div_mul,
    uint32_t div_shift, uint32_t nb, uint32_t n_workgroups, long long row_stride, GeluParams p)
{
    constexpr int kWaves = kGeluThreads / 64;
    constexpr int kLdsSeda = kLdsGelu + kGeluTableBytes;
    __shared__ __align__(16) uint8_t lds[kLdsSeda + (kSeda ? (kMaxFusedProducerGroups + 1) * 32 : 0)];
    __shared__ uint32_t wg_next;
    const uint16_t* lds_tab = reinterpret_cast<const uint16_t*>(lds + kLdsGelu);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t W = n_workgroups;
    FastParams sp = {};   // addressing and stores as in the streaming kernel
    sp.x = x; sp.row_stride = row_stride; sp.nb = nb; sp.n_blocks = n_blocks; sp.n_tiles = n_tiles;
    sp.div_mul = div_mul; sp.div_shift = div_shift; sp.codes = p.codes; sp.meta = p.meta;

    // A chunk past the end is read from the last one instead: no branch around the loads, nothing of it stored.
    auto request = [&](uint32_t t, uint32_t (&q)[16], int32_t& grp) {
        const uint32_t gbc = min(t * 64u + lane, n_blocks - 1u);
        if (kSeda) grp = p.token_group[(uint32_t)(((unsigned long long)gbc * div_mul) >> div_shift)];
        const uint4* px = reinterpret_cast<const uint4*>(x + block_offset<false>(sp, gbc));
        const uint4 q0 = px[0], q1 = px[1], q2 = px[2], q3 = px[3];
        q[0] = q0.x; q[1] = q0.y; q[2] = q0.z; q[3] = q0.w; q[4] = q1.x; q[5] = q1.y; q[6] = q1.z; q[7] = q1.w;
        q[8] = q2.x; q[9] = q2.y; q[10] = q2.z; q[11] = q2.w; q[12] = q3.x; q[13] = q3.y; q[14] = q3.z; q[15] = q3.w;
    };
    uint32_t t = blockIdx.x + wave * W;
    uint32_t t_next = blockIdx.x + (kWaves + wave) * W;
    if (threadIdx.x == 0) wg_next = 2 * kWaves;
    uint32_t w[16];
    int32_t grp = -1;   // SeDA: the token group of the chunk's row

    // ---- tables (layout of the streaming kernel) and the GeLU table.  Loads are answered in the order they were
    // issued: the table pieces are requested first (into registers, one of each kind per thread) and the first
    // tile right behind them, so that the tables can be written -- and most of the GeLU table generated -- while
    // the tile is still on its way, instead of after it.
    static_assert(64 * kRowCopies <= kGeluThreads && 256 <= kGeluThreads, "one piece of each table per thread");
    // Most of the GeLU table follows from the bit pattern: GeLU(x) rounds to x / 2 (pattern - 0x80) for
    // 2^-125 <= |x| < 2^-9.25, to x from 2.875 upwards, a positive NaN gives the quiet NaN.  Only the
    // 16-byte pieces outside these runs are read from memory, at most one per thread.
    constexpr int kPieces = kGeluTableBytes / 16;   // 6193 pieces of 8 entries
    constexpr int kSub = kGeluSubnormalEnd / 8, kHalf = kGeluHalfEnd / 8, kIdent = kGeluIdentityBegin / 8;
    constexpr int kNeg = 0x8000 / 8;
    constexpr int kRunA = kSub, kRunB = kIdent - kHalf, kRunC = kSub, kRunD = kPieces - (kNeg + kHalf);
    static_assert(kRunA + kRunB + kRunC + kRunD <= kGeluThreads, "one loaded piece per thread");
    const int tid = threadIdx.x;
    int mine = -1;   // the piece of the GeLU table this thread reads
    if (tid < kRunA) mine = tid;
    else if (tid < kRunA + kRunB) mine = kHalf + (tid - kRunA);
    else if (tid < kRunA + kRunB + kRunC) mine = kNeg + (tid - kRunA - kRunB);
    else if (tid < kRunA + kRunB + kRunC + kRunD) mine = kNeg + kHalf + (tid - kRunA - kRunB - kRunC);
    // (indices are clamped, not predicated: a thread without a piece loads one it does not write)
    const int ri = min(tid, 64 * kRowCopies - 1);
    const uint4 rowv = *reinterpret_cast<const uint4*>(blob + kOffQerror8 + (ri / (2 * kRowCopies)) * 32 + ((ri / kRowCopies) & 1) * 16);
    const uint32_t nibv = reinterpret_cast<const uint32_t*>(blob + kOffQvalueT)[tid & 255];
    const uint32_t rngv = kTwoStage ? reinterpret_cast<const uint32_t*>(blob + kOffRangeExcl)[tid & 63] : 0u;
    const uint4 loaded = reinterpret_cast<const uint4*>(table)[mine < 0 ? 0 : mine];
    __builtin_amdgcn_sched_barrier(0);
    request(min(t, n_tiles - 1u), w, grp);
    __builtin_amdgcn_sched_barrier(0);
    {
        uint4* dst = reinterpret_cast<uint4*>(lds + kLdsGelu);
        for (int i = tid; i < kPieces; i += kGeluThreads) {
            const int ip = i & (kNeg - 1);   // piece index within its sign
            const bool from_memory = ip < kSub || (i < kNeg ? (ip >= kHalf && ip < kIdent) : ip >= kHalf);
            if (from_memory) continue;
            uint32_t e[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t pair = 0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t k = 8u * i + 2u * j + h;
                    const uint32_t v = ip < kHalf ? k - 0x80u : (k <= 0x7F80u ? k : 0x7FC0u);
                    pair |= v << (16 * h);
                }
                e[j] = pair;
            }
            dst[i] = make_uint4(e[0], e[1], e[2], e[3]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (tid < 64 * kRowCopies) reinterpret_cast<uint4*>(lds + kLdsRows)[tid] = rowv;
        if (tid < 256) reinterpret_cast<uint32_t*>(lds + kLdsNibT)[tid] = nibv;
        if (kTwoStage && tid < 64) reinterpret_cast<uint32_t*>(lds + kLdsRange)[tid] = rngv;
        if (mine >= 0) dst[mine] = loaded;
    }
    if (kSeda) build_seda_rows(lds, kLdsSeda, p.sub, p.n_groups, p.n_dialects, kGeluThreads);
    __syncthreads();
    for (int i = threadIdx.x; i < 1024; i += kGeluThreads) {   // pair table: byte(hi, lo, d) = index(d, lo) | index(d, hi) << 4
        const int hi = i >> 5, lo = i & 31;
        const uint4* rl = reinterpret_cast<const uint4*>(lds + kLdsNibT + lo * 32);
        const uint4* rh = reinterpret_cast<const uint4*>(lds + kLdsNibT + hi * 32);
        uint4* dst = reinterpret_cast<uint4*>(lds + kLdsPair + i * 32);
        const uint4 l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
        dst[0] = make_uint4(l0.x | (h0.x << 4), l0.y | (h0.y << 4), l0.z | (h0.z << 4), l0.w | (h0.w << 4));
        dst[1] = make_uint4(l1.x | (h1.x << 4), l1.y | (h1.y << 4), l1.z | (h1.z << 4), l1.w | (h1.w << 4));
    }
    __syncthreads();
    const TileConsts K = make_tile_consts(lane, 0);
    const bool meta_aligned = (reinterpret_cast<uintptr_t>(p.meta) & 15u) == 0;
    const uint32_t kclamp = sgpr_const(kGeluClamp | (kGeluClamp << 16));

    while (t < n_tiles) {
        uint32_t claim = 0;
        if (lane == 0) claim = atomicAdd(&wg_next, 1u);
        const uint32_t t_after = blockIdx.x + (uint32_t)__builtin_amdgcn_readfirstlane(claim) * W;
        const uint32_t gb = t * 64u + lane;
        const uint32_t excl = kSeda ? kLdsSeda + 32u * ((grp >= 0 && (uint32_t)grp < p.n_groups) ? (uint32_t)grp : p.n_groups) : 0u;
        // ---- GeLU of the 32 elements: two table lookups per register
        uint32_t y[16];
        uint32_t top = 0;   // largest bit pattern of the chunk, per half
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t idx = pk_min(w[k], kclamp);
            y[k] = (uint32_t)lds_tab[idx & 0xFFFFu] | ((uint32_t)lds_tab[idx >> 16] << 16);
            top = pk_max(top, w[k]);
        }
        if (__builtin_amdgcn_ballot_w64(halves_max(top) > 0xFF80u) != 0) {
            // rare: a negative NaN somewhere in the tile (the clamp made it -0)
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                if ((w[k] & 0xFFFFu) > 0xFF80u) y[k] = (y[k] & 0xFFFF0000u) | 0x7FC0u;
                if ((w[k] >> 16) > 0xFF80u) y[k] = (y[k] & 0xFFFFu) | 0x7FC00000u;
            }
        }
        // the registers of the tile are free: the next tile is requested into them, ahead of the selection
        request(min(t_next, n_tiles - 1u), w, grp);
        __builtin_amdgcn_sched_barrier(0);
        uint32_t stage[16];   // the plain routine reads its block from memory: used by special tiles only
        uint32_t code[4], meta;
        bool tile_special;
        const uint32_t no_code[4] = {0, 0, 0, 0};
        compute_tile<kBlock, G, kTwoStage, kSeda>(y, lds, K, nullptr, gb < n_blocks, excl, code, meta, no_code, 0u, tile_special, stage);
        store_tile<kBlock>(sp, gb, lane, make_uint4(code[0], code[1], code[2], code[3]), meta, meta_aligned);
        t = t_next;
        t_next = t_after;
    }
}

}  // namespace fb4
