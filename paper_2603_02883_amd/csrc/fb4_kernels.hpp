// gfx950 kernels of the FB4 online quantizer (Sec. 3.1-3.4 of the paper).
//
// Work mapping.  A wavefront (64 lanes) handles one "tile": 512 consecutive
// elements of ONE tensor row.  Every lane loads 16 bytes = 8 bf16 elements, so a
// wavefront load is 1 KiB of contiguous memory.  LPB neighbouring lanes own one
// block: the four lanes of a quad for block size 32, a pair of lanes for block
// size 16.  Reductions over a block are DPP operations inside the quad.  The lookup tables live in LDS.  All arithmetic is integer
// arithmetic on the bf16 bit pattern, so results do not depend on floating
// point modes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fb4_tables.hpp"

namespace fb4 {

constexpr int kThreads = 256;          // 4 wavefronts per workgroup
constexpr int kWavesPerGroup = kThreads / 64;
constexpr int kTileElems = 512;         // elements of one row a wavefront handles at a time

enum Mode : int { kPlain = 0, kSeda = 1, kDecomp = 2 };
enum Selector : int { kSelSse = 0, kSelLut = 1 };

struct QuantParams {
    const uint16_t* x;       // [rows][row_stride] bf16 bits
    long long row_stride;    // elements
    long long rows;          // rows of x
    long long cols;          // elements per row (a multiple of the block size)
    int nb;                  // blocks per row
    int tiles_per_row;       // ceil(cols / 512)
    int n_tiles;             // tiles over the OUTPUT rows
    uint8_t* codes;          // [out_rows][nb*16]
    uint16_t* meta;          // [out_rows][nb]
    const int32_t* token_group;  // [rows] or null
    const uint8_t* sub;          // [n_groups][8] or null
    int n_groups;
    const uint8_t* codes1;   // decomposition: first plane
    const uint16_t* meta1;
    const int32_t* salient;  // [out_rows] source row of each output row
    const uint8_t* blob;     // lookup tables (device)
    int n_dialects;
};

struct DequantParams {
    const uint8_t* codes1;
    const uint16_t* meta1;
    const uint8_t* codes2;   // null for the plane-1 pass
    const uint16_t* meta2;
    const int32_t* salient;  // null for the plane-1 pass
    long long rows;          // rows of the output tensor
    long long cols;
    int nb;                  // blocks per row
    int block_shift;         // log2(block size): 4 or 5
    int tiles_per_row;
    int n_tiles;
    void* out;
    long long out_row_stride;
    const uint8_t* blob;
};

// ------------------------------------------------------------------ helpers
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v, int l)
{
    switch (l) {
    case 0: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x00, 0xF, 0xF, true);
    case 1: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x55, 0xF, 0xF, true);
    case 2: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xAA, 0xF, 0xF, true);
    default: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xFF, 0xF, 0xF, true);
    }
}
__device__ __forceinline__ uint32_t quad_xor1(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t quad_xor2(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t quad_max(uint32_t v)
{
    v = max(v, quad_xor1(v));
    return max(v, quad_xor2(v));
}
__device__ __forceinline__ uint32_t quad_min(uint32_t v)
{
    v = min(v, quad_xor1(v));
    return min(v, quad_xor2(v));
}
__device__ __forceinline__ uint32_t quad_or(uint32_t v)
{
    v |= quad_xor1(v);
    return v | quad_xor2(v);
}

// Reductions and broadcasts over the LPB lanes of one block.
template <int LPB>
__device__ __forceinline__ uint32_t blk_max(uint32_t v)
{
    v = max(v, quad_xor1(v));
    return LPB == 4 ? max(v, quad_xor2(v)) : v;
}
template <int LPB>
__device__ __forceinline__ uint32_t blk_min(uint32_t v)
{
    v = min(v, quad_xor1(v));
    return LPB == 4 ? min(v, quad_xor2(v)) : v;
}
// value held by lane l of this lane's block
template <int LPB>
__device__ __forceinline__ uint32_t blk_bcast(uint32_t v, int l)
{
    if (LPB == 4) return quad_bcast(v, l);
    if (l == 0) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xA0, 0xF, 0xF, true);   // lanes 0,0,2,2
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xF5, 0xF, 0xF, true);                // lanes 1,1,3,3
}
// N consecutive dwords from LDS with the widest loads
template <int N>
__device__ __forceinline__ void lds_dwords(const uint8_t* p, uint32_t (&o)[N])
{
    static_assert(N == 2 || N == 4 || N == 8, "2, 4 or 8 dwords");
    if (N == 2) {
        const uint2 r = *reinterpret_cast<const uint2*>(p);
        o[0] = r.x; o[1] = r.y;
    } else {
#pragma unroll
        for (int k = 0; k < N / 4; ++k) {
            const uint4 r = reinterpret_cast<const uint4*>(p)[k];
            o[4 * k] = r.x; o[4 * k + 1] = r.y; o[4 * k + 2] = r.z; o[4 * k + 3] = r.w;
        }
    }
}

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b)
{
    ushort2_t r = __builtin_elementwise_min(__builtin_bit_cast(ushort2_t, a),
                                            __builtin_bit_cast(ushort2_t, b));
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ void copy_tables_to_lds(uint8_t* lds, const uint8_t* blob)
{
    const uint4* src = reinterpret_cast<const uint4*>(blob);
    uint4* dst = reinterpret_cast<uint4*>(lds);
    for (int i = threadIdx.x; i < (int)(kBlobBytes / 16); i += kThreads) dst[i] = src[i];
    __syncthreads();
}

// One lane's eight elements after normalization (Sec. 3.1).
struct Lane8 {
    uint32_t bin[8];   // min(31, floor(2 * xhat))             (Sec. 3.2 bins)
    uint32_t frac[8];  // 256*xhat - 128*bin, 0..128           (exhaustive selector only)
    uint32_t sign[8];  // 0 / 1
    uint32_t ebyte;    // shared exponent + 127, 4..254
    uint32_t binmax;   // bin of the block maximum
};

// Shared exponent and bins from the raw bf16 patterns of a block.
//   h[i]: the 16-bit patterns of this lane's elements.
template <bool kNeedFrac, int LPB>
__device__ __forceinline__ void normalize_block(const uint32_t (&h)[8], Lane8& o)
{
    uint32_t a[8];
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        o.sign[i] = h[i] >> 15;
        uint32_t m = h[i] & 0x7FFFu;
        a[i] = (m > 0x7F80u) ? 0u : m;  // NaN: ignored (treated as a signed zero)
        amax = max(amax, a[i]);
    }
    amax = blk_max<LPB>(amax);                        // block maximum (bit patterns are monotonic)
    uint32_t eb = min(max(amax >> 7, 4u), 254u);      // floor(log2 max) + 127, clamped
    o.ebyte = eb;
    uint32_t bmax = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t ef = a[i] >> 7;
        uint32_t sig = (a[i] & 0x7Fu) | (ef ? 0x80u : 0u);   // 1.m as an 8-bit integer (0.m if subnormal)
        uint32_t sh = eb + 3u - max(ef, 1u);                 // >= 2; xhat = sig * 2^-sh * ... see below
        // X = 256 * xhat = sig * 2^(7 - sh); exact whenever xhat >= 0.5 (sh <= 7)
        uint32_t X = (sh <= 7u) ? (sig << (7u - sh)) : (sig >> min(sh - 7u, 31u));
        uint32_t b = min(X >> 7, 31u);
        o.bin[i] = b;
        if (kNeedFrac) o.frac[i] = X - (b << 7);
        bmax = max(bmax, b);
    }
    o.binmax = blk_max<LPB>(bmax);
}

// LDS table views
struct Tables {
    const uint8_t* qerr8;
    const uint8_t* qval;
    const uint8_t* qerr16;
    const uint8_t* mag16;
    const uint8_t* gain16;
    const uint16_t* decode;
    const uint8_t* top;
};
__device__ __forceinline__ Tables table_views(const uint8_t* lds)
{
    Tables t;
    t.qerr8 = lds + kOffQerror8;
    t.qval = lds + kOffQvalue64;
    t.qerr16 = lds + kOffQerror16;
    t.mag16 = lds + kOffMag16;
    t.gain16 = lds + kOffGain16;
    t.decode = reinterpret_cast<const uint16_t*>(lds + kOffDecode);
    t.top = lds + kOffTop;
    return t;
}

// Group-wise maxima (Sec. 3.2): the bin of a group's maximum is the maximum of
// its bins.  Groups are contiguous runs of PER elements; this lane owns 8 / PER.
template <int PER>
__device__ __forceinline__ void group_bins(const Lane8& e, uint32_t (&gb)[8 / PER])
{
#pragma unroll
    for (int g = 0; g < 8 / PER; ++g) {
        uint32_t m = e.bin[g * PER];
#pragma unroll
        for (int i = 1; i < PER; ++i) m = max(m, e.bin[g * PER + i]);
        gb[g] = m;
    }
}

// ---------------------------------------------------------------- selection
// Every select_* returns the winning DID, identical in all lanes of a block.
// Lane jb of a block (0..LPB-1) scores a share of the candidates.

// Keys of the lane's N candidates are (score << 5 | DID); smaller is better,
// 0xFFFFFFFF = no candidate.
// range = 0: no first stage; otherwise keep only dialects whose top magnitude
// equals `range`, unless no candidate of the block has it.
template <bool kTwoStage, int N, int LPB>
__device__ __forceinline__ uint32_t finish_min_keys(const uint32_t (&key)[N], const Tables& T, uint32_t range)
{
    uint32_t best = 0xFFFFFFFFu, bestf = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        best = min(best, key[i]);
        if (kTwoStage) {
            bool ok = key[i] != 0xFFFFFFFFu && T.top[key[i] & 31u] == range;
            bestf = min(bestf, ok ? key[i] : 0xFFFFFFFFu);
        }
    }
    best = blk_min<LPB>(best);
    if (kTwoStage) {
        bestf = blk_min<LPB>(bestf);
        if (bestf != 0xFFFFFFFFu) best = bestf;
    }
    return best & 31u;
}

// The paper's online rule over the full formatbook: lane jb of the block scores
// dialects jb*DPL .. jb*DPL + DPL-1 for all G group maxima of the block.
template <int G, bool kTwoStage, int LPB>
__device__ __forceinline__ uint32_t select_lut_full(const Lane8& e, const Tables& T, int jb, uint32_t range)
{
    constexpr int PER = 8 * LPB / G;     // elements per group
    constexpr int GL = 8 / PER;          // groups owned by this lane
    constexpr int DPL = 32 / LPB;        // dialects scored by this lane
    static_assert(PER >= 1 && PER <= 8, "a group lies inside one lane");
    uint32_t gb[GL];
    group_bins<PER>(e, gb);
    uint32_t key[DPL];
    if (G == 8) {
        // 8-bit fields: 8 groups x Qerror <= 31 stays below 256
        uint32_t acc[DPL / 4];
#pragma unroll
        for (int k = 0; k < DPL / 4; ++k) acc[k] = 0;
#pragma unroll
        for (int l = 0; l < LPB; ++l)
#pragma unroll
            for (int g = 0; g < GL; ++g) {
                const uint32_t b = blk_bcast<LPB>(gb[g], l);
                uint32_t r[DPL / 4];
                lds_dwords<DPL / 4>(T.qerr8 + b * 32 + jb * DPL, r);
#pragma unroll
                for (int k = 0; k < DPL / 4; ++k) acc[k] += r[k];
            }
#pragma unroll
        for (int k = 0; k < DPL / 4; ++k)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                key[4 * k + i] = (((acc[k] >> (8 * i)) & 0xFFu) << 5) | (uint32_t)(jb * DPL + 4 * k + i);
    } else {
        // 16-bit fields holding Qerror*32: 32 groups x 31*32 stays below 65536
        uint32_t acc[DPL / 2];
#pragma unroll
        for (int k = 0; k < DPL / 2; ++k) acc[k] = 0;
#pragma unroll
        for (int l = 0; l < LPB; ++l)
#pragma unroll
            for (int g = 0; g < GL; ++g) {
                const uint32_t b = blk_bcast<LPB>(gb[g], l);
                uint32_t r[DPL / 2];
                lds_dwords<DPL / 2>(T.qerr16 + b * 64 + jb * DPL * 2, r);
#pragma unroll
                for (int k = 0; k < DPL / 2; ++k) acc[k] += r[k];
            }
#pragma unroll
        for (int k = 0; k < DPL / 2; ++k) {
            key[2 * k] = (acc[k] & 0xFFFFu) | (uint32_t)(jb * DPL + 2 * k);
            key[2 * k + 1] = (acc[k] >> 16) | (uint32_t)(jb * DPL + 2 * k + 1);
        }
    }
    return finish_min_keys<kTwoStage, DPL, LPB>(key, T, range);
}

// The online rule over a SeDA sub-formatbook (Sec. 3.4): lane jb scores NC = 8 / LPB
// of the row's eight DIDs (bytes jb*NC .. of the list).
template <int G, bool kTwoStage, int LPB>
__device__ __forceinline__ uint32_t select_lut_seda(const Lane8& e, const Tables& T, const uint32_t (&c)[8 / LPB],
                                                    int n_dialects, uint32_t range)
{
    constexpr int PER = 8 * LPB / G, GL = 8 / PER, NC = 8 / LPB;
    uint32_t gb[GL];
    group_bins<PER>(e, gb);
    uint32_t d[NC], s[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        d[k] = c[k] < (uint32_t)n_dialects ? c[k] : 0u;
        s[k] = 0;
    }
#pragma unroll
    for (int l = 0; l < LPB; ++l)
#pragma unroll
        for (int g = 0; g < GL; ++g) {
            const uint32_t b = blk_bcast<LPB>(gb[g], l);
#pragma unroll
            for (int k = 0; k < NC; ++k) s[k] += T.qerr8[b * 32 + d[k]];
        }
    uint32_t key[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) key[k] = c[k] < (uint32_t)n_dialects ? ((s[k] << 5) | d[k]) : 0xFFFFFFFFu;
    return finish_min_keys<kTwoStage, NC, LPB>(key, T, range);
}

// Exhaustive squared error (Sec. 3.2, first paragraph).  With X = 256*xhat =
// 128*bin + frac and m the nearest magnitude of a dialect,
//   (X - 256 m)^2 = X^2 - 512 * Z,   Z = 128 * m*(bin-m) + frac*m,
// so the dialect with the smallest error is the one with the largest
// Z_d = 128 * sum gain[bin][d] + sum frac * mag[bin][d].  Both sums fit 16-bit
// fields over a whole block (<= 7680 and <= 61440), so two dialects share a
// 32-bit register.  Lane jb accumulates its DPL dialects over all elements.
template <bool kTwoStage, int LPB>
__device__ __forceinline__ uint32_t select_sse_full(const Lane8& e, const Tables& T, int jb, uint32_t range)
{
    constexpr int DPL = 32 / LPB;
    uint32_t U[DPL / 2], V[DPL / 2];
#pragma unroll
    for (int k = 0; k < DPL / 2; ++k) U[k] = V[k] = 0;
#pragma unroll
    for (int l = 0; l < LPB; ++l)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t b = blk_bcast<LPB>(e.bin[i], l);
            const uint32_t f = blk_bcast<LPB>(e.frac[i], l);
            uint32_t m[DPL / 2], g[DPL / 2];
            lds_dwords<DPL / 2>(T.mag16 + b * 64 + jb * DPL * 2, m);
            lds_dwords<DPL / 2>(T.gain16 + b * 64 + jb * DPL * 2, g);
#pragma unroll
            for (int k = 0; k < DPL / 2; ++k) {
                U[k] += g[k];
                V[k] += m[k] * f;
            }
        }
    // key: smaller is better -> invert Z (Z < 2^20)
    uint32_t key[DPL];
#pragma unroll
    for (int k = 0; k < DPL / 2; ++k) {
        const uint32_t zlo = ((U[k] & 0xFFFFu) << 7) + (V[k] & 0xFFFFu);
        const uint32_t zhi = ((U[k] >> 16) << 7) + (V[k] >> 16);
        key[2 * k] = ((0xFFFFFu - zlo) << 5) | (uint32_t)(jb * DPL + 2 * k);
        key[2 * k + 1] = ((0xFFFFFu - zhi) << 5) | (uint32_t)(jb * DPL + 2 * k + 1);
    }
    return finish_min_keys<kTwoStage, DPL, LPB>(key, T, range);
}

template <bool kTwoStage, int LPB>
__device__ __forceinline__ uint32_t select_sse_seda(const Lane8& e, const Tables& T, const uint32_t (&c)[8 / LPB],
                                                    int n_dialects, uint32_t range)
{
    constexpr int NC = 8 / LPB;
    const uint16_t* mag = reinterpret_cast<const uint16_t*>(T.mag16);
    const uint16_t* gain = reinterpret_cast<const uint16_t*>(T.gain16);
    uint32_t d[NC], z[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        d[k] = c[k] < (uint32_t)n_dialects ? c[k] : 0u;
        z[k] = 0;
    }
#pragma unroll
    for (int l = 0; l < LPB; ++l)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t b = blk_bcast<LPB>(e.bin[i], l);
            const uint32_t f = blk_bcast<LPB>(e.frac[i], l);
#pragma unroll
            for (int k = 0; k < NC; ++k)
                z[k] += ((uint32_t)gain[b * 32 + d[k]] << 7) + (uint32_t)mag[b * 32 + d[k]] * f;
        }
    uint32_t key[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k)
        key[k] = c[k] < (uint32_t)n_dialects ? (((0xFFFFFu - z[k]) << 5) | d[k]) : 0xFFFFFFFFu;
    return finish_min_keys<kTwoStage, NC, LPB>(key, T, range);
}

// ------------------------------------------------------------ quantize kernel
// LPB = lanes per block: 4 for block size 32, 2 for block size 16.
// What a lane reads for one tile: its eight elements and, for the second plane (Sec. 3.3), the first
// plane's code word and metadata of its block.
struct TileInput {
    uint4 w;
    uint32_t c1, m1;
    long long srow;   // source row of x
    bool live;        // false: the salient list names a row outside the tensor (wave-uniform)
};

// The leading scalar arguments repeat the fields of `p` that the first loads depend on; they arrive in
// registers when the wavefront starts (kernel-argument preload), the rest by a load.
template <int SEL, int G, int MODE, bool kTwoStage, int LPB>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const uint8_t* blob, const uint16_t* x,
                                                            const int32_t* salient, int n_tiles, int tiles_per_row,
                                                            int n_workgroups, long long row_stride, long long cols,
                                                            QuantParams p)
{
    p.blob = blob; p.x = x; p.salient = salient; p.n_tiles = n_tiles; p.tiles_per_row = tiles_per_row;
    p.row_stride = row_stride; p.cols = cols;
    __shared__ __align__(16) uint8_t lds[kBlobBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int jb = lane & (LPB - 1);      // lane within its block
    const int stride = n_workgroups * kWavesPerGroup;
    const long long code_pitch = p.cols / 2;

    auto request = [&](int t) {
        TileInput in;
        in.w = make_uint4(0, 0, 0, 0);
        in.c1 = in.m1 = 0;
        in.live = true;
        const int orow = t / p.tiles_per_row;               // output row (wave-uniform)
        const int chunk = t - orow * p.tiles_per_row;
        in.srow = orow;
        if (MODE == kDecomp) {
            in.srow = p.salient[orow];
            if (in.srow < 0 || in.srow >= p.rows) {
                in.live = false;
                return in;
            }
        }
        const long long col = (long long)chunk * kTileElems + lane * 8;   // first of this lane's 8 elements
        if (col < p.cols) {
            in.w = *reinterpret_cast<const uint4*>(p.x + in.srow * p.row_stride + col);
            if (MODE == kDecomp) {
                in.c1 = *reinterpret_cast<const uint32_t*>(p.codes1 + in.srow * code_pitch + col / 2);
                in.m1 = p.meta1[in.srow * p.nb + col / (8 * LPB)];
            }
        }
        return in;
    };

    // The wavefront's first tile is requested before the tables: it is on its way while they are copied.
    const int t_first = blockIdx.x * kWavesPerGroup + wave;
    TileInput in;
    in.live = false;
    if (t_first < p.n_tiles) in = request(t_first);
    copy_tables_to_lds(lds, p.blob);
    const Tables T = table_views(lds);

    for (int t = t_first; t < p.n_tiles; t += stride) {
        if (t != t_first) in = request(t);
        if (!in.live) continue;                             // wave-uniform
        const int orow = t / p.tiles_per_row;
        const int chunk = t - orow * p.tiles_per_row;
        const long long srow = in.srow;
        const long long col = (long long)chunk * kTileElems + lane * 8;
        const bool valid = col < p.cols;                    // the same for all lanes of a block
        const long long blk = col / (8 * LPB);              // block within the row

        const uint4 w = in.w;
        uint32_t h[8] = {w.x & 0xFFFFu, w.x >> 16, w.y & 0xFFFFu, w.y >> 16,
                         w.z & 0xFFFFu, w.z >> 16, w.w & 0xFFFFu, w.w >> 16};

        if (MODE == kDecomp) {
            // Sec. 3.3: residual of the first plane, exact, rounded once to bf16
            const uint32_t c1 = in.c1, m1 = in.m1;
            const uint32_t did1 = m1 & 0xFFu, e1 = m1 >> 8;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (((h[i] >> 7) & 0xFFu) == 0xFFu) continue;   // Inf / NaN: its own residual
                uint32_t nib = (c1 >> (4 * i)) & 0xFu;
                uint32_t mb = (did1 < 32u) ? (uint32_t)T.decode[did1 * 8 + (nib & 7u)] : 0u;
                uint32_t yb = mb ? ((mb + ((e1 - 130u) << 7)) & 0x7FFFu) : 0u;
                yb |= (nib & 8u) << 12;
                float d = __uint_as_float(h[i] << 16) - __uint_as_float(yb << 16);
                uint32_t u = __float_as_uint(d);
                u += 0x7FFFu + ((u >> 16) & 1u);
                h[i] = u >> 16;
            }
        }

        Lane8 e;
        normalize_block<SEL == kSelSse, LPB>(h, e);
        const uint32_t range = kTwoStage ? min(max(e.binmax >> 1, 8u), 15u) : 0u;

        // ---- candidates
        constexpr int NC = 8 / LPB;
        bool seda = false;
        uint32_t c[NC];
#pragma unroll
        for (int k = 0; k < NC; ++k) c[k] = 0;
        if (MODE == kSeda || MODE == kDecomp) {
            if (p.token_group != nullptr) {
                const int grp = p.token_group[srow];           // wave-uniform
                if (grp >= 0 && grp < p.n_groups) {
                    const uint8_t* s = p.sub + (long long)grp * 8;
                    bool any = false;
#pragma unroll
                    for (int k = 0; k < NC; ++k) {
                        c[k] = s[NC * jb + k];
                        any = any || (c[k] < (uint32_t)p.n_dialects);
                    }
                    seda = __builtin_amdgcn_ballot_w64(any) != 0;   // wave-uniform
                }
            }
        }

        uint32_t did;
        if (seda) {
            did = (SEL == kSelSse) ? select_sse_seda<kTwoStage, LPB>(e, T, c, p.n_dialects, range)
                                   : select_lut_seda<G, kTwoStage, LPB>(e, T, c, p.n_dialects, range);
        } else {
            did = (SEL == kSelSse) ? select_sse_full<kTwoStage, LPB>(e, T, jb, range)
                                   : select_lut_full<G, kTwoStage, LPB>(e, T, jb, range);
        }

        // ---- emit (Sec. 3.2: every element through Qvalue of the chosen dialect)
        uint32_t code = 0;
        const uint8_t* qv = T.qval + did * 64;
#pragma unroll
        for (int i = 0; i < 8; ++i) code |= (uint32_t)qv[(e.sign[i] << 5) | e.bin[i]] << (4 * i);
        if (valid) {
            *reinterpret_cast<uint32_t*>(p.codes + (long long)orow * code_pitch + col / 2) = code;
            if (jb == 0) p.meta[(long long)orow * p.nb + blk] = (uint16_t)(did | (e.ebyte << 8));
        }
    }
}

// ---------------------------------------------------------- dequantize kernel
// kSum = false: every row from plane 1.  kSum = true: the salient rows again,
// as the fp32 sum of both planes (Sec. 3.3).
template <bool kSum, bool kF32>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(DequantParams p)
{
    __shared__ __align__(16) uint16_t dec[32 * 8];
    for (int i = threadIdx.x; i < 32 * 8; i += kThreads)
        dec[i] = reinterpret_cast<const uint16_t*>(p.blob + kOffDecode)[i];
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int stride = gridDim.x * kWavesPerGroup;
    const long long code_pitch = p.cols / 2;

    for (int t = blockIdx.x * kWavesPerGroup + wave; t < p.n_tiles; t += stride) {
        const int prow = t / p.tiles_per_row;
        const int chunk = t - prow * p.tiles_per_row;
        long long orow = prow;
        if (kSum) {
            orow = p.salient[prow];
            if (orow < 0 || orow >= p.rows) continue;
        }
        const long long col = (long long)chunk * kTileElems + lane * 8;
        if (col >= p.cols) continue;   // no cross-lane operation below
        const long long blk = col >> p.block_shift;

        const uint32_t c1 = *reinterpret_cast<const uint32_t*>(p.codes1 + orow * code_pitch + col / 2);
        const uint32_t m1 = p.meta1[orow * p.nb + blk];
        uint32_t c2 = 0, m2 = 0;
        if (kSum) {
            c2 = *reinterpret_cast<const uint32_t*>(p.codes2 + (long long)prow * code_pitch + col / 2);
            m2 = p.meta2[(long long)prow * p.nb + blk];
        }
        uint32_t outb[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t nib = (c1 >> (4 * i)) & 0xFu;
            uint32_t mb = ((m1 & 0xFFu) < 32u) ? (uint32_t)dec[(m1 & 0xFFu) * 8 + (nib & 7u)] : 0u;
            uint32_t yb = mb ? ((mb + (((m1 >> 8) - 130u) << 7)) & 0x7FFFu) : 0u;
            yb |= (nib & 8u) << 12;
            uint32_t f = yb << 16;                      // fp32 bit pattern of y1
            if (kSum) {
                uint32_t nib2 = (c2 >> (4 * i)) & 0xFu;
                uint32_t mb2 = ((m2 & 0xFFu) < 32u) ? (uint32_t)dec[(m2 & 0xFFu) * 8 + (nib2 & 7u)] : 0u;
                uint32_t yb2 = mb2 ? ((mb2 + (((m2 >> 8) - 130u) << 7)) & 0x7FFFu) : 0u;
                yb2 |= (nib2 & 8u) << 12;
                f = __float_as_uint(__uint_as_float(f) + __uint_as_float(yb2 << 16));
            }
            outb[i] = f;
        }
        if (kF32) {
            float* o = reinterpret_cast<float*>(p.out) + orow * p.out_row_stride + col;
            reinterpret_cast<uint4*>(o)[0] = make_uint4(outb[0], outb[1], outb[2], outb[3]);
            reinterpret_cast<uint4*>(o)[1] = make_uint4(outb[4], outb[5], outb[6], outb[7]);
        } else {
            uint32_t hb[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t u = outb[i];
                if (kSum) u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest even
                hb[i] = u >> 16;
            }
            uint16_t* o = reinterpret_cast<uint16_t*>(p.out) + orow * p.out_row_stride + col;
            *reinterpret_cast<uint4*>(o) = make_uint4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16),
                                                      hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16));
        }
    }
}

}  // namespace fb4
