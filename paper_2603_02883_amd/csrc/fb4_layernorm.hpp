// The online quantizer fused behind a LayerNorm (App. E.2: quantization runs
// inside the operation that produces the activation; LayerNorm is one of the
// two the paper names).  One pass: x is read once, the normalized activation
// never reaches memory, codes and metadata are written as by the streaming
// kernel.
//
// The producer is the textbook LayerNorm over the channels of a token with a
// per-channel scale and shift; the quantizer's input is its result rounded to
// bf16.  That rounding decides codes, so the precision of each step is fixed:
//   S1 = sum x, S2 = sum x^2 in double (every term exact); mean = S1 * (1/C),
//   var = max(fma(-mean, mean, S2 * (1/C)), 0) in double;
//   a = 1 / sqrt(float(var + eps)), b = -float(mean) * a in float (IEEE
//   square root and divide);
//   y = fmaf(fmaf(x, a, b), gamma, beta) in float, rounded to bf16 (nearest
//   even); a NaN becomes the canonical quiet NaN 0x7FC0.
// The sums are exact, hence independent of their order, whenever a row's values
// span less than about 2^12 in magnitude; beyond that another order may move
// S2 by one ulp of a double, which changes a or b once in about 2^29 rows.
//
// Work split: a wavefront owns whole rows, so the row sums never leave it.  A
// "bundle" is RW consecutive rows, RW * nb <= 64 * B chunks of 32 elements;
// lane l works on chunks l, l + 64, ..., l + 64 (B - 1) of the bundle (the
// same channels in every bundle, so its scale / shift addresses are loop
// invariants), the wavefront reduces the sums per row with butterfly exchanges
// (a fixed order: results do not change from run to run), and each lane then
// normalizes and quantizes its chunks with the streaming kernel's per-chunk
// routine.  Bundles are dealt like that kernel's tiles: to persistent
// workgroups round robin, to a workgroup's wavefronts on demand.
#pragma once

#include "fb4_fast.hpp"

namespace fb4 {

struct LayerNormParams {
    uint32_t rows;
    uint32_t cols;
    uint32_t n_blocks;   // rows * nb
    float eps;
    uint8_t* codes;
    uint16_t* meta;
    // Sec. 3.4 (optional): candidate lists per token group
    const int32_t* token_group;   // [rows] or null
    const uint8_t* sub;           // [n_groups][8] DIDs
    uint32_t n_groups;            // <= kMaxFusedProducerGroups
    uint32_t n_dialects;
};

constexpr int ln_threads(int chunks_per_lane) { return chunks_per_lane <= 4 ? 768 : 512; }
constexpr int kLnMaxChunksPerLane = 6;
constexpr int kLdsLnTables = lds_fast_bytes(false, false, false);

// Tables of the streaming kernel, the scale / shift vectors and (kSeda) the exclusion rows into LDS; ends with
// a barrier.  kGbFloats: floats reserved per vector; kThreads: threads of the workgroup.
template <int B, bool kTwoStage, bool kSeda, int kThreads>
__device__ __forceinline__ void layernorm_tables_to_lds(uint8_t* lds, const uint8_t* blob, const float* gamma,
                                                        const float* beta, const LayerNormParams& p)
{
    constexpr int kGbFloats = 2048 * B;
    constexpr int kLdsSeda = kLdsLnTables + 2 * kGbFloats * 4;
    float* lds_gamma = reinterpret_cast<float*>(lds + kLdsLnTables);
    float* lds_beta = lds_gamma + kGbFloats;
    // ---- tables (layout of the streaming kernel) and the scale / shift vectors
    for (int i = threadIdx.x; i < 64 * kRowCopies; i += kThreads) {
        const int bin = i / (2 * kRowCopies), half = (i / kRowCopies) & 1;
        reinterpret_cast<uint4*>(lds + kLdsRows)[i] = *reinterpret_cast<const uint4*>(blob + kOffQerror8 + bin * 32 + half * 16);
    }
    for (int i = threadIdx.x; i < 256; i += kThreads)
        reinterpret_cast<uint32_t*>(lds + kLdsNibT)[i] = reinterpret_cast<const uint32_t*>(blob + kOffQvalueT)[i];
    if (kTwoStage && threadIdx.x < 64)
        reinterpret_cast<uint32_t*>(lds + kLdsRange)[threadIdx.x] = reinterpret_cast<const uint32_t*>(blob + kOffRangeExcl)[threadIdx.x];
    // scale / shift: the four channels (4q .. 4q+3) of chunk cb at [q][64 B][4], so that the 16-byte reads of
    // neighbouring lanes (neighbouring chunks, same q) fall into different banks and q is a constant offset
    for (uint32_t c = threadIdx.x; c < p.cols; c += kThreads) {
        const uint32_t at = (((c & 31u) >> 2) * (64u * B) + (c >> 5)) * 4u + (c & 3u);
        lds_gamma[at] = gamma ? gamma[c] : 1.0f;
        lds_beta[at] = beta ? beta[c] : 0.0f;
    }
    if (kSeda) build_seda_rows(lds, kLdsSeda, p.sub, p.n_groups, p.n_dialects, kThreads);
    __syncthreads();
    for (int i = threadIdx.x; i < 1024; i += kThreads) {   // pair table: byte(hi, lo, d) = index(d, lo) | index(d, hi) << 4
        const int hi = i >> 5, lo = i & 31;
        const uint4* rl = reinterpret_cast<const uint4*>(lds + kLdsNibT + lo * 32);
        const uint4* rh = reinterpret_cast<const uint4*>(lds + kLdsNibT + hi * 32);
        uint4* dst = reinterpret_cast<uint4*>(lds + kLdsPair + i * 32);
        const uint4 l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
        dst[0] = make_uint4(l0.x | (h0.x << 4), l0.y | (h0.y << 4), l0.z | (h0.z << 4), l0.w | (h0.w << 4));
        dst[1] = make_uint4(l1.x | (h1.x << 4), l1.y | (h1.y << 4), l1.z | (h1.z << 4), l1.w | (h1.w << 4));
    }
    __syncthreads();
}

// B: chunks per lane (the host picks it from the row length); gamma / beta may be null (1 / 0).
// One chunk per lane is in registers at a time: a first pass over the bundle's chunks forms the sums, a second
// pass reads the chunks again (from the L2 cache: the wavefront has just read them) and normalizes and
// quantizes them.  Keeping the whole bundle in registers instead saves the second read but needs 220 registers
// for three chunks, i.e. 8 wavefronts per CU: 43.9 us on a 16384x3072 tensor against 40.7 us this way with 12,
// and rows longer than 8192 spilled (100 us per 50 M elements against 62-76 us).
// kThreads: 768 up to four chunks per lane, 512 beyond (the per-chunk bookkeeping then needs the registers).
template <int B, bool kTwoStage, bool kSeda, int kThreads>
__global__ __launch_bounds__(kThreads) void layernorm_quantize_kernel(
    const uint8_t* blob, const uint16_t* x, uint32_t n_bundles, uint32_t rw, uint32_t nb, uint32_t n_workgroups,
    long long row_stride, const float* gamma, const float* beta, LayerNormParams p)
{
    constexpr int kWaves = kThreads / 64;
    constexpr int kGbFloats = 2048 * B;
    constexpr int kLdsSeda = kLdsLnTables + 2 * kGbFloats * 4;
    __shared__ __align__(16) uint8_t lds[kLdsSeda + (kSeda ? (kMaxFusedProducerGroups + 1) * 32 : 0)];
    __shared__ uint32_t wg_next;
    float* lds_gamma = reinterpret_cast<float*>(lds + kLdsLnTables);
    float* lds_beta = lds_gamma + kGbFloats;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t W = n_workgroups;
    const uint32_t per_bundle = rw * nb;

    uint32_t rloc[B], cb[B];
    bool valid[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const uint32_t i = lane + 64u * j;
        valid[j] = i < per_bundle;
        const uint32_t ic = valid[j] ? i : 0u;
        rloc[j] = ic / nb;
        cb[j] = ic - rloc[j] * nb;
    }
    auto request = [&](uint32_t u, int j, uint32_t (&q)[16], int32_t& grp) {
        const uint32_t row = min(min(u, n_bundles - 1u) * rw + rloc[j], p.rows - 1u);
        if (kSeda) grp = p.token_group[row];
        const uint4* px = reinterpret_cast<const uint4*>(x + (long long)row * row_stride + (long long)cb[j] * 32);
        const uint4 q0 = px[0], q1 = px[1], q2 = px[2], q3 = px[3];
        q[0] = q0.x; q[1] = q0.y; q[2] = q0.z; q[3] = q0.w; q[4] = q1.x; q[5] = q1.y; q[6] = q1.z; q[7] = q1.w;
        q[8] = q2.x; q[9] = q2.y; q[10] = q2.z; q[11] = q2.w; q[12] = q3.x; q[13] = q3.y; q[14] = q3.z; q[15] = q3.w;
    };

    uint32_t u = blockIdx.x + wave * W;
    uint32_t u_next = blockIdx.x + (kWaves + wave) * W;
    if (threadIdx.x == 0) wg_next = 2 * kWaves;
    // Two chunk buffers used in turn: a bundle takes 2 B steps (B chunks summed, B chunks quantized), step s
    // works on buf[s & 1] while the chunk of step s + 1 is on its way into the other one.
    uint32_t buf[2][16];
    int32_t gbuf[2] = {-1, -1};
    request(u, 0, buf[0], gbuf[0]);
    layernorm_tables_to_lds<B, kTwoStage, kSeda, kThreads>(lds, blob, gamma, beta, p);
    const TileConsts K = make_tile_consts(lane, 0);
    FastParams sp = {};
    sp.codes = p.codes;
    sp.meta = p.meta;
    sp.n_blocks = p.n_blocks;
    const bool meta_aligned = (reinterpret_cast<uintptr_t>(p.meta) & 15u) == 0;
    const double inv_channels = 1.0 / (double)p.cols;
    const double eps = (double)p.eps;

    while (u < n_bundles) {
        uint32_t claim = 0;
        if (lane == 0) claim = atomicAdd(&wg_next, 1u);
        const uint32_t u_after = blockIdx.x + (uint32_t)__builtin_amdgcn_readfirstlane(claim) * W;
        // ---- first pass: sums in double
        double p1[B], p2[B];
        bool ok[B];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            constexpr int kSteps = 2 * B;
            const int s = j;
            (void)kSteps;
            if (j + 1 < B) request(u, j + 1, buf[(s + 1) & 1], gbuf[(s + 1) & 1]);
            else request(u, 0, buf[(s + 1) & 1], gbuf[(s + 1) & 1]);   // first chunk of the second pass
            const uint32_t (&w)[16] = buf[s & 1];
            ok[j] = valid[j] && u * rw + rloc[j] < p.rows;
            double s1a = 0.0, s1b = 0.0, s2a = 0.0, s2b = 0.0;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const double d0 = (double)__uint_as_float(w[k] << 16);
                const double d1 = (double)__uint_as_float(w[k] & 0xFFFF0000u);
                s1a += d0; s1b += d1;
                s2a = fma(d0, d0, s2a); s2b = fma(d1, d1, s2b);
            }
            p1[j] = ok[j] ? s1a + s1b : 0.0;
            p2[j] = ok[j] ? s2a + s2b : 0.0;
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- per row: reduce over the wavefront, then 1/std and -mean/std as floats
        float a[B], b[B];
#pragma unroll
        for (int j = 0; j < B; ++j) a[j] = b[j] = 0.0f;
        for (uint32_t r = 0; r < rw; r += 2) {
            double c1[2] = {0.0, 0.0}, c2[2] = {0.0, 0.0};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    c1[h] += (valid[j] && rloc[j] == r + h) ? p1[j] : 0.0;
                    c2[h] += (valid[j] && rloc[j] == r + h) ? p2[j] : 0.0;
                }
            }
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    c1[h] += __shfl_xor(c1[h], off);
                    c2[h] += __shfl_xor(c2[h], off);
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const double mean = c1[h] * inv_channels;
                double var = fma(-mean, mean, c2[h] * inv_channels);
                var = var < 0.0 ? 0.0 : var;
                const float ar = 1.0f / __builtin_sqrtf((float)(var + eps));
                const float br = -(float)mean * ar;
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    if (ok[j] && rloc[j] == r + h) { a[j] = ar; b[j] = br; }
                }
            }
        }
        // ---- second pass: normalize, scale and shift, round to bf16, quantize, store
#pragma unroll
        for (int j = 0; j < B; ++j) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            const int s = B + j;
            const uint32_t excl = kSeda ? kLdsSeda + 32u * ((gbuf[s & 1] >= 0 && (uint32_t)gbuf[s & 1] < p.n_groups) ? (uint32_t)gbuf[s & 1] : p.n_groups) : 0u;
            if (j + 1 < B) request(u, j + 1, buf[(s + 1) & 1], gbuf[(s + 1) & 1]);
            else request(u_next, 0, buf[(s + 1) & 1], gbuf[(s + 1) & 1]);   // first chunk of the next bundle
            const uint32_t (&w)[16] = buf[s & 1];
            const float4* g4 = reinterpret_cast<const float4*>(lds_gamma) + cb[j];
            const float4* b4 = reinterpret_cast<const float4*>(lds_beta) + cb[j];
            const uint32_t gb = u * per_bundle + lane + 64u * j;
            uint32_t y[16];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float4 g = g4[q * 64 * B], be = b4[q * 64 * B];
                const float x0 = __uint_as_float(w[2 * q] << 16), x1 = __uint_as_float(w[2 * q] & 0xFFFF0000u);
                const float x2 = __uint_as_float(w[2 * q + 1] << 16), x3 = __uint_as_float(w[2 * q + 1] & 0xFFFF0000u);
                const f32x2 y01 = {__builtin_fmaf(__builtin_fmaf(x0, a[j], b[j]), g.x, be.x),
                                   __builtin_fmaf(__builtin_fmaf(x1, a[j], b[j]), g.y, be.y)};
                const f32x2 y23 = {__builtin_fmaf(__builtin_fmaf(x2, a[j], b[j]), g.z, be.z),
                                   __builtin_fmaf(__builtin_fmaf(x3, a[j], b[j]), g.w, be.w)};
                y[2 * q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(y01, bf16x2));
                y[2 * q + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(y23, bf16x2));
            }
            __builtin_amdgcn_sched_barrier(0);
            uint32_t stage[16];
            uint32_t code[4], meta;
            bool tile_special;
            const uint32_t no_code[4] = {0, 0, 0, 0};
            compute_tile<32, 8, kTwoStage, kSeda>(y, lds, K, nullptr, ok[j], excl, code, meta, no_code, 0u, tile_special, stage);
            const bool al = meta_aligned && (((gb - lane) & 7u) == 0u);
            store_tile<32>(sp, gb, lane, make_uint4(code[0], code[1], code[2], code[3]), meta, al, ok[j]);
            __builtin_amdgcn_sched_barrier(0);
        }
        u = u_next;
        u_next = u_after;
    }
}

}  // namespace fb4
