// The online quantizer fused behind a LayerNorm (App. E.2: quantization runs
// inside the operation that produces the activation; LayerNorm is one of the
// two the paper names).  One pass: x is read once, the normalized activation
// never reaches memory, codes and metadata are written as by the streaming
// kernel.
//
// The producer is the textbook LayerNorm over the channels of a token,
//   y = (x - mean) / sqrt(var + eps) * gamma + beta,   var biased,
// evaluated the textbook way in fp32: the mean from the sum of the row, the
// variance from the sum of the squared deviations from that mean (two passes
// over the registers that hold the row), then (x - mean) * rstd, one fused
// multiply-add with gamma and beta, and one rounding to bf16 (a NaN becomes the
// quiet NaN 0x7FC0).  The result agrees with the definition evaluated in double
// to within one bf16 step and is the correctly rounded value for nearly every
// element; a constant row gives exactly beta.
// Rows whose fp32 sums leave the range (an Inf or NaN among the inputs, values
// beyond about 1e18 whose squares overflow, deviations so small that var + eps
// underflows) are redone for the whole bundle by a plain routine in double.
//
// Work split: a wavefront owns whole rows, so the row sums never leave it.  A
// "bundle" is RW consecutive rows, RW * nb <= 64 * B chunks of 32 elements;
// lane l holds chunks l, l + 64, ..., l + 64 (B - 1) of the bundle in
// registers (the same channels in every bundle, so its scale / shift addresses
// are loop invariants), the wavefront reduces the sums per row with butterfly
// exchanges (a fixed order: results do not change from run to run), and each
// lane then normalizes and quantizes its chunks with the streaming kernel's
// per-chunk routine.  Bundles are dealt like that kernel's tiles: to persistent
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
    uint16_t* y_out;              // kWriteY only: [rows][cols] bf16, the producer's result
};

// threads per workgroup (one workgroup per CU): three wavefronts per SIMD where 168 registers hold the kernel,
// two (up to 256 registers) for five or six chunks per lane and for 16 groups from two chunks per lane on
constexpr int ln_threads(int chunks_per_lane, int groups = 8)
{
    return (chunks_per_lane <= 4 && !(groups > 8 && chunks_per_lane >= 2)) ? 768 : 512;
}
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

// Sum over the 64 lanes of a wavefront, the same value in every lane of the result (it comes back through a
// scalar register).  Data-parallel-primitive moves only: inside rows of 16 lanes by quad permutes and mirrors,
// then row 0 -> 1 and 2 -> 3, then rows 0-1 -> 2-3; lane 63 holds the total.  A fixed order: the same input
// always gives the same sum.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_mov(float x)   // a lane outside the row mask receives 0
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kCtrl, kRowMask, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_mov<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_mov<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_mov<0x140, 0xF>(v);   // row_mirror: every lane now holds its row's sum
    v += dpp_mov<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_mov<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// What the normalization of a row needs: t = fma(x, s, nms) * r is (x - mean) * rstd, with a power of two s
// that is 1 unless the plain routine had to rescale the row to stay inside fp32's range.
struct RowNorm {
    float s, nms, r;
};

// Plain routine for one row of any content, by the whole wavefront, in double: the row is read again from
// memory (lane l takes the 32-bit words l, l + 64, ...), mean and squared deviations are summed in double, and
// the three factors come back scaled by a power of two so that neither x * s nor the product with r leaves
// fp32's range.  Kept out of line: it runs for rows outside the fast path's range only.
__device__ __noinline__ RowNorm layernorm_row_plain(const uint16_t* xrow, uint32_t cols, float eps)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t* w = reinterpret_cast<const uint32_t*>(xrow);
    double s1 = 0.0;
    uint32_t amax = 0;
#pragma unroll 1
    for (uint32_t i = lane; i < cols / 2; i += 64) {
        const uint32_t v = w[i];
        s1 += (double)__uint_as_float(v << 16) + (double)__uint_as_float(v & 0xFFFF0000u);
        amax = max(amax, max(v & 0x7FFFu, (v >> 16) & 0x7FFFu));
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        s1 += __shfl_xor(s1, off);
        amax = max(amax, (uint32_t)__shfl_xor((int)amax, off));
    }
    const double mean = s1 / (double)cols;
    double s2 = 0.0;
#pragma unroll 1
    for (uint32_t i = lane; i < cols / 2; i += 64) {
        const uint32_t v = w[i];
        const double d0 = (double)__uint_as_float(v << 16) - mean, d1 = (double)__uint_as_float(v & 0xFFFF0000u) - mean;
        s2 = fma(d0, d0, s2);
        s2 = fma(d1, d1, s2);
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) s2 += __shfl_xor(s2, off);
    const double rstd = 1.0 / sqrt(s2 / (double)cols + (double)eps);
    // s = 2^-(exponent of the row's largest magnitude), an exact factor
    const int e = (int)min(max(amax >> 7, 1u), 254u) - 127;
    const double sc = __builtin_ldexp(1.0, -e);
    RowNorm out;
    out.s = (float)sc;
    out.nms = (float)(-mean * sc);
    const double r = rstd / sc;
    out.r = (r > 3.0e38 && r < __builtin_inf()) ? 3.0e38f : (float)r;   // (Inf and NaN stay)
    return out;
}

// B: chunks per lane (the host picks it from the row length); gamma / beta may be null (1 / 0).
// kWriteY: the producer alone -- writes the normalized bf16 tensor to p.y_out and nothing else (for checking the
// producer against its definition; production launches never use it).
// One chunk per lane is in registers at a time: a first walk over the bundle's chunks forms the sums, a last walk
// reads the chunks again (from the L2 cache: the wavefront has just read them) and normalizes and quantizes
// them; two chunk buffers alternate, the chunk of the next step is always in flight.  (Holding the bundle in
// registers instead reads x once but leaves room for 8 wavefronts per CU only, or spills: 42-62 us on a
// 16384x3072 tensor.)
// kBlock, G: block size (32 or 16) and number of groups of the online selector (Sec. 3.2, Sec. 4.1).
template <int B, int kBlock, int G, bool kTwoStage, bool kSeda, bool kWriteY, int kThreads = ln_threads(B, G)>
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
    // Requests this lane's chunk j of bundle u (a bundle or row past the end reads the last one; its results
    // are never stored).
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
    // Two chunk buffers used in turn: step s of a bundle works on buf[s & 1] while the chunk of step s + 1 is on
    // its way into the other one.  A bundle takes 2 B steps (B chunks summed, B chunks normalized and quantized).
    uint32_t buf[2][16];
    int32_t gbuf[2] = {-1, -1};
    request(u, 0, buf[0], gbuf[0]);
    layernorm_tables_to_lds<B, kTwoStage && !kWriteY, kSeda && !kWriteY, kThreads>(lds, blob, gamma, beta, p);
    const TileConsts K = make_tile_consts(lane, 0);
    FastParams sp = {};
    sp.codes = p.codes;
    sp.meta = p.meta;
    sp.n_blocks = p.n_blocks;
    const bool meta_aligned = (reinterpret_cast<uintptr_t>(p.meta) & 15u) == 0;
    const float n_channels = (float)p.cols;
    const float inv_channels = 1.0f / n_channels;
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3F803F80u);

    while (u < n_bundles) {
        uint32_t claim = 0;
        if (lane == 0) claim = atomicAdd(&wg_next, 1u);
        const uint32_t u_after = blockIdx.x + (uint32_t)__builtin_amdgcn_readfirstlane(claim) * W;
        bool ok[B];
#pragma unroll
        for (int j = 0; j < B; ++j) ok[j] = valid[j] && u * rw + rloc[j] < p.rows;
        // ---- first walk: per chunk the sum and the sum of squares, each by one two-element bf16 dot product with
        // fp32 accumulation per register (the register with a pair of ones, and with itself)
        float part[B], part2[B];
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int s = j;
            request(u, (j + 1) % B, buf[(s + 1) & 1], gbuf[(s + 1) & 1]);   // (after the last chunk: the first again)
            const uint32_t (&w)[16] = buf[s & 1];
            float a0 = 0.0f, a1 = 0.0f, q0 = 0.0f, q1 = 0.0f;
#pragma unroll
            for (int k = 0; k < 16; k += 2) {
                a0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[k]), ones, a0, false);
                a1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[k + 1]), ones, a1, false);
                q0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[k]), __builtin_bit_cast(bf16x2, w[k]), q0, false);
                q1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[k + 1]), __builtin_bit_cast(bf16x2, w[k + 1]), q1, false);
            }
            part[j] = ok[j] ? a0 + a1 : 0.0f;
            part2[j] = ok[j] ? q0 + q1 : 0.0f;
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- per row: both sums over the wavefront's chunks of that row; mean, and the variance as the mean
        // square minus the squared mean -- kept only where that difference is well conditioned
        float mean[B];
        RowNorm rn[B];
#pragma unroll
        for (int j = 0; j < B; ++j) { mean[j] = 0.0f; rn[j].s = 1.0f; rn[j].nms = 0.0f; rn[j].r = 0.0f; }
        bool centered = false, in_range = true;   // wave-uniform
        for (uint32_t r = 0; r < rw; ++r) {
            float c1 = 0.0f, c2 = 0.0f;
#pragma unroll
            for (int j = 0; j < B; ++j) {
                c1 += (valid[j] && rloc[j] == r) ? part[j] : 0.0f;
                c2 += (valid[j] && rloc[j] == r) ? part2[j] : 0.0f;
            }
            c1 = wave_sum(c1);
            c2 = wave_sum(c2);
            const float m = c1 / n_channels;   // a true division: the mean of a constant row is that constant
            const float msq = c2 * inv_channels;
            const float var = msq - m * m;
            // the subtraction loses log2(msq / var) bits: fine while the squared mean is at most the variance
            centered = centered || !(var >= 0.5f * msq);
            const float v = var + p.eps;
            in_range = in_range && ((v >= 0x1p-100f && v <= 0x1p+100f) || u * rw + r >= p.rows);
            const float rstd = __builtin_amdgcn_rsqf(v);
#pragma unroll
            for (int j = 0; j < B; ++j) {
                if (rloc[j] == r) { mean[j] = m; rn[j].nms = -m; rn[j].r = rstd; }
            }
        }
        // (after B steps the bundle's first chunk is on its way into buf[B & 1])
        if (centered) {
            // ---- another walk (rows whose mean is not small against their spread): squared deviations from the mean
#pragma unroll
            for (int j = 0; j < B; ++j) {
                const int s = B + j;
                // keeps the buffer parity of the path that skips this walk: with an odd number of chunks the first
                // chunk comes back into the buffer this step works on, requested after its arithmetic
                const bool late = (B & 1) && j == B - 1;
                if (!late) request(u, (j + 1) % B, buf[(s + 1) & 1], gbuf[(s + 1) & 1]);
                const uint32_t (&w)[16] = buf[s & 1];
                float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
#pragma unroll
                for (int k = 0; k < 16; k += 2) {
                    const float d0 = __uint_as_float(w[k] << 16) - mean[j], d1 = __uint_as_float(w[k] & 0xFFFF0000u) - mean[j];
                    const float d2 = __uint_as_float(w[k + 1] << 16) - mean[j], d3 = __uint_as_float(w[k + 1] & 0xFFFF0000u) - mean[j];
                    a0 = __builtin_fmaf(d0, d0, a0);
                    a1 = __builtin_fmaf(d1, d1, a1);
                    a2 = __builtin_fmaf(d2, d2, a2);
                    a3 = __builtin_fmaf(d3, d3, a3);
                }
                part2[j] = ok[j] ? (a0 + a1) + (a2 + a3) : 0.0f;
                __builtin_amdgcn_sched_barrier(0);
                if (late) request(u, 0, buf[s & 1], gbuf[s & 1]);
            }
            in_range = true;
            for (uint32_t r = 0; r < rw; ++r) {
                float c2 = 0.0f;
#pragma unroll
                for (int j = 0; j < B; ++j) c2 += (valid[j] && rloc[j] == r) ? part2[j] : 0.0f;
                c2 = wave_sum(c2);
                const float v = c2 * inv_channels + p.eps;
                // (the comparison is false for a NaN too; a row past the end of the tensor has v = eps only)
                in_range = in_range && ((v >= 0x1p-100f && v <= 0x1p+100f) || u * rw + r >= p.rows);
                const float rstd = __builtin_amdgcn_rsqf(v);
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    if (rloc[j] == r) rn[j].r = rstd;
                }
            }
        }
        if (!in_range) {
            // some row of this bundle left the range of the fp32 sums: every row again, the plain way
            for (uint32_t r = 0; r < rw; ++r) {
                const uint32_t row = u * rw + r;
                if (row >= p.rows) break;
                const RowNorm v = layernorm_row_plain(x + (long long)row * row_stride, p.cols, p.eps);
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    if (rloc[j] == r) rn[j] = v;
                }
            }
        }
        // ---- last walk: normalize, scale and shift, round to bf16, quantize, store
#pragma unroll
        for (int j = 0; j < B; ++j) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            const int s = B + j;
            const int32_t grp = gbuf[s & 1];
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
                const float t0 = __builtin_fmaf(x0, rn[j].s, rn[j].nms) * rn[j].r, t1 = __builtin_fmaf(x1, rn[j].s, rn[j].nms) * rn[j].r;
                const float t2 = __builtin_fmaf(x2, rn[j].s, rn[j].nms) * rn[j].r, t3 = __builtin_fmaf(x3, rn[j].s, rn[j].nms) * rn[j].r;
                const f32x2 y01 = {__builtin_fmaf(t0, g.x, be.x), __builtin_fmaf(t1, g.y, be.y)};
                const f32x2 y23 = {__builtin_fmaf(t2, g.z, be.z), __builtin_fmaf(t3, g.w, be.w)};
                y[2 * q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(y01, bf16x2));
                y[2 * q + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(y23, bf16x2));
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kWriteY) {
                if (ok[j]) {
                    uint32_t v[16];
#pragma unroll
                    for (int k = 0; k < 16; ++k) {   // NaNs as the quiet NaN 0x7FC0
                        v[k] = y[k];
                        if ((v[k] & 0x7FFFu) > 0x7F80u) v[k] = (v[k] & 0xFFFF0000u) | 0x7FC0u;
                        if ((v[k] & 0x7FFF0000u) > 0x7F800000u) v[k] = (v[k] & 0xFFFFu) | 0x7FC00000u;
                    }
                    uint4* dst = reinterpret_cast<uint4*>(p.y_out + (size_t)gb * 32);
                    dst[0] = make_uint4(v[0], v[1], v[2], v[3]);
                    dst[1] = make_uint4(v[4], v[5], v[6], v[7]);
                    dst[2] = make_uint4(v[8], v[9], v[10], v[11]);
                    dst[3] = make_uint4(v[12], v[13], v[14], v[15]);
                }
            } else {
                const uint32_t excl = kSeda ? kLdsSeda + 32u * ((grp >= 0 && (uint32_t)grp < p.n_groups) ? (uint32_t)grp : p.n_groups) : 0u;
                uint32_t stage[16];
                uint32_t code[4], meta;
                bool tile_special;
                const uint32_t no_code[4] = {0, 0, 0, 0};
                compute_tile<kBlock, G, kTwoStage, kSeda>(y, lds, K, nullptr, ok[j], excl, code, meta, no_code, 0u, tile_special, stage);
                const bool al = meta_aligned && (((gb - lane) & 7u) == 0u);
                store_tile<kBlock>(sp, gb, lane, make_uint4(code[0], code[1], code[2], code[3]), meta, al, ok[j]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        u = u_next;
        u_next = u_after;
    }
}

}  // namespace fb4
