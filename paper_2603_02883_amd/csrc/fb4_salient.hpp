// Attention-guided salient tokens (Sec. 3.3, App. F): the rows that the
// activation decomposition gives a second plane are, per tile of tokens, the one
// whose query attends most strongly on average -- the mean over the keys of
// its attention group of |Q.K^T| (spatial / 3D attention) or max(Q.K^T, 0)
// (temporal attention), pre-softmax.
//
// attention_scores_kernel: the one dense contraction of this library, on the
// matrix cores.  A workgroup of four wavefronts takes 256 queries of one group;
// every wavefront keeps its 64 queries as B operands in registers for the whole
// pass and walks over the group's keys 64 at a time: the key block goes through
// LDS once for the four wavefronts (rows padded by 16 bytes so that the 16-byte
// operand reads of the 16 lanes of a pass fall into 16 different bank groups),
// each step is a 32x32x16 bf16 MFMA with fp32 accumulation computing S^T = K Q^T -- transposed
// so that a lane's 16 accumulators are 16 keys of ONE query: |.| or max(., 0)
// and the sum over keys then stay inside the lane, and the two half-wavefronts
// are only added up once at the very end.
//
// select_salient_kernel: per frame the head mean (in double, head by head), the
// best token of every tile (lowest index on ties, a NaN never wins), and the
// chosen tokens as ascending row numbers of the [frames * tokens] tensor.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fb4 {

typedef __bf16 mfma_bf16x8 __attribute__((ext_vector_type(8)));
typedef float mfma_f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t lds_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kScoreThreads = 256;

// Workgroups are dealt to the eight XCDs in turn, and each XCD has its own L2.  The workgroups of one attention
// group read the same keys, so they should share an L2: workgroup b works on position (b % 8) * (n / 8) + b / 8
// of the launch, which puts consecutive positions on one XCD (the last n % 8 workgroups keep their own number).
__device__ __forceinline__ uint32_t xcd_local_position(uint32_t b, uint32_t n)
{
    const uint32_t chunk = n / 8u;
    return b < chunk * 8u ? (b % 8u) * chunk + b / 8u : b;
}
// Two shapes of the kernel: 64 queries per wavefront and 64 keys per barrier for long groups (spatial / 3D
// attention), 32 and 32 for short ones (temporal attention: a group is a handful of frames).
constexpr uint32_t kScoreShortGroup = 64;   // tokens up to which the small shape is used

// D32: channels / 32, rounded up (channels beyond `dim` are zero on both sides).  kRelu: max(., 0), else |.|.
// kScoreQB: blocks of 32 queries per wavefront; kScoreKeys: keys per barrier (a multiple of 32).
template <int D32, bool kRelu, int kScoreQB, int kScoreKeys>
__global__ __launch_bounds__(kScoreThreads) void attention_scores_kernel(const uint16_t* q, const uint16_t* k,
                                                                         uint32_t tokens, uint32_t dim,
                                                                         uint32_t blocks_per_group, float* scores)
{
    constexpr int kScoreQueries = 128 * kScoreQB;    // per workgroup
    constexpr int kSteps = D32 * 2;                  // MFMA steps of 16 channels
    constexpr int kRowBytes = D32 * 64 + 16;         // one key row in LDS: channels, then 16 bytes of padding
    __shared__ __align__(16) uint8_t lds[2][kScoreKeys * kRowBytes];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t pos = xcd_local_position(blockIdx.x, gridDim.x);
    const uint32_t g = pos / blocks_per_group;
    const uint32_t q0 = (pos - g * blocks_per_group) * kScoreQueries + wave * (32u * kScoreQB);
    const uint16_t* qg = q + (size_t)g * tokens * dim;
    const uint16_t* kg = k + (size_t)g * tokens * dim;
    const uint32_t half = lane >> 5, col = lane & 31u;

    // ---- this wavefront's queries as B operands: lane holds query q0 + lane % 32, channels 16 s + 8 (lane / 32) ..
    // (a query past the end reads the last one; a channel past `dim` is zero)
    mfma_bf16x8 qf[kScoreQB][kSteps];
#pragma unroll
    for (int b = 0; b < kScoreQB; ++b) {
        const uint16_t* row = qg + (size_t)min(q0 + 32u * b + col, tokens - 1u) * dim;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const uint32_t c = 16u * s + 8u * half;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (c + 8u <= dim) v = *reinterpret_cast<const uint4*>(row + c);   // dim is a multiple of 8
            qf[b][s] = __builtin_bit_cast(mfma_bf16x8, v);
        }
    }
    // ---- key blocks: 32 keys x dim channels; thread t stages 16-byte pieces t, t + 256, ...
    constexpr int kPiecesPerRow = D32 * 4;           // 16-byte pieces of a padded row's channel part
    constexpr int kPieces = kScoreKeys * kPiecesPerRow;
    constexpr int kPerThread = (kPieces + kScoreThreads - 1) / kScoreThreads;
    uint4 stage[kPerThread];
    auto fetch = [&](uint32_t kb) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const uint32_t piece = threadIdx.x + i * kScoreThreads;
            const uint32_t r = piece / kPiecesPerRow, c8 = (piece - r * kPiecesPerRow) * 8u;   // key row, first channel
            const uint32_t key = kb * kScoreKeys + r;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (piece < (uint32_t)kPieces && key < tokens && c8 + 8u <= dim)
                v = *reinterpret_cast<const uint4*>(kg + (size_t)key * dim + c8);
            stage[i] = v;
        }
    };
    auto deposit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const uint32_t piece = threadIdx.x + i * kScoreThreads;
            const uint32_t r = piece / kPiecesPerRow, cb = (piece - r * kPiecesPerRow) * 16u;
            if (piece < (uint32_t)kPieces) {
                *reinterpret_cast<uint4*>(&lds[buf][r * kRowBytes + cb]) = stage[i];
            }
        }
    };
    const uint32_t n_kb = (tokens + kScoreKeys - 1) / kScoreKeys;
    fetch(0);
    deposit(0);
    __syncthreads();
    float sum[kScoreQB];   // over this lane's keys of f(S[query][key])
#pragma unroll
    for (int b = 0; b < kScoreQB; ++b) sum[b] = 0.0f;
    for (uint32_t kb = 0; kb < n_kb; ++kb) {
        const int buf = kb & 1;
        if (kb + 1 < n_kb) fetch(kb + 1);
#pragma unroll
        for (int kk = 0; kk < kScoreKeys / 32; ++kk) {   // 32 keys at a time
            mfma_f32x16 acc[kScoreQB];
#pragma unroll
            for (int b = 0; b < kScoreQB; ++b) acc[b] = mfma_f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                // A operand: key row lane % 32 of the 32 keys, channels 16 s + 8 (lane / 32) ..; one read feeds the
                // MFMAs of all the wavefront's query blocks (with one block per read the kernel is bound by LDS bandwidth)
                const uint4 a = *reinterpret_cast<const uint4*>(&lds[buf][(kk * 32 + col) * kRowBytes + s * 32 + half * 16]);
#pragma unroll
                for (int b = 0; b < kScoreQB; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mfma_bf16x8, a), qf[b][s], acc[b], 0, 0, 0);
            }
#pragma unroll
            for (int b = 0; b < kScoreQB; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sum[b] += kRelu ? fmaxf(acc[b][r], 0.0f) : fabsf(acc[b][r]);
            }
        }
        if (kb + 1 < n_kb) deposit(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int b = 0; b < kScoreQB; ++b) {
        const float total = sum[b] + __shfl_xor(sum[b], 32);   // the two half-wavefronts hold different keys of the same query
        const uint32_t qi = q0 + 32u * b + col;
        if (half == 0 && qi < tokens) scores[(size_t)g * tokens + qi] = total / (float)tokens;
    }
}

// The same scores for groups whose rows are exactly 128 channels and whose tokens are a multiple of 128: four blocks
// of 32 queries per wavefront, so that one 16-byte operand read from LDS feeds four MFMAs (the kernel above feeds
// two and is bound by that LDS traffic).  128 queries x 128 channels of B operands and four accumulator blocks
// need about 220 registers; to keep two wavefronts per SIMD beside them, key blocks are not staged through
// registers: `global_load_lds_dwordx4` writes a wavefront's 64 x 16 bytes straight into LDS.  Those 1 KiB land
// contiguously, so rows cannot be padded; instead piece p (16 bytes) of key row r sits at position p ^ (r % 16) of
// the row (the load fetches the matching piece of global memory), which spreads the 16 rows that the lanes of one
// LDS pass read over all 64 banks.
// A workgroup of four wavefronts takes 256 queries: wavefront w holds queries 128 (w % 2) .. and walks the keys of
// half w / 2 of the group, 64 per barrier, from that half's own double-buffered LDS region; the two halves' sums
// meet in LDS at the end (always half 0 + half 1).
constexpr int kDmaQB = 4;                  // blocks of 32 queries per wavefront
constexpr int kDmaQueries = 2 * 32 * kDmaQB;   // per workgroup
constexpr int kDmaKeys = 64;               // per barrier and half
constexpr int kDmaDim = 128;
constexpr uint32_t kDmaBlockBytes = kDmaKeys * kDmaDim * 2;   // 16 KiB

template <bool kRelu>
__global__ __launch_bounds__(kScoreThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attention_scores_dma_kernel(const uint16_t* q, const uint16_t* k, uint32_t tokens, uint32_t blocks_per_group,
                                 float* scores)
{
    constexpr int kSteps = kDmaDim / 16;
    // Two buffers per key half, as two arrays: the compiler then sees that the loads into one do not touch the
    // operand reads from the other and does not wait for them.
    __shared__ __align__(1024) uint8_t lds_a[2 * kDmaBlockBytes];   // [half], even key blocks
    __shared__ __align__(1024) uint8_t lds_b[2 * kDmaBlockBytes];   // [half], odd key blocks
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t qset = wave & 1u, kh = wave >> 1;
    const uint32_t pos = xcd_local_position(blockIdx.x, gridDim.x);
    const uint32_t g = pos / blocks_per_group;
    const uint32_t q0 = (pos - g * blocks_per_group) * kDmaQueries + qset * (32u * kDmaQB);
    const uint16_t* qg = q + (size_t)g * tokens * kDmaDim;
    const uint32_t half_keys = tokens / 2;                       // a multiple of 64
    const uint8_t* kbase = reinterpret_cast<const uint8_t*>(k + ((size_t)g * tokens + (size_t)kh * half_keys) * kDmaDim);
    const uint32_t half = lane >> 5, col = lane & 31u;

    // ---- key blocks: this wavefront loads rows 32 (w % 2) .. + 31 of its half's block, eight loads of four rows
    const uint32_t lrow = lane >> 4, lpos = lane & 15u;          // row within a load, position within the row
    auto fetch = [&](uint32_t kb, uint8_t* buffer) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t row = qset * 32u + 4u * i + lrow;      // key row of the block
            const uint8_t* src = kbase + ((size_t)kb * kDmaKeys + row) * (kDmaDim * 2) + ((lpos ^ (row & 15u)) << 4);
            const uint32_t dst = __builtin_amdgcn_readfirstlane(kh * kDmaBlockBytes + (qset * 32u + 4u * i) * 256u);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(buffer + dst), 16, 0, 0);
        }
    };
    const uint32_t n_kb = half_keys / kDmaKeys;
    fetch(0, lds_a);

    // ---- this wavefront's queries as B operands (a query past the end reads the last one)
    mfma_bf16x8 qf[kDmaQB][kSteps];
#pragma unroll
    for (int b = 0; b < kDmaQB; ++b) {
        const uint16_t* row = qg + (size_t)min(q0 + 32u * b + col, tokens - 1u) * kDmaDim;
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
            qf[b][s] = __builtin_bit_cast(mfma_bf16x8, *reinterpret_cast<const uint4*>(row + 16u * s + 8u * half));
    }
    float sum[kDmaQB];
#pragma unroll
    for (int b = 0; b < kDmaQB; ++b) sum[b] = 0.0f;
    // A operand of step s: key row 32 kk + lane % 32, piece 2 s + lane / 32, swizzled
    const uint32_t a0 = kh * kDmaBlockBytes + col * 256u + (((col & 15u) ^ half) << 4);
    auto compute = [&](const uint8_t* buffer) {
        // the operand of the next step is read while this step's MFMAs run
        uint4 a_next = *reinterpret_cast<const uint4*>(buffer + a0);
#pragma unroll
        for (int kk = 0; kk < kDmaKeys / 32; ++kk) {
            mfma_f32x16 acc[kDmaQB];
#pragma unroll
            for (int b = 0; b < kDmaQB; ++b) acc[b] = mfma_f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                const uint4 a = a_next;
                const int ns = (s + 1) % kSteps, nk = kk + (s + 1) / kSteps;
                if (nk < kDmaKeys / 32)
                    a_next = *reinterpret_cast<const uint4*>(buffer + ((a0 ^ ((uint32_t)ns << 5)) + nk * 32 * 256));
#pragma unroll
                for (int b = 0; b < kDmaQB; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mfma_bf16x8, a), qf[b][s], acc[b], 0, 0, 0);
            }
#pragma unroll
            for (int b = 0; b < kDmaQB; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sum[b] += kRelu ? fmaxf(acc[b][r], 0.0f) : fabsf(acc[b][r]);
            }
        }
    };
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the first block is in LDS
    __syncthreads();
    for (uint32_t kb = 0; kb < n_kb; kb += 2) {
        if (kb + 1 < n_kb) fetch(kb + 1, lds_b);
        compute(lds_a);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // the next block has landed before anyone reads it
        __syncthreads();
        if (kb + 1 < n_kb) {
            if (kb + 2 < n_kb) fetch(kb + 2, lds_a);
            compute(lds_b);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
        }
    }
    // ---- the two key halves meet: half 1 through LDS, then half 0 + half 1
    float* meet = reinterpret_cast<float*>(lds_a);               // [query set][128]
#pragma unroll
    for (int b = 0; b < kDmaQB; ++b) sum[b] += __shfl_xor(sum[b], 32);   // the two half-wavefronts hold different keys
    if (kh == 1 && half == 0) {
#pragma unroll
        for (int b = 0; b < kDmaQB; ++b) meet[qset * 128u + 32u * b + col] = sum[b];
    }
    __syncthreads();
    if (kh == 0 && half == 0) {
#pragma unroll
        for (int b = 0; b < kDmaQB; ++b) {
            const uint32_t qi = q0 + 32u * b + col;
            if (qi < tokens) scores[(size_t)g * tokens + qi] = (sum[b] + meet[qset * 128u + 32u * b + col]) / (float)tokens;
        }
    }
}

// Diagnostic: the rate at which this device sustains v_mfma_f32_32x32x16_bf16 on operands held in registers -- four
// independent accumulator chains per wavefront, no memory traffic inside the loop -- so that the attention
// kernel's rate can be read against what the matrix cores deliver at the clock the power management allows.
// random != 0: operands with random signs and mantissas (magnitudes in [0.5, 2)), as real activations toggle
// the datapath; random == 0: the same bit pattern in every element.
__global__ __launch_bounds__(256) void probe_mfma_rate_kernel(float* out, uint32_t iters, uint32_t random)
{
    auto word = [&](uint32_t i) {
        uint32_t h = (threadIdx.x * 2654435761u + i * 40503u + blockIdx.x) * 2246822519u;
        h ^= h >> 13;
        h *= 3266489917u;
        h ^= h >> 16;
        return random ? ((h & 0x80FF80FFu) | 0x3F003F00u) : 0x3F803F80u;   // two bf16 per word
    };
    const lds_u32x4 av = {word(1), word(2), word(3), word(4)}, bv = {word(5), word(6), word(7), word(8)};
    const mfma_bf16x8 a = __builtin_bit_cast(mfma_bf16x8, av), b = __builtin_bit_cast(mfma_bf16x8, bv);
    mfma_f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = mfma_f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

constexpr int kSelectThreads = 256;
constexpr uint32_t kSelectMaxTokens = 8192;   // per frame (the head means sit in LDS)

__global__ __launch_bounds__(kSelectThreads) void select_salient_kernel(const float* scores, uint32_t heads,
                                                                        uint32_t grid_h, uint32_t grid_w, uint32_t tile_h,
                                                                        uint32_t tile_w, int32_t* rows_out)
{
    __shared__ double mean[kSelectMaxTokens];
    __shared__ uint8_t chosen[kSelectMaxTokens];
    __shared__ uint32_t wave_total[kSelectThreads / 64];
    const uint32_t tokens = grid_h * grid_w, frame = blockIdx.x;
    const float* sf = scores + (size_t)frame * heads * tokens;
    for (uint32_t t = threadIdx.x; t < tokens; t += kSelectThreads) {
        double m = 0.0;
        uint32_t h = 0;
        for (; h + 8 <= heads; h += 8) {   // eight loads in flight, added in head order
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = sf[(size_t)(h + j) * tokens + t];
#pragma unroll
            for (int j = 0; j < 8; ++j) m += (double)v[j];
        }
        for (; h < heads; ++h) m += (double)sf[(size_t)h * tokens + t];
        mean[t] = m / (double)heads;
        chosen[t] = 0;
    }
    __syncthreads();
    const uint32_t th = (grid_h + tile_h - 1) / tile_h, tw = (grid_w + tile_w - 1) / tile_w;
    for (uint32_t tile = threadIdx.x; tile < th * tw; tile += kSelectThreads) {
        const uint32_t ty = tile / tw, tx = tile - ty * tw;
        uint32_t best = 0xFFFFFFFFu;
        double best_v = 0.0;
        for (uint32_t y = ty * tile_h; y < min(grid_h, (ty + 1) * tile_h); ++y) {
            for (uint32_t x = tx * tile_w; x < min(grid_w, (tx + 1) * tile_w); ++x) {
                double v = mean[y * grid_w + x];
                if (v != v) v = -__builtin_inf();
                if (best == 0xFFFFFFFFu || v > best_v) { best = y * grid_w + x; best_v = v; }
            }
        }
        chosen[best] = 1;   // (tiles are disjoint: no two threads write the same byte)
    }
    __syncthreads();
    // ascending compaction: thread t owns a contiguous run of tokens
    const uint32_t per = (tokens + kSelectThreads - 1) / kSelectThreads;
    const uint32_t first = threadIdx.x * per, last = min(tokens, first + per);
    uint32_t count = 0;
    for (uint32_t t = first; t < last; ++t) count += chosen[t];
    uint32_t incl = count;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_up(incl, off);
        if ((int)(threadIdx.x & 63) >= off) incl += v;
    }
    if ((threadIdx.x & 63) == 63) wave_total[threadIdx.x >> 6] = incl;
    __syncthreads();
    uint32_t at = incl - count;
    for (uint32_t w = 0; w < (threadIdx.x >> 6); ++w) at += wave_total[w];
    int32_t* out = rows_out + (size_t)frame * th * tw;
    for (uint32_t t = first; t < last; ++t)
        if (chosen[t]) out[at++] = (int32_t)(frame * tokens + t);
}

// Sec. 3.4 ("Attention-Guided Semantic Relatedness Extraction"), the marking step: every anchor marks the tokens
// of a window x window (x window_t frames) box around it whose raw attention score from the anchor -- Q[anchor] .
// K[token], averaged over the heads -- exceeds a threshold.  The group of an anchor is the row-major number of the
// spatial tile it lies in (the per-frame candidates of a tile share one sub-formatbook); a token marked by anchors
// of several groups belongs to the highest group number (App. D: the subsequent anchor), an anchor to its own
// group.  Three small launches: fill with -1, mark (one workgroup per anchor and frame of the window: 64 window
// slots x 4 shares of the heads, a maximum on the group number), anchors.
// Token (frame f, head h, token t) of Q / K sits at ((f * stride_f + h * stride_h) + t) * dim: factorized
// attention [frames][heads][tokens][dim], 3D attention [heads][frames * tokens][dim].
constexpr int kAssignThreads = 256;   // 64 window slots x 4 groups of heads

__global__ __launch_bounds__(256) void seda_fill_kernel(int32_t* a, int32_t* b, uint32_t n)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < n) {
        a[i] = -1;
        if (b) b[i] = -1;
    }
}

__device__ __forceinline__ uint32_t tile_of(uint32_t token, uint32_t grid_w, uint32_t tile_h, uint32_t tile_w)
{
    const uint32_t y = token / grid_w, x = token - y * grid_w;
    return (y / tile_h) * ((grid_w + tile_w - 1) / tile_w) + x / tile_w;
}

// Dot product of two bf16 rows of `dim` channels (a multiple of 8) in fp32: four chains over the 16-byte pieces
// c, c + 1, c + 2, c + 3 (mod 4), added as (0 + 1) + (2 + 3).
__device__ __forceinline__ float dot_bf16_rows(const uint16_t* qrow, const uint16_t* krow, uint32_t dim)
{
    const uint4* qr = reinterpret_cast<const uint4*>(qrow);
    const uint4* kr = reinterpret_cast<const uint4*>(krow);
    const uint32_t n16 = dim / 8;
    float part[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (uint32_t c = 0; c < n16; c += 4) {
        uint4 qa[4], kb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {   // (a piece past the row's end re-reads the last one and is skipped)
            qa[j] = qr[min(c + j, n16 - 1u)];
            kb[j] = kr[min(c + j, n16 - 1u)];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (c + j < n16) {
                const uint32_t qs[4] = {qa[j].x, qa[j].y, qa[j].z, qa[j].w}, ks[4] = {kb[j].x, kb[j].y, kb[j].z, kb[j].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    part[j] = __builtin_fmaf(__uint_as_float(qs[i] << 16), __uint_as_float(ks[i] << 16), part[j]);
                    part[j] = __builtin_fmaf(__uint_as_float(qs[i] & 0xFFFF0000u), __uint_as_float(ks[i] & 0xFFFF0000u), part[j]);
                }
            }
        }
    }
    return (part[0] + part[1]) + (part[2] + part[3]);
}

struct AssignParams {
    uint32_t frames, heads, grid_h, grid_w, dim, tile_h, tile_w, window, window_t;
    uint64_t stride_f, stride_h;   // in tokens
    float threshold;
};

__global__ __launch_bounds__(kAssignThreads) void seda_mark_kernel(const uint16_t* q, const uint16_t* k,
                                                                   const int32_t* anchors, AssignParams p,
                                                                   int32_t* token_group, float* scores)
{
    __shared__ float partial[4][64];
    const uint32_t tokens = p.grid_h * p.grid_w;
    const uint32_t i = blockIdx.x, wt = blockIdx.y;
    const int64_t row = anchors[i];
    const uint32_t w = threadIdx.x & 63u, hq = threadIdx.x >> 6;
    // (no early exit: every thread reaches the barrier)
    const bool slot = w < p.window * p.window;
    const bool anchor_ok = row >= 0 && row < (int64_t)p.frames * tokens;   // otherwise: no token of the clip, marks nothing
    const uint32_t rc = anchor_ok ? (uint32_t)row : 0u;
    const uint32_t fa = rc / tokens, ac = rc - fa * tokens;
    const uint32_t g = tile_of(ac, p.grid_w, p.tile_h, p.tile_w);
    const int32_t ay = (int32_t)(ac / p.grid_w), ax = (int32_t)(ac % p.grid_w);
    const int32_t f = (int32_t)fa + (int32_t)wt - (int32_t)(p.window_t / 2);
    const int32_t y = ay + (int32_t)(w / p.window) - (int32_t)(p.window / 2), x = ax + (int32_t)(w % p.window) - (int32_t)(p.window / 2);
    const bool inside = slot && anchor_ok && f >= 0 && f < (int32_t)p.frames && y >= 0 && y < (int32_t)p.grid_h && x >= 0 &&
                        x < (int32_t)p.grid_w;
    const uint32_t t = inside ? (uint32_t)y * p.grid_w + (uint32_t)x : 0u;
    const uint32_t fc = inside ? (uint32_t)f : 0u;
    float acc = 0.0f;
    if (inside) {
        for (uint32_t h = hq; h < p.heads; h += 4)   // this thread's share of the heads
            acc += dot_bf16_rows(q + (fa * p.stride_f + h * p.stride_h + ac) * p.dim,
                                 k + (fc * p.stride_f + h * p.stride_h + t) * p.dim, p.dim);
    }
    partial[hq][w] = acc;
    __syncthreads();
    if (hq == 0 && slot) {
        const size_t per = (size_t)p.window_t * p.window * p.window;
        float* out = scores ? scores + (size_t)i * per + (size_t)wt * p.window * p.window + w : nullptr;
        const float sc = (partial[0][w] + partial[1][w] + partial[2][w] + partial[3][w]) / (float)p.heads;   // fixed order
        if (out) *out = inside ? sc : __builtin_nanf("");
        if (inside && sc > p.threshold) atomicMax(token_group + (size_t)fc * tokens + t, (int32_t)g);
    }
}

__global__ __launch_bounds__(256) void seda_anchor_kernel(const int32_t* anchors, uint32_t n, uint32_t frames,
                                                          uint32_t grid_h, uint32_t grid_w, uint32_t tile_h, uint32_t tile_w,
                                                          int32_t* token_group, int32_t* anchor_group)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n) return;
    const uint32_t tokens = grid_h * grid_w;
    const int64_t row = anchors[i];
    if (row < 0 || row >= (int64_t)frames * tokens) return;
    const int32_t g = (int32_t)tile_of((uint32_t)row % tokens, grid_w, tile_h, tile_w);
    token_group[row] = g;    // (two entries naming one row write the same value)
    anchor_group[row] = g;
}

// Sec. 3.4, factorized attention, step 2: one workgroup per spatial tile, one wavefront per frame at a time.  Per
// frame the tile's candidate (the first entry of the frame's list that lies in this tile of this frame) and its
// temporal mean score averaged over the heads (in double, head by head); the main anchor is the best of them
// (earliest frame on ties, a NaN never wins); a frame stays if it is the main anchor's or if the raw temporal
// score from the main anchor to it -- Qt[p*][h][f*] . Kt[p*][h][f], head mean in fp32 -- exceeds the threshold.
// Every entry of `kept` is written exactly once: by the workgroup of the tile the entry lies in (an entry that is
// no candidate of its frame by the workgroup of tile 0), so no launch has to clear it first.
constexpr int kMainThreads = 256;
constexpr uint32_t kMainMaxFrames = 1024;

__global__ __launch_bounds__(kMainThreads) void seda_main_anchor_kernel(
    const float* temporal_scores, const uint16_t* qt, const uint16_t* kt, uint32_t frames, uint32_t heads, uint32_t grid_h,
    uint32_t grid_w, uint32_t dim, const int32_t* cand, uint32_t n_per_frame, uint32_t tile_h, uint32_t tile_w,
    float prune_threshold, int32_t* main_anchor, int32_t* kept, float* prune_scores)
{
    __shared__ double score[kMainMaxFrames];
    __shared__ int32_t slot[kMainMaxFrames];
    __shared__ int32_t best_frame;
    constexpr uint32_t kWaves = kMainThreads / 64, kNone = 0xFFFFFFFFu;
    const uint32_t tokens = grid_h * grid_w, tile = blockIdx.x, tiles = gridDim.x;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    for (uint32_t f = wave; f < frames; f += kWaves) {
        const int32_t* list = cand + (size_t)f * n_per_frame;
        int32_t* out = kept + (size_t)f * n_per_frame;
        uint32_t found = kNone;
        for (uint32_t j0 = 0; j0 < n_per_frame; j0 += 64) {
            const uint32_t j = j0 + lane;
            bool mine = false;
            if (j < n_per_frame) {
                const int64_t row = list[j];
                const bool valid = row >= (int64_t)f * tokens && row < (int64_t)(f + 1) * tokens;
                mine = valid && tile_of((uint32_t)(row - (int64_t)f * tokens), grid_w, tile_h, tile_w) == tile;
                if (!valid && tile == 0) out[j] = -1;
            }
            const unsigned long long m = __ballot(mine);
            const uint32_t first = m ? j0 + (uint32_t)__builtin_ctzll(m) : kNone;
            if (mine && (found != kNone || j != first)) out[j] = -1;   // a later entry of the same tile
            if (found == kNone) found = first;
        }
        double v = 0.0;
        if (found != kNone) {
            const uint32_t pos = (uint32_t)(list[found] - (int32_t)(f * tokens));
            for (uint32_t h0 = 0; h0 < heads; h0 += 64) {
                const uint32_t cnt = min(64u, heads - h0);
                const float own = lane < cnt ? temporal_scores[((size_t)pos * heads + h0 + lane) * frames + f] : 0.0f;
                for (uint32_t i = 0; i < cnt; ++i) v += (double)__shfl(own, (int)i);
            }
            v /= (double)heads;
            if (v != v) v = -__builtin_inf();
        }
        if (lane == 0) {
            slot[f] = found == kNone ? -1 : (int32_t)found;
            score[f] = v;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t bf = -1;
        double bv = 0.0;
        for (uint32_t f = 0; f < frames; ++f) {
            if (slot[f] < 0) continue;
            if (bf < 0 || score[f] > bv) { bf = (int32_t)f; bv = score[f]; }
        }
        best_frame = bf;
        main_anchor[tile] = bf < 0 ? -1 : cand[(size_t)bf * n_per_frame + slot[bf]];
    }
    __syncthreads();
    const int32_t bf = best_frame;
    const uint32_t n16 = dim / 8;
    for (uint32_t f = wave; f < frames; f += kWaves) {
        float sc = __builtin_nanf("");
        if (slot[f] >= 0) {   // (then the tile has a main anchor)
            const uint32_t pos = (uint32_t)(cand[(size_t)bf * n_per_frame + slot[bf]] - (int32_t)((uint32_t)bf * tokens));
            // 16 lanes share a row's 16-byte pieces, four heads at a time; the wavefront's sum in a fixed order
            float acc = 0.0f;
            for (uint32_t h = lane >> 4; h < heads; h += 4) {
                const size_t base = ((size_t)pos * heads + h) * frames;
                const uint4* qr = reinterpret_cast<const uint4*>(qt + (base + (uint32_t)bf) * dim);
                const uint4* kr = reinterpret_cast<const uint4*>(kt + (base + f) * dim);
                for (uint32_t c = lane & 15u; c < n16; c += 16) {
                    const uint4 a = qr[c], b = kr[c];
                    const uint32_t qs[4] = {a.x, a.y, a.z, a.w}, ks[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        acc = __builtin_fmaf(__uint_as_float(qs[i] << 16), __uint_as_float(ks[i] << 16), acc);
                        acc = __builtin_fmaf(__uint_as_float(qs[i] & 0xFFFF0000u), __uint_as_float(ks[i] & 0xFFFF0000u), acc);
                    }
                }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
            sc = acc / (float)heads;
            if (lane == 0) {
                const int32_t row = cand[(size_t)f * n_per_frame + slot[f]];
                kept[(size_t)f * n_per_frame + slot[f]] = ((int32_t)f == bf || sc > prune_threshold) ? row : -1;
            }
        }
        if (lane == 0 && prune_scores) prune_scores[(size_t)f * tiles + tile] = sc;
    }
}

// Sec. 3.4, 3D attention: the main anchor of a spatial tile is the best token among its tile_h x tile_w x frames
// tokens by the head mean (double, head by head) of the clip-wide scores [heads][frames * tokens]; the lowest row
// on ties, a NaN never wins.  One workgroup per tile.
__global__ __launch_bounds__(kMainThreads) void seda_main_anchor_3d_kernel(const float* scores, uint32_t frames, uint32_t heads,
                                                                            uint32_t grid_h, uint32_t grid_w, uint32_t tile_h,
                                                                            uint32_t tile_w, int32_t* anchors)
{
    __shared__ double best_v[kMainThreads];
    __shared__ uint32_t best_row[kMainThreads];
    const uint32_t tokens = grid_h * grid_w, tile = blockIdx.x;
    const uint32_t tw = (grid_w + tile_w - 1) / tile_w;
    const uint32_t y0 = (tile / tw) * tile_h, x0 = (tile % tw) * tile_w;
    const uint32_t hh = min(tile_h, grid_h - y0), ww = min(tile_w, grid_w - x0);
    const uint32_t n = frames * hh * ww;
    const size_t total = (size_t)frames * tokens;
    double bv = 0.0;
    uint32_t br = 0xFFFFFFFFu;
    for (uint32_t i = threadIdx.x; i < n; i += kMainThreads) {   // ascending rows per thread
        const uint32_t f = i / (hh * ww), r = i - f * (hh * ww);
        const uint32_t row = f * tokens + (y0 + r / ww) * grid_w + x0 + r % ww;
        double v = 0.0;
        for (uint32_t h = 0; h < heads; ++h) v += (double)scores[(size_t)h * total + row];
        v /= (double)heads;
        if (v != v) v = -__builtin_inf();
        if (br == 0xFFFFFFFFu || v > bv) { br = row; bv = v; }
    }
    best_v[threadIdx.x] = bv;
    best_row[threadIdx.x] = br;
    __syncthreads();
    for (uint32_t s = kMainThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) {
            const double ov = best_v[threadIdx.x + s];
            const uint32_t orow = best_row[threadIdx.x + s];
            const double mv = best_v[threadIdx.x];
            const uint32_t mrow = best_row[threadIdx.x];
            const bool take = orow != 0xFFFFFFFFu && (mrow == 0xFFFFFFFFu || ov > mv || (ov == mv && orow < mrow));
            if (take) { best_v[threadIdx.x] = ov; best_row[threadIdx.x] = orow; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) anchors[tile] = (int32_t)best_row[0];
}

}  // namespace fb4
