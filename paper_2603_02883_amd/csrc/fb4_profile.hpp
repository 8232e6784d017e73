// SeDA sub-formatbook construction (Sec. 3.4, "Constructing an 8-Dialect
// Sub-Formatbook"): count how often each dialect was selected on the anchor
// tokens of each group, then keep, per dynamic-range bucket (largest magnitude
// 8..15), the most frequently selected dialect of that bucket.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fb4_tables.hpp"

namespace fb4 {

constexpr int kProfileThreads = 256;

__global__ __launch_bounds__(kProfileThreads) void profile_clear_kernel(uint32_t* counts, uint32_t n)
{
    const uint32_t i = blockIdx.x * kProfileThreads + threadIdx.x;
    if (i < n) counts[i] = 0;
}

// One wavefront per row: a 32-bin histogram of the row's DIDs in LDS, then at most 32 global atomics.
__global__ __launch_bounds__(kProfileThreads) void profile_count_kernel(const uint16_t* meta, long long rows,
                                                                        long long nb, const int32_t* anchor_group,
                                                                        int n_groups, uint32_t* counts)
{
    __shared__ uint32_t hist[kProfileThreads / 64][32];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long stride = (long long)gridDim.x * (kProfileThreads / 64);
    for (long long r = (long long)blockIdx.x * (kProfileThreads / 64) + wave; r < rows; r += stride) {
        const int g = anchor_group[r];                    // wave-uniform
        if (g < 0 || g >= n_groups) continue;
        if (lane < 32) hist[wave][lane] = 0;
        __builtin_amdgcn_wave_barrier();
        const uint16_t* row = meta + r * nb;
        for (long long b = lane; b < nb; b += 64) {
            const uint32_t did = row[b] & 0xFFu;
            if (did < 32u) atomicAdd(&hist[wave][did], 1u);
        }
        __builtin_amdgcn_wave_barrier();
        if (lane < 32) {
            const uint32_t c = hist[wave][lane];
            if (c) atomicAdd(counts + (long long)g * 32 + lane, c);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// One thread per (group, range bucket): the most frequent dialect of the bucket, lowest DID on ties (and when
// none was selected); 255 when the formatbook has no dialect of that range.
__global__ __launch_bounds__(kProfileThreads) void profile_select_kernel(const uint32_t* counts, int n_groups,
                                                                         const uint8_t* blob, uint8_t* sub)
{
    const uint32_t i = blockIdx.x * kProfileThreads + threadIdx.x;
    if (i >= (uint32_t)n_groups * 8u) return;
    const uint32_t g = i >> 3, k = i & 7u;
    const int n = *reinterpret_cast<const int32_t*>(blob + kOffCount);
    uint32_t best = 255u;
    long long best_count = -1;
    for (int d = 0; d < n; ++d) {
        const long long c = counts[(size_t)g * 32 + d];
        if (blob[kOffTop + d] == 8u + k && c > best_count) {
            best = (uint32_t)d;
            best_count = c;
        }
    }
    sub[i] = (uint8_t)best;
}

}  // namespace fb4
