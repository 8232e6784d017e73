// Streaming decode of the first code plane (Sec. 3.1; the 4-bit -> 16-bit decode
// of App. E.2): y = (-1)^sign * M[DID][index] * 2^(e-3).
//
// One lane decodes one code word (4 bytes = 8 elements) into 16 bytes of bf16
// (or 32 bytes of fp32), so that every load and store instruction of a
// wavefront covers one contiguous span of memory.  A pair table in LDS
// maps (DID, code byte) to the two decoded bf16 magnitudes with their signs for
// exponent byte 130 (scale 1); the block exponent is then added to the exponent
// field of every non-zero half with packed 16-bit arithmetic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fb4_fast.hpp"
#include "fb4_tables.hpp"

namespace fb4 {

constexpr int kDeqThreads = 512;
constexpr int kDeqWaves = kDeqThreads / 64;

struct DeqFastParams {
    const uint8_t* codes;     // [n_blocks][16]; a "block" here is a 32-element chunk of a row
    const uint16_t* meta;     // one word per 4 code words (block size 32) or per 2 (block size 16)
    uint32_t meta_shift;      // 2 or 1
    void* out;                // bf16 or fp32, [rows][out_row_stride]
    long long out_row_stride; // elements
    uint32_t nb, n_blocks, n_tiles, div_mul, div_shift;
    const uint8_t* blob;
};

template <bool kFlat, bool kF32>
__global__ __launch_bounds__(kDeqThreads) void dequantize_fast_kernel(DeqFastParams p)
{
    __shared__ __align__(16) uint32_t pair[32 * 256];   // [DID][code byte] -> two bf16 patterns
    {
        // thread (DID, high nibble) fills 16 entries
        const uint32_t did = threadIdx.x >> 4, hn = threadIdx.x & 15;
        const uint4 dq = *reinterpret_cast<const uint4*>(p.blob + kOffDecode + did * 16);   // 8 bf16 magnitudes
        const uint32_t dv[8] = {dq.x & 0xFFFFu, dq.x >> 16, dq.y & 0xFFFFu, dq.y >> 16,
                                dq.z & 0xFFFFu, dq.z >> 16, dq.w & 0xFFFFu, dq.w >> 16};
        uint32_t hi = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) hi = ((hn & 7u) == (uint32_t)k) ? dv[k] : hi;
        hi = (hi | ((hn & 8u) << 12)) << 16;
        uint32_t* dst = pair + did * 256 + hn * 16;
#pragma unroll
        for (int ln = 0; ln < 16; ++ln) dst[ln] = hi | dv[ln & 7] | ((uint32_t)(ln & 8) << 12);
        __syncthreads();
    }
    // Work item = one code word (4 bytes = 8 elements) -> 16 bytes of bf16: consecutive lanes take consecutive
    // words, so every load and store instruction of a wavefront covers one contiguous span.
    constexpr int U = 4;
    const uint32_t n_words = p.n_blocks * 4u;
    const uint32_t stride = gridDim.x * kDeqThreads;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    for (uint32_t i0 = blockIdx.x * kDeqThreads + threadIdx.x; i0 < n_words; i0 += stride * U) {
        uint32_t cw[U], mw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * stride;
            cw[u] = 0;
            mw[u] = 0;
            if (i < n_words) {
                cw[u] = reinterpret_cast<const uint32_t*>(p.codes)[i];
                mw[u] = p.meta[i >> p.meta_shift];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * stride;
            if (i >= n_words) break;
            const uint32_t m = mw[u];
            const uint32_t did = m & 0xFFu;
            // exponent offset for both halves; a DID outside the table decodes as zeros
            const uint32_t eoff = (((m >> 8) - 130u) << 7) & 0xFFFFu;
            const uint32_t eoff2 = eoff | (eoff << 16);
            const uint32_t base = (did < 32u ? did : 0u) * 1024u;
            const uint32_t live = did < 32u ? 0xFFFFFFFFu : 0u;
            uint32_t o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t byte = (cw[u] >> (8 * k)) & 0xFFu;
                const uint32_t v = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(pair) + base + byte * 4) & live;
                const uint32_t nz = pk_min(v & 0x7FFF7FFFu, 0x00010001u);          // 1 where the magnitude is not zero
                const u16x2 r = __builtin_bit_cast(u16x2, nz) * __builtin_bit_cast(u16x2, eoff2) + __builtin_bit_cast(u16x2, v);
                o[k] = __builtin_bit_cast(uint32_t, r);
            }
            long long off;   // elements
            if (kFlat) {
                off = (long long)i * 8;
            } else {
                const uint32_t gb = i >> 2;
                const uint32_t row = (uint32_t)(((unsigned long long)gb * p.div_mul) >> p.div_shift);
                off = (long long)row * p.out_row_stride + (long long)(gb - row * p.nb) * 32 + (i & 3u) * 8;
            }
            if (kF32) {
                u32x4* dst = reinterpret_cast<u32x4*>(reinterpret_cast<float*>(p.out) + off);
                const u32x4 v0 = {o[0] << 16, o[0] & 0xFFFF0000u, o[1] << 16, o[1] & 0xFFFF0000u};
                const u32x4 v1 = {o[2] << 16, o[2] & 0xFFFF0000u, o[3] << 16, o[3] & 0xFFFF0000u};
                __builtin_nontemporal_store(v0, dst);
                __builtin_nontemporal_store(v1, dst + 1);
            } else {
                const u32x4 v = {o[0], o[1], o[2], o[3]};
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(p.out) + off));
            }
        }
    }
}

}  // namespace fb4
