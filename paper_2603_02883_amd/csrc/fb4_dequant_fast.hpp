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
    // kSum: second plane of the salient rows (Sec. 3.3), added in fp32
    const uint8_t* codes2;    // [n_sal][nb * 16]
    const uint16_t* meta2;
    const int32_t* salient;   // [n_sal] ascending, unique
    uint32_t n_sal;
    uint32_t rows;            // <= kMaxFusedRows
};

// Decoded pair (two bf16 patterns) of one code byte: table entry for exponent byte 130 plus the block's
// exponent offset on every non-zero half.
__device__ __forceinline__ uint32_t decode_pair(const uint32_t* pair, uint32_t base, uint32_t byte, uint32_t live,
                                                uint32_t eoff2)
{
    const uint32_t v = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(pair) + base + byte * 4) & live;
    const uint32_t nz = pk_min(v & 0x7FFF7FFFu, 0x00010001u);          // 1 where the magnitude is not zero
    const u16x2 r = __builtin_bit_cast(u16x2, nz) * __builtin_bit_cast(u16x2, eoff2) + __builtin_bit_cast(u16x2, v);
    return __builtin_bit_cast(uint32_t, r);
}

// kSum: rows listed in p.salient are written as round(fp32(plane 1) + fp32(plane 2)); a bitmap of those rows
// with a running count per bitmap word (LDS) gives a row's position in the compact second plane.
// The leading scalar arguments repeat the fields of `p` that the first loads depend on; they arrive in
// registers when the wavefront starts (kernel-argument preload), the rest by a load.
template <bool kFlat, bool kF32, bool kSum = false>
__global__ __launch_bounds__(kDeqThreads) void dequantize_fast_kernel(
    const uint8_t* blob, const uint8_t* codes, const uint16_t* meta, uint32_t n_blocks, uint32_t meta_shift,
    uint32_t n_workgroups, DeqFastParams p)
{
    p.blob = blob; p.codes = codes; p.meta = meta; p.n_blocks = n_blocks; p.meta_shift = meta_shift;
    __shared__ __align__(16) uint32_t pair[32 * 256];   // [DID][code byte] -> two bf16 patterns
    __shared__ __align__(16) uint32_t sal_bits[kSum ? kMaxFusedRows / 32 : 4];
    __shared__ uint16_t sal_rank[kSum ? kMaxFusedRows / 32 : 4];
    __shared__ uint32_t sal_before, sal_wave[kDeqWaves];
    // Work item = one code word (4 bytes = 8 elements) -> 16 bytes of bf16: consecutive lanes take consecutive
    // words, so every load and store instruction of a wavefront covers one contiguous span.
    constexpr int U = 4;
    const uint32_t n_words = p.n_blocks * 4u;
    const uint32_t stride = n_workgroups * kDeqThreads;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    uint32_t cw[U], mw[U];
    // (indices are clamped, not predicated: a lane past the end reads the last word and stores nothing)
    auto request = [&](unsigned long long i64) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long i = i64 + (unsigned long long)u * stride;
            const uint32_t ic = (uint32_t)(i < n_words ? i : n_words - 1u);
            cw[u] = reinterpret_cast<const uint32_t*>(p.codes)[ic];
            mw[u] = p.meta[ic >> p.meta_shift];
        }
    };
    const unsigned long long first = blockIdx.x * kDeqThreads + threadIdx.x;
    // the table's source and the first round of codes are requested together; the table is built while the
    // codes are on their way
    const uint32_t did_t = threadIdx.x >> 4, hn_t = threadIdx.x & 15;
    const uint4 dq = *reinterpret_cast<const uint4*>(p.blob + kOffDecode + did_t * 16);   // 8 bf16 magnitudes
    __builtin_amdgcn_sched_barrier(0);
    request(first);
    __builtin_amdgcn_sched_barrier(0);
    {
        // thread (DID, high nibble) fills 16 entries
        const uint32_t dv[8] = {dq.x & 0xFFFFu, dq.x >> 16, dq.y & 0xFFFFu, dq.y >> 16,
                                dq.z & 0xFFFFu, dq.z >> 16, dq.w & 0xFFFFu, dq.w >> 16};
        uint32_t hi = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) hi = ((hn_t & 7u) == (uint32_t)k) ? dv[k] : hi;
        hi = (hi | ((hn_t & 8u) << 12)) << 16;
        uint32_t* dst = pair + did_t * 256 + hn_t * 16;
#pragma unroll
        for (int ln = 0; ln < 16; ++ln) dst[ln] = hi | dv[ln & 7] | ((uint32_t)(ln & 8) << 12);
        __syncthreads();
    }
    // (the salient list is read after the codes were requested: both are then on their way together)
    if (kSum) {
        static_assert(kDeqThreads * 4 * 32 == (int)kMaxFusedRows, "four bitmap words per thread");
        for (uint32_t i = threadIdx.x; i < kMaxFusedRows / 32; i += kDeqThreads) sal_bits[i] = 0;
        if (threadIdx.x == 0) sal_before = 0;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < p.n_sal; i += kDeqThreads) {
            const int32_t r = p.salient[i];
            if (r < 0) atomicAdd(&sal_before, 1u);
            else if ((uint32_t)r < p.rows) atomicOr(&sal_bits[(uint32_t)r >> 5], 1u << (r & 31));
        }
        __syncthreads();
        const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const uint4 wv = reinterpret_cast<const uint4*>(sal_bits)[threadIdx.x];
        const uint32_t c0 = __builtin_popcount(wv.x), c1 = c0 + __builtin_popcount(wv.y);
        const uint32_t c2 = c1 + __builtin_popcount(wv.z), c3 = c2 + __builtin_popcount(wv.w);
        uint32_t incl = c3;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t v = __shfl_up(incl, off);
            if ((int)lane >= off) incl += v;
        }
        if (lane == 63) sal_wave[wave] = incl;
        __syncthreads();
        uint32_t base = sal_before + incl - c3;
        for (uint32_t k = 0; k < wave; ++k) base += sal_wave[k];
        sal_rank[threadIdx.x * 4] = (uint16_t)base;
        sal_rank[threadIdx.x * 4 + 1] = (uint16_t)(base + c0);
        sal_rank[threadIdx.x * 4 + 2] = (uint16_t)(base + c1);
        sal_rank[threadIdx.x * 4 + 3] = (uint16_t)(base + c2);
        __syncthreads();
    }
    // 64-bit loop counter: i0 + stride * U may pass 2^32 for the largest tensors
    for (unsigned long long i64 = first; i64 < n_words; i64 += (unsigned long long)stride * U) {
        const uint32_t i0 = (uint32_t)i64;
        if (i64 != first) request(i64);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i64 + (unsigned long long)u * stride >= n_words) break;
            const uint32_t i = i0 + u * stride;
            const uint32_t m = mw[u];
            const uint32_t did = m & 0xFFu;
            // exponent offset for both halves; a DID outside the table decodes as zeros
            const uint32_t eoff = (((m >> 8) - 130u) << 7) & 0xFFFFu;
            const uint32_t eoff2 = eoff | (eoff << 16);
            const uint32_t base = (did < 32u ? did : 0u) * 1024u;
            const uint32_t live = did < 32u ? 0xFFFFFFFFu : 0u;
            uint32_t o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) o[k] = decode_pair(pair, base, (cw[u] >> (8 * k)) & 0xFFu, live, eoff2);
            float fsum[8];
            bool summed = false;
            if (kSum) {
                const uint32_t gb = i >> 2;
                const uint32_t row = (uint32_t)(((unsigned long long)gb * p.div_mul) >> p.div_shift);
                const uint32_t wbits = sal_bits[row >> 5];
                if ((wbits >> (row & 31)) & 1u) {
                    // second plane: same decode, then one fp32 addition per element
                    summed = true;
                    const size_t pos = sal_rank[row >> 5] + __builtin_popcount(wbits & ((1u << (row & 31)) - 1u));
                    const size_t w2 = (pos * p.nb + (gb - row * p.nb)) * 4 + (i & 3u);
                    const uint32_t c2 = reinterpret_cast<const uint32_t*>(p.codes2)[w2];
                    const uint32_t m2 = p.meta2[w2 >> p.meta_shift];
                    const uint32_t did2 = m2 & 0xFFu;
                    const uint32_t e2 = (((m2 >> 8) - 130u) << 7) & 0xFFFFu;
                    const uint32_t base2 = (did2 < 32u ? did2 : 0u) * 1024u;
                    const uint32_t live2 = did2 < 32u ? 0xFFFFFFFFu : 0u;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t q = decode_pair(pair, base2, (c2 >> (8 * k)) & 0xFFu, live2, e2 | (e2 << 16));
                        fsum[2 * k] = __uint_as_float(o[k] << 16) + __uint_as_float(q << 16);
                        fsum[2 * k + 1] = __uint_as_float(o[k] & 0xFFFF0000u) + __uint_as_float(q & 0xFFFF0000u);
                    }
                    if (!kF32) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            uint32_t a = __float_as_uint(fsum[2 * k]), b = __float_as_uint(fsum[2 * k + 1]);
                            a += 0x7FFFu + ((a >> 16) & 1u);           // round to nearest even
                            b += 0x7FFFu + ((b >> 16) & 1u);
                            o[k] = (a >> 16) | (b & 0xFFFF0000u);
                        }
                    }
                }
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
                u32x4 v0 = {o[0] << 16, o[0] & 0xFFFF0000u, o[1] << 16, o[1] & 0xFFFF0000u};
                u32x4 v1 = {o[2] << 16, o[2] & 0xFFFF0000u, o[3] << 16, o[3] & 0xFFFF0000u};
                if (kSum && summed) {
                    v0 = u32x4{__float_as_uint(fsum[0]), __float_as_uint(fsum[1]), __float_as_uint(fsum[2]), __float_as_uint(fsum[3])};
                    v1 = u32x4{__float_as_uint(fsum[4]), __float_as_uint(fsum[5]), __float_as_uint(fsum[6]), __float_as_uint(fsum[7])};
                }
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
