// FB4 code plane -> MXFP8 operands (Sec. 4.5 and App. E.2: the integer
// magnitudes 0..15 are exact in FP8 E4M3 and the block scale is a power of
// two, so the codes feed a block-scaled FP8 matrix unit without a detour
// through 16-bit values).
//
// Per 32 elements: one E8M0 scale byte and 32 E4M3 bytes.  With block size 32
// the scale byte is the stored exponent byte minus 3 and every element is its
// magnitude; with block size 16 the two blocks of an MX block share the larger
// exponent and the other block's magnitudes are shifted down by the exponent
// difference k and rounded to E4M3 (exact for k <= 9).
//
// One lane re-encodes one code word (8 elements) into 8 bytes, so a wavefront
// reads 256 and writes 512 contiguous bytes.  LDS tables: block 32: (DID, code
// byte) -> the two finished E4M3 bytes; block 16: (DID, code byte) -> the two
// magnitudes, then (k, magnitude pair) -> their two E4M3 bytes after the shift.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fb4_tables.hpp"

namespace fb4 {

constexpr int kRepackThreads = 512;

struct RepackParams {
    const uint8_t* codes;      // [rows][cols/2]
    const uint16_t* meta;      // [rows][cols/block]
    uint8_t* elems;            // [rows][elem_row_stride] E4M3
    long long elem_row_stride; // bytes = elements
    uint8_t* scales;           // [rows][cols/32] E8M0
    uint32_t nb32;             // MX blocks per row
    uint32_t n_chunks;         // rows * nb32
    uint32_t div_mul, div_shift;
    const uint8_t* blob;
};

// E4M3 byte (no sign) of m * 2^-k, m in 0..15, k in 0..15, round to nearest even.
__device__ __forceinline__ uint32_t e4m3_of_shifted(uint32_t m, uint32_t k)
{
    if (m == 0) return 0;
    const int top = 31 - __builtin_clz(m);          // floor(log2 m), 0..3
    const int E = top - (int)k;                     // exponent of the value
    if (E >= -6) return (uint32_t)((E + 7) << 3) | ((m << (3 - top)) & 7u);   // normal, exact
    // subnormal: multiples of 2^-9
    if (k <= 9) return m << (9 - k);                // exact, below 8 because the value is below 2^-6
    const uint32_t s = k - 9;
    uint32_t q = m >> s;
    const uint32_t rem = m & ((1u << s) - 1u), half = 1u << (s - 1);
    if (rem > half || (rem == half && (q & 1u))) ++q;
    return q;
}

// The leading scalar arguments repeat the fields of `p` that the first loads depend on; they arrive in
// registers when the wavefront starts (kernel-argument preload), the rest by a load.
template <bool kFlat, bool kB16>
__global__ __launch_bounds__(kRepackThreads) void repack_mxfp8_kernel(
    const uint8_t* blob, const uint8_t* codes, const uint16_t* meta, uint32_t n_chunks, uint32_t n_workgroups,
    RepackParams p)
{
    p.blob = blob; p.codes = codes; p.meta = meta; p.n_chunks = n_chunks;
    // block 32: [DID][code byte] -> E4M3 of element 2j | element 2j+1 << 8 (no signs).  Block 16, two steps
    // because the shift k varies: magP [DID][code byte] -> the two magnitudes as nibbles, then
    // shP [k][magnitude pair] -> their two E4M3 bytes.
    __shared__ __align__(16) uint16_t pair[kB16 ? 16 * 256 : 32 * 256];   // block 16: shP
    __shared__ uint8_t magP[kB16 ? 32 * 256 : 4];
    __shared__ uint8_t magT[32 * 8];                     // [DID][index] -> integer magnitude
    __shared__ uint8_t shT[16 * 16];                     // [k][magnitude] -> E4M3 byte of magnitude * 2^-k
    const uint32_t n_words = p.n_chunks * 4u;
    const uint32_t stride = n_workgroups * kRepackThreads;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    uint32_t cw, mcur, mother = 0;
    // (the index is clamped, not predicated: a lane past the end reads the last word and stores nothing)
    auto request = [&](unsigned long long i64) {
        const uint32_t ic = (uint32_t)(i64 < n_words ? i64 : n_words - 1u);
        cw = reinterpret_cast<const uint32_t*>(p.codes)[ic];
        if (kB16) {
            mcur = p.meta[ic >> 1];
            mother = p.meta[(ic >> 1) ^ 1u];
        } else {
            mcur = p.meta[ic >> 2];
        }
    };
    const unsigned long long first = blockIdx.x * kRepackThreads + threadIdx.x;
    // the tables' source and the first code word are requested together; the tables are built while the
    // codes are on their way
    const uint32_t bits = reinterpret_cast<const uint16_t*>(p.blob + kOffDecode)[threadIdx.x & 255u];
    __builtin_amdgcn_sched_barrier(0);
    request(first);
    __builtin_amdgcn_sched_barrier(0);
    if (threadIdx.x < 256) {
        magT[threadIdx.x] = (uint8_t)(int)__uint_as_float(bits << 16);
        shT[threadIdx.x] = (uint8_t)e4m3_of_shifted(threadIdx.x & 15u, threadIdx.x >> 4);
    }
    __syncthreads();
    if (kB16) {
        for (uint32_t i = threadIdx.x; i < 32u * 256u; i += kRepackThreads) {
            const uint32_t did = i >> 8, cb = i & 255u;
            magP[i] = (uint8_t)(magT[did * 8 + (cb & 7u)] | (magT[did * 8 + ((cb >> 4) & 7u)] << 4));
        }
        for (uint32_t i = threadIdx.x; i < 16u * 256u; i += kRepackThreads) {
            const uint32_t k = i >> 8, mp = i & 255u;
            pair[i] = (uint16_t)(shT[k * 16 + (mp & 15u)] | (shT[k * 16 + (mp >> 4)] << 8));
        }
    } else {
        const uint32_t did = threadIdx.x >> 4, hn = threadIdx.x & 15;
        const uint32_t hi = (uint32_t)shT[magT[did * 8 + (hn & 7u)]] | ((hn & 8u) << 4);
#pragma unroll
        for (uint32_t ln = 0; ln < 16; ++ln) {
            const uint32_t lo = (uint32_t)shT[magT[did * 8 + (ln & 7u)]] | ((ln & 8u) << 4);
            pair[did * 256 + hn * 16 + ln] = (uint16_t)(lo | (hi << 8));
        }
    }
    __syncthreads();

    // 64-bit loop counter: i + stride may pass 2^32 for the largest tensors
    for (unsigned long long i64 = first; i64 < n_words; i64 += stride) {
        const uint32_t i = (uint32_t)i64;
        if (i64 != first) request(i64);
        const uint32_t chunk = i >> 2;
        uint32_t m, k = 0, sbyte;
        if (kB16) {
            m = mcur;
            const uint32_t other = mother;
            const uint32_t emax = max(m >> 8, other >> 8);
            k = min(emax - (m >> 8), 15u);          // 14 and more: every magnitude rounds to zero
            sbyte = emax - 3u;
        } else {
            m = mcur;
            sbyte = (m >> 8) - 3u;
        }
        const uint32_t did = m & 0xFFu;
        const bool live = did < 32u;                 // a DID outside the table decodes as zeros
        const uint32_t d = live ? did : 0u;
        uint32_t o0 = 0, o1 = 0;
        if (!kB16) {
            const uint32_t base = d * 256u;
            const uint32_t v0 = pair[base + (cw & 0xFFu)], v1 = pair[base + ((cw >> 8) & 0xFFu)];
            const uint32_t v2 = pair[base + ((cw >> 16) & 0xFFu)], v3 = pair[base + (cw >> 24)];
            o0 = v0 | (v1 << 16);
            o1 = v2 | (v3 << 16);
        } else {
            // magnitudes of the byte's two elements, then their E4M3 bytes after the shift by k; sign bits
            // (bit 3 and bit 7 of a code byte) go to bit 7 of either output byte
            uint32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t cb = (cw >> (8 * j)) & 0xFFu;
                v[j] = (uint32_t)pair[k * 256u + magP[d * 256u + cb]] | ((cb & 0x08u) << 4) | ((cb & 0x80u) << 8);
            }
            o0 = v[0] | (v[1] << 16);
            o1 = v[2] | (v[3] << 16);
        }
        if (!live) {
            // keep the sign bits, drop the magnitudes
            o0 = ((cw & 0x8u) << 4) | ((cw & 0x80u) << 8) | ((cw & 0x800u) << 12) | ((cw & 0x8000u) << 16);
            o1 = (((cw >> 16) & 0x8u) << 4) | (((cw >> 16) & 0x80u) << 8) | (((cw >> 16) & 0x800u) << 12) |
                 (((cw >> 16) & 0x8000u) << 16);
        }
        long long off;
        if (kFlat) {
            off = (long long)i * 8;
        } else {
            const uint32_t row = (uint32_t)(((unsigned long long)chunk * p.div_mul) >> p.div_shift);
            off = (long long)row * p.elem_row_stride + (long long)(chunk - row * p.nb32) * 32 + (i & 3u) * 8;
        }
        const u32x2 ov = {o0, o1};
        __builtin_nontemporal_store(ov, reinterpret_cast<u32x2*>(p.elems + off));
        if ((i & 3u) == 0u) p.scales[chunk] = (uint8_t)sbyte;
    }
}

}  // namespace fb4
