// Host-side construction of the FB4 lookup tables (Sec. 3.2, "LUT-Based
// Quantization Error Approximation").  Pure C++, no GPU calls: the blob built
// here is what the kernels copy into LDS.
#pragma once

#include <cstdint>
#include <cstring>

namespace fb4 {

constexpr int kMaxDialects = 32;
constexpr int kBins = 32;  // 0.5-wide bins over the normalized range [0,16)

// Blob layout (byte offsets); documented in include/fb4.h.
constexpr size_t kOffQerror8 = 0;      // u8  [32 bins][32 dialects]
constexpr size_t kOffQvalue64 = 1024;  // u8  [32 dialects][64]
constexpr size_t kOffQerror16 = 3072;  // u16 [32 bins][32 dialects], Qerror*32
constexpr size_t kOffMag16 = 5120;     // u16 [32 bins][32 dialects]
constexpr size_t kOffGain16 = 7168;    // u16 [32 bins][32 dialects]
constexpr size_t kOffDecode = 9216;    // u16 [32 dialects][8]
constexpr size_t kOffTop = 9728;       // u8  [32]
constexpr size_t kOffCount = 9760;     // i32
constexpr size_t kOffQvalueT = 9792;   // u8  [32 bins][32 dialects]: 3-bit index, bin-major
constexpr size_t kOffRangeExcl = 10816;  // u8 [8 ranges][32 dialects]: 0xFF = not in that dynamic range
constexpr size_t kBlobBytes = 11072;

// A formatbook row is valid when its magnitudes ascend strictly from 0 and its
// largest one lies in 8..15: one dynamic range per integer block maximum
// (Sec. 3.1, Sec. 3.4), index 0 decoding to zero (App. E.1).
inline bool formatbook_ok(const uint8_t* fbk, int n)
{
    if (!fbk || n < 1 || n > kMaxDialects) return false;
    for (int d = 0; d < n; ++d) {
        const uint8_t* m = fbk + 8 * d;
        if (m[0] != 0 || m[7] < 8 || m[7] > 15) return false;
        for (int k = 0; k < 7; ++k)
            if (m[k + 1] <= m[k]) return false;
    }
    return true;
}

// bf16 bit pattern of a small non-negative integer (exact).
inline uint16_t bf16_of_small_int(int v)
{
    if (v == 0) return 0;
    int e = 0;
    while ((v >> (e + 1)) != 0) ++e;  // floor(log2 v)
    uint32_t mant = (uint32_t)(v << (7 - e)) & 0x7F;
    return (uint16_t)(((127 + e) << 7) | mant);
}

inline void build_blob(const uint8_t* fbk, int n, uint8_t* blob)
{
    std::memset(blob, 0, kBlobBytes);
    uint8_t* qerr8 = blob + kOffQerror8;
    uint8_t* qval = blob + kOffQvalue64;
    uint16_t* qerr16 = reinterpret_cast<uint16_t*>(blob + kOffQerror16);
    uint16_t* mag16 = reinterpret_cast<uint16_t*>(blob + kOffMag16);
    uint16_t* gain16 = reinterpret_cast<uint16_t*>(blob + kOffGain16);
    uint16_t* decode = reinterpret_cast<uint16_t*>(blob + kOffDecode);
    uint8_t* top = blob + kOffTop;
    uint8_t* qvalT = blob + kOffQvalueT;
    for (int d = 0; d < kMaxDialects; ++d) {
        if (d >= n) {
            // A dialect that does not exist must never be selected: worst
            // possible approximate error, zero gain; ties go to lower DIDs.
            for (int b = 0; b < kBins; ++b) {
                qerr8[b * 32 + d] = 31;
                qerr16[b * 32 + d] = 31 * 32;
            }
            continue;
        }
        const uint8_t* m = fbk + 8 * d;
        top[d] = m[7];
        for (int k = 0; k < 8; ++k) decode[d * 8 + k] = bf16_of_small_int(m[k]);
        for (int b = 0; b < kBins; ++b) {
            // Bin b covers [b/2, (b+1)/2).  The decision boundary between two
            // neighbouring magnitudes is (m[k-1]+m[k])/2, a multiple of 1/2, so
            // it never falls inside a bin: the whole bin maps to one index, the
            // number of boundaries at or below its left edge (ties upward).
            int idx = 0;
            for (int k = 1; k < 8; ++k)
                if (m[k - 1] + m[k] <= b) idx = k;
            int mag = m[idx];
            // Qerror: |midpoint - magnitude| with midpoint b/2 + 1/4, in quarters.
            int e4 = 2 * b + 1 - 4 * mag;
            if (e4 < 0) e4 = -e4;
            qerr8[b * 32 + d] = (uint8_t)e4;
            qerr16[b * 32 + d] = (uint16_t)(e4 * 32);
            mag16[b * 32 + d] = (uint16_t)mag;
            // Exhaustive selector: with X = 128*b + f the normalized value in
            // 1/256 units, (X - 256 m)^2 = X^2 - 512 * (128*m*(b-m) + f*m); the
            // first product depends on (bin, dialect) only.  m <= b always,
            // because 0 is a magnitude of every dialect.
            gain16[b * 32 + d] = (uint16_t)(mag * (b - mag));
            qval[d * 64 + b] = (uint8_t)idx;
            qvalT[b * 32 + d] = (uint8_t)idx;
            qval[d * 64 + 32 + b] = (uint8_t)(8 | idx);
        }
    }
    // Two-stage selection (Sec. 3.2): range r = 8..15 keeps the dialects whose largest magnitude is r.  A range
    // that no dialect has keeps everything (the first stage is skipped).
    uint8_t* rex = blob + kOffRangeExcl;
    for (int r = 0; r < 8; ++r) {
        bool any = false;
        for (int d = 0; d < n; ++d) any = any || (fbk[8 * d + 7] == 8 + r);
        for (int d = 0; d < kMaxDialects; ++d)
            rex[r * 32 + d] = !any ? 0x00 : ((d < n && fbk[8 * d + 7] == 8 + r) ? 0x00 : 0xFF);
    }
    int32_t cnt = n;
    std::memcpy(blob + kOffCount, &cnt, 4);
}

}  // namespace fb4
