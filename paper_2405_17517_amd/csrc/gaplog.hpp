// Arithmetic of the "gap" mask stream, shared by the host (per-segment scale) and the kernel
// (one logarithm per draw).  log2 is a fixed sequence of IEEE double operations so that every
// implementation of the stream produces the same bits:
//   x = m * 2^e with m in (sqrt(1/2), sqrt(2)];  ln m = 2 atanh(s), s = (m-1)/(m+1), odd series to s^21.
// Inversion of the geometric law: the distance to the next selected coordinate is
//   1 + floor(log2(u) / log2(1-p)),  u uniform on (0,1],  so that  P(distance > k) = (1-p)^k.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

namespace wash {

#pragma clang fp contract(off)

__host__ __device__ inline double gap_log2(double x)
{
    uint64_t bits;
    memcpy(&bits, &x, sizeof(bits));
    int e = static_cast<int>((bits >> 52) & 0x7FFu) - 1023;
    bits = (bits & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull;
    double m;
    memcpy(&m, &bits, sizeof(m));
    if (m > 1.4142135623730951) {
        m = m * 0.5;
        e += 1;
    }
    const double s = (m - 1.0) / (m + 1.0);
    const double z = s * s;
    double poly = 1.0 / 21.0;
    poly = poly * z + 1.0 / 19.0;
    poly = poly * z + 1.0 / 17.0;
    poly = poly * z + 1.0 / 15.0;
    poly = poly * z + 1.0 / 13.0;
    poly = poly * z + 1.0 / 11.0;
    poly = poly * z + 1.0 / 9.0;
    poly = poly * z + 1.0 / 7.0;
    poly = poly * z + 1.0 / 5.0;
    poly = poly * z + 1.0 / 3.0;
    poly = poly * z + 1.0;
    const double t = s * poly;
    const double ln_m = t + t;
    return static_cast<double>(e) + ln_m * 1.4426950408889634;
}

// A probability so small that 1 - p rounds to 1 has no usable log2(1 - p): such a segment selects
// nothing (the Bernoulli(p) law of Eq. 3 is then met to within 2^-54 per coordinate).
inline bool gap_never_selects(double p) { return p == 0.0 || 1.0 - p == 1.0; }

// 1 / log2(1-p) for 2^-54 < p < 1; 0 for p = 1 (every distance is 1).
inline double gap_scale(double p)
{
    if (p >= 1.0) return 0.0;
    return 1.0 / gap_log2(1.0 - p);
}

// Distance (>= 1, capped at 2048) from a 53-bit uniform integer U and the segment scale.
__device__ __forceinline__ uint32_t gap_distance(uint64_t U, double scale)
{
    const double L = gap_log2(static_cast<double>(U + 1u)) - 53.0;   // log2 of (U+1)/2^53, in [-53, 0]
    double q = L * scale;                                            // >= 0 for the scale of a probability
    if (!(q < 2047.0)) q = 2047.0;                                   // also NaN
    if (q < 0.0) q = 0.0;
    return 1u + static_cast<uint32_t>(q);
}

constexpr uint32_t kGapPiece = 1024;   // the walk restarts at every multiple of this many coordinates

}  // namespace wash
