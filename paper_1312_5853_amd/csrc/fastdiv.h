// Division of a 31-bit unsigned numerator by a run-time constant through one
// 64-bit multiply and a shift.  Host code builds the constant; device code
// applies it where a per-element `/` would cost ~25 VALU instructions.
//
// For 0 <= n < 2^31 and 1 <= d < 2^31, with L = ceil(log2 d) and
// m = ceil(2^(31+L) / d) (which fits in 32 bits), floor(n / d) equals
// (n * m) >> (31 + L): m*d lies in [2^(31+L), 2^(31+L) + 2^L], the condition
// of Granlund & Montgomery's round-up method for 31-bit numerators.
#ifndef CONVNET_FASTDIV_H
#define CONVNET_FASTDIV_H

#include <stdint.h>

#if defined(__HIPCC__)
#define CONVNET_HD __host__ __device__ __forceinline__
#else
#define CONVNET_HD inline
#endif

struct FastDiv {
    uint32_t mul;
    uint32_t shift;   // 31 + L
    uint32_t d;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    if (d == 0) d = 1;
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    const uint64_t two = 1ull << (31 + L);
    f.mul = (uint32_t)((two + d - 1) / d);
    f.shift = 31 + L;
    f.d = d;
    return f;
}

CONVNET_HD uint32_t fastdiv(uint32_t n, const FastDiv f)
{
    return (uint32_t)(((uint64_t)n * f.mul) >> f.shift);
}

#endif
