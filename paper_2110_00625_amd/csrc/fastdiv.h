// Division by a runtime constant as a multiply and a shift, for the index arithmetic of the implicit
// convolution loaders (position -> (image, row, column), contraction index -> (tap, channel)).
//
// For a divisor 2 <= d < 2^14:  s = 31 + ceil(log2 d),  m = floor(2^s / d) + 1 < 2^32  (d = 1: m = 2^31, s = 31).
// Then for every n < 2^30:  floor(n / d) = (n * m) >> s, because n * m / 2^s = n/d + n * (m d - 2^s) / (d 2^s), where
// 0 < m d - 2^s <= d, so the excess is below n / 2^s < 1/d: too small to reach the next integer.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define KAVG_FD __host__ __device__ __forceinline__
#else
#define KAVG_FD inline
#endif

namespace kavg {

KAVG_FD uint32_t fastdiv(uint32_t n, uint32_t m, int s) { return (uint32_t)(((uint64_t)n * m) >> s); }

inline void fastdiv_make(uint32_t d, uint32_t* m, int* s) {
    if (d <= 1) { *m = 0x80000000u; *s = 31; return; }       // n * 2^31 >> 31 = n
    int L = 0;
    while ((1u << L) < d) ++L;
    *s = 31 + L;
    *m = (uint32_t)(((uint64_t)1 << *s) / d) + 1u;           // d > 2^(L-1), so 2^s / d < 2^32
}

}  // namespace kavg
