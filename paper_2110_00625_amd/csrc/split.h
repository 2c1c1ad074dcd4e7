// Split storage of an fp32 master parameter (mixed-precision mode).
//
// The learners' fp32 parameters are kept as two 16-bit planes:
//   hi = the bf16 value the matrix products use: the fp32 pattern plus half a unit of its 16th bit,
//        cut to the top 16 bits (nearest, ties away from zero);
//   lo = the low 16 bits of the fp32 pattern, unchanged.
// The pair determines the fp32 value exactly: its top 16 bits are hi, minus one when the
// rounding went up, which is the case exactly when lo >= 0x8000.  So the "bf16 shadow" of the
// weights is not a copy next to the master but one half of it: a forward pass reads 2 bytes per
// weight, an update reads and writes 4, and nothing is stored twice.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define KAVG_HD __host__ __device__ __forceinline__
#else
#define KAVG_HD inline
#endif

namespace kavg {

KAVG_HD uint32_t split_hi(uint32_t f32_bits) { return ((f32_bits + 0x8000u) >> 16) & 0xFFFFu; }
KAVG_HD uint32_t split_lo(uint32_t f32_bits) { return f32_bits & 0xFFFFu; }
KAVG_HD uint32_t split_join(uint32_t hi, uint32_t lo) { return ((hi - (lo >> 15)) << 16) | lo; }

// two parameters at once: hi2 / lo2 hold elements (e, e+1) in their (low, high) halves
KAVG_HD void split_join2(uint32_t hi2, uint32_t lo2, uint32_t& bits0, uint32_t& bits1) {
    bits0 = split_join(hi2 & 0xFFFFu, lo2 & 0xFFFFu);
    bits1 = split_join(hi2 >> 16, lo2 >> 16);
}
KAVG_HD void split_pack2(uint32_t bits0, uint32_t bits1, uint32_t& hi2, uint32_t& lo2) {
    hi2 = split_hi(bits0) | (split_hi(bits1) << 16);
    lo2 = split_lo(bits0) | (bits1 << 16);
}

}  // namespace kavg
