// Gradient of the mean over the positions, eight channels at a time: what the layer above hands the last
// convolution is dpool[image][channel]; the gradient w.r.t. that convolution's pre-activation at a position is
// bf16( [act > 0] * dpool / (H W) ).  Used by pool_backward_kernel and by the kernels that form these values
// while loading, instead of reading them from a buffer.
#pragma once
#include <stdint.h>

namespace kavg {

typedef uint32_t pool_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pool_pack2(float lo, float hi) {
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;          // round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

// m: eight activations (ReLU outputs, bf16 pairs); g: the eight channels' dpool; inv = 1 / (H W)
__device__ __forceinline__ pool_u32x4 pool_grad_piece(pool_u32x4 m, pool_u32x4 g, float inv) {
    pool_u32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float g0 = __builtin_bit_cast(float, g[q] << 16) * inv, g1 = __builtin_bit_cast(float, g[q] & 0xFFFF0000u) * inv;
        // stored activations are never negative: positive <=> non-zero magnitude
        o[q] = pool_pack2((m[q] & 0x7FFFu) ? g0 : 0.f, (m[q] & 0x7FFF0000u) ? g1 : 0.f);
    }
    return o;
}

}  // namespace kavg
