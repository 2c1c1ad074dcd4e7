// 3x3 convolution, forward and data gradient, on image tiles held in LDS (conv_direct.hip).
#pragma once
#include "kavg_internal.h"

namespace kavg {

// Whether the tile kernels cover a layer: images 32 pixels wide whose height is a multiple of 8;
// forward: 32, 64 or 128 channels in and out; data gradient: 32, 64 or 128 out, 32 or 64 in.
bool conv_direct_ok(int H, int W, int c_in, int c_out, bool backward);

// c.out = relu(conv(c.in, W) + b) as bf16 images; reads the hi plane of the weights and both bias planes.
hipError_t conv_direct_forward(const ConvCall& c, hipStream_t st);
// c.dz_in = [c.in > 0] * (transposed convolution of c.dz with W), bf16; reads the hi plane of the weights
// directly (no rotated copy needed).  dpool != null (the last convolution, below the mean over the positions):
// c.dz is not read; the gradient images are formed while loading from the layer's own activations c.out and
// dpool [P][B][c_out] (bf16), as pool_backward_kernel would.
hipError_t conv_direct_backward_data(const ConvCall& c, const void* dpool, hipStream_t st);

}  // namespace kavg
