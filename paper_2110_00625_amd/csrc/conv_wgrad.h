// Weight gradient of a 3x3 convolution with all nine taps served from one LDS tile (conv_wgrad.hip).
#pragma once
#include "kavg_internal.h"

namespace kavg {

// Number of ranges of whole images a learner's positions are split into (each a workgroup), or 0 when the
// kernel does not cover the shape (it takes images 32 pixels wide of even height, 32 or 64 input channels,
// 32, 64 or 128 output channels).
int conv_wgrad_halo_splits(int P, int B, int H, int W, int c_in, int c_out);

// partial[(learner * splits + range)][c_out][9 c_in] = sum over the range's positions of dZ^T patches (fp32), and
// the column sums of dZ in partial_bias; c.splits = conv_wgrad_halo_splits(...).  Reads c.dz and c.in.
// dpool != null (the last convolution, below the mean over the positions): c.dz is not read; dZ is formed while
// loading from the layer's own activations c.out and dpool [P][B][c_out] (bf16), as pool_backward_kernel would.
// Needs c.B / c.splits <= conv_wgrad_halo_pool_images() (the dpool rows of a workgroup's images are kept in LDS).
hipError_t conv_wgrad_halo(const ConvCall& c, const void* dpool, hipStream_t st);
int conv_wgrad_halo_pool_images();

}  // namespace kavg
