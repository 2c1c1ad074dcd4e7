// The first convolution of the learner (8 input channels, images gathered by the minibatch indices) without a
// patch matrix: forward pass and weight gradient (conv_first.hip).
#pragma once
#include "kavg_internal.h"

namespace kavg {

// Ranges of whole images the weight gradient of a learner is split into, or 0 when the kernels do not cover
// the layer (they take images 32 pixels wide whose height is a multiple of 8, 8 channels in, 32 or 64 out).
int conv_first_splits(int P, int B, int H, int W, int c_in, int c_out);

// c.out = relu(conv(images, W) + b); image n of learner j is row idx[j * idx_lstride + n] of the data set X
// ([N][H][32][8] bf16).  Reads the hi plane of the weights and both bias planes.
hipError_t conv_first_forward(const ConvCall& c, const void* X, const int32_t* idx, long idx_lstride, hipStream_t st);
// partial[(learner * splits + range)][c_out][72] and partial_bias as for the later convolutions (conv_step_kernel
// applies them); c.splits = conv_first_splits(...).  Reads c.dz and the gathered images.
hipError_t conv_first_wgrad(const ConvCall& c, const void* X, const int32_t* idx, long idx_lstride, hipStream_t st);

}  // namespace kavg
