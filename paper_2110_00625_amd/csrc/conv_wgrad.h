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
hipError_t conv_wgrad_halo(const ConvCall& c, hipStream_t st);

}  // namespace kavg
