// Convolutional layers of the learner step (KAVG_BF16): 3x3 convolutions, stride 1, zero padding 1,
// on channels-last images, as dense products on patch matrices.
//
// A layer out[n,h,w,o] = b[o] + sum_{kh,kw,c} in[n,h+kh-1,w+kw-1,c] * W[o,kh,kw,c] is the product of the
// patch matrix  Pm[(n,h,w)][(kh,kw,c)]  (B*H*W rows, 9*c_in columns) with W^T ([c_out][9*c_in], the
// layer's weights exactly as they lie in the flat parameter vector), and its gradients are the two
// other products of a dense layer on the same matrix (gemm_bf16.hip).
//
// Convolutions 2..M never write Pm out: the MFMA kernel's operand loaders form its rows on the fly
// from the images (ConvDirectLoader / ConvTransLoader: a 16-byte piece of a row is 8 channels of the
// pixel its tap points at, or zeros outside the image).  Their data gradient is the same kind of
// product on the dZ images with the taps mirrored and the weights read as [(tap, o)][c_in]
// (rotate_weights_kernel rebuilds that view from the current weights before every use), so it comes
// out of the MFMA kernel already masked by the ReLU of the layer below and rounded to bf16.
//
// The first convolution gathers its images out of the data set and has only 9*c_0 = 72 columns: its
// patch matrix is written out (im2col_kernel) and feeds the generic dense kernels.  The same explicit
// path, with the fp32 product dZ * W per (position, tap, channel) folded back onto the image by
// col2im_mask_kernel, serves every convolution when an image has 2^14 positions or more (beyond the
// range of the loaders' multiply-shift divisions).
//
// The weight gradient of a convolution has few outputs (c_out x 9 c_in) and a very long contraction;
// it is split over S ranges of positions that run as separate workgroups (the update kernel writes
// fp32 partial tiles instead of stepping the master), and conv_step_kernel adds the S partials in
// ascending order and takes the SGD step of Algorithm 1 on the master's two planes (split.h).
// Between the last convolution and the MLP sits the mean over the H*W positions.
//
// Images 32 pixels wide do not take these paths where the tile kernels cover the layer (conv_first.hip,
// conv_direct.hip, conv_wgrad.hip: the image rows a workgroup needs are held in LDS and every tap reads them
// at a shifted pixel); what is here serves every other shape, and the pooling and the master step for all.
#include "kavg_internal.h"
#include "split.h"
#include "conv_pool.h"

namespace kavg {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t bf16_bits(float x) {
    __bf16 h = (__bf16)x;                         // round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)bf16_bits(lo) | ((uint32_t)bf16_bits(hi) << 16);
}

// one lane per 16-byte piece (8 channels) of the patch matrix
__global__ void __launch_bounds__(256)
im2col_kernel(const uint16_t* __restrict__ in, size_t in_lstride, const int32_t* __restrict__ gather, long gstride,
              uint16_t* __restrict__ out, int B, int H, int W, int c, size_t total) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int c8 = c / 8;
    size_t r = e;
    const int cc = (int)(r % c8); r /= c8;
    const int tap = (int)(r % 9); r /= 9;
    const int w = (int)(r % W); r /= W;
    const int h = (int)(r % H); r /= H;
    const int n = (int)(r % B);
    const int j = (int)(r / B);
    const int hh = h + tap / 3 - 1, ww = w + tap % 3 - 1;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (hh >= 0 && hh < H && ww >= 0 && ww < W) {
        const uint16_t* img = gather ? in + (size_t)gather[(long)j * gstride + n] * ((size_t)H * W * c)
                                     : in + (size_t)j * in_lstride + (size_t)n * H * W * c;
        v = *(const u32x4*)(img + ((size_t)hh * W + ww) * c + cc * 8);
    }
    *(u32x4*)(out + e * 8) = v;
}

// dprev[j,n,h,w,c] = bf16( [act[j,n,h,w,c] > 0] * sum_{kh,kw} draw[j][(n,h-kh+1,w-kw+1)][(kh,kw,c)] ), 8 channels per lane
__global__ void __launch_bounds__(256)
col2im_mask_kernel(const float* __restrict__ draw, const uint16_t* __restrict__ act, uint16_t* __restrict__ dprev,
                   int B, int H, int W, int c, size_t total) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int c8 = c / 8;
    size_t r = e;
    const int cc = (int)(r % c8); r /= c8;
    const int w = (int)(r % W); r /= W;
    const int h = (int)(r % H); r /= H;
    const size_t img = r;                                     // j*B + n
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {                       // ascending taps: fixed summation order
        const int ph = h - (tap / 3 - 1), pw = w - (tap % 3 - 1);      // the output position whose patch holds this pixel at `tap`
        if (ph < 0 || ph >= H || pw < 0 || pw >= W) continue;
        const float* p = draw + ((img * H + ph) * W + pw) * (size_t)(9 * c) + (size_t)tap * c + cc * 8;
        const f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
        s[0] += a.x; s[1] += a.y; s[2] += a.z; s[3] += a.w; s[4] += b.x; s[5] += b.y; s[6] += b.z; s[7] += b.w;
    }
    const u32x4 m = *(const u32x4*)(act + e * 8);
    u32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        o[q] = pack2((m[q] & 0x7FFFu) ? s[2 * q] : 0.f, (m[q] & 0x7FFF0000u) ? s[2 * q + 1] : 0.f);
    *(u32x4*)(dprev + e * 8) = o;
}

// pooled[j,n,c] = bf16(mean over the H*W positions).  One workgroup per image: a lane owns 8 channels and every
// G-th position (G = 256 / (c/8) position groups, 16-byte loads), the G partial sums of a channel meet in LDS and
// are added in ascending group order -- a fixed summation order.
__global__ void __launch_bounds__(256)
pool_forward_kernel(const uint16_t* __restrict__ act, uint16_t* __restrict__ pooled, int HW, int c, float inv) {
    __shared__ float part[256 * 8];
    const int c8 = c / 8;                                     // lanes per position (<= 256: c <= 2048)
    const int G = 256 / c8;                                   // position groups
    const int tid = threadIdx.x, cc = tid % c8, g = tid / c8;
    const size_t img = blockIdx.x;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (g < G) {
        const uint16_t* p = act + img * (size_t)HW * c + cc * 8;
#pragma unroll 4
        for (int i = g; i < HW; i += G) {
            const u32x4 v = *(const u32x4*)(p + (size_t)i * c);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                s[2 * q] += __builtin_bit_cast(float, v[q] << 16);
                s[2 * q + 1] += __builtin_bit_cast(float, v[q] & 0xFFFF0000u);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) part[(g * c8 + cc) * 8 + e] = s[e];
    }
    __syncthreads();
    for (int ch = tid; ch < c; ch += 256) {
        float t = 0.f;
        for (int g2 = 0; g2 < G; ++g2) t += part[(g2 * c8 + ch / 8) * 8 + ch % 8];
        pooled[img * c + ch] = bf16_bits(t * inv);
    }
}

// dz[j,n,hw,c] = bf16( [act > 0] * dpool[j,n,c] / (H*W) ), 8 channels per lane
__global__ void __launch_bounds__(256)
pool_backward_kernel(const uint16_t* __restrict__ dpool, const uint16_t* __restrict__ act, uint16_t* __restrict__ dz,
                     int HW, int c, float inv, size_t total) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int c8 = c / 8;
    const int cc = (int)(e % c8);
    const size_t img = e / c8 / HW;
    const u32x4 g = *(const u32x4*)(dpool + img * c + cc * 8);
    const u32x4 m = *(const u32x4*)(act + e * 8);
    *(u32x4*)(dz + e * 8) = pool_grad_piece(m, g, inv);
}

// W[j][e] -= lr * sum_s partial[(j*S+s)][e]  and  b[j][r] -= lr * sum_s pbias[(j*S+s)][r]  on the master's planes
__global__ void __launch_bounds__(256)
conv_step_kernel(uint16_t* whi, uint16_t* wlo, uint16_t* bhi, uint16_t* blo, size_t lstride, const float* __restrict__ partial,
                 const float* __restrict__ pbias, int S, int n_w, int n_b, float lr) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int j = blockIdx.y;
    if (e >= n_w + n_b) return;
    const bool is_w = e < n_w;
    const int i = is_w ? e : e - n_w;
    const float* p = is_w ? partial + (size_t)j * S * n_w + i : pbias + (size_t)j * S * n_b + i;
    const size_t step = is_w ? (size_t)n_w : (size_t)n_b;
    float s = 0.f;
    for (int q = 0; q < S; ++q) s += p[(size_t)q * step];
    uint16_t* hi = (is_w ? whi : bhi) + (size_t)j * lstride + i;
    uint16_t* lo = (is_w ? wlo : blo) + (size_t)j * lstride + i;
    const float v = __builtin_bit_cast(float, split_join(*hi, *lo)) - lr * s;
    *hi = (uint16_t)split_hi(__builtin_bit_cast(uint32_t, v));
    *lo = (uint16_t)split_lo(__builtin_bit_cast(uint32_t, v));
}

// one lane per 16-byte piece of the rotated weights
__global__ void __launch_bounds__(256)
rotate_weights_kernel(const uint16_t* __restrict__ whi, size_t w_lstride, uint16_t* __restrict__ wrot, size_t wrot_lstride,
                      int c_out, int c_in, size_t per_learner) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= per_learner) return;
    const int j = blockIdx.y;
    const int c8 = c_in / 8;
    size_t r = e;
    const int cc = (int)(r % c8); r /= c8;
    const int o = (int)(r % c_out);
    const int tap = (int)(r / c_out);
    const u32x4 v = *(const u32x4*)(whi + (size_t)j * w_lstride + ((size_t)o * 9 + tap) * c_in + cc * 8);
    *(u32x4*)(wrot + (size_t)j * wrot_lstride + e * 8) = v;
}

unsigned blocks(size_t total) { return (unsigned)((total + 255) / 256); }

}  // namespace

hipError_t launch_im2col(const void* in, size_t in_lstride, const int32_t* gather, long gstride, void* patches,
                         int P, int B, int H, int W, int c, hipStream_t st) {
    const size_t total = (size_t)P * B * H * W * 9 * (c / 8);
    hipLaunchKernelGGL(im2col_kernel, dim3(blocks(total)), dim3(256), 0, st, (const uint16_t*)in, in_lstride, gather, gstride,
                       (uint16_t*)patches, B, H, W, c, total);
    return hipGetLastError();
}

hipError_t launch_col2im_mask(const float* draw, const void* act, void* dprev, int P, int B, int H, int W, int c,
                              hipStream_t st) {
    const size_t total = (size_t)P * B * H * W * (c / 8);
    hipLaunchKernelGGL(col2im_mask_kernel, dim3(blocks(total)), dim3(256), 0, st, draw, (const uint16_t*)act, (uint16_t*)dprev,
                       B, H, W, c, total);
    return hipGetLastError();
}

hipError_t launch_pool_forward(const void* act, void* pooled, int P, int B, int HW, int c, hipStream_t st) {
    if (c < 8 || c % 8 != 0 || c > 2048) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pool_forward_kernel, dim3((unsigned)((size_t)P * B)), dim3(256), 0, st, (const uint16_t*)act, (uint16_t*)pooled, HW, c,
                       1.0f / (float)HW);
    return hipGetLastError();
}

hipError_t launch_pool_backward(const void* dpool, const void* act, void* dz, int P, int B, int HW, int c, hipStream_t st) {
    const size_t total = (size_t)P * B * HW * (c / 8);
    hipLaunchKernelGGL(pool_backward_kernel, dim3(blocks(total)), dim3(256), 0, st, (const uint16_t*)dpool, (const uint16_t*)act,
                       (uint16_t*)dz, HW, c, 1.0f / (float)HW, total);
    return hipGetLastError();
}

hipError_t launch_rotate_weights(const uint16_t* whi, size_t w_lstride, uint16_t* wrot, size_t wrot_lstride, int P, int c_out,
                                 int c_in, hipStream_t st) {
    const size_t per_learner = (size_t)9 * c_out * (c_in / 8);
    hipLaunchKernelGGL(rotate_weights_kernel, dim3(blocks(per_learner), P), dim3(256), 0, st, whi, w_lstride, wrot, wrot_lstride,
                       c_out, c_in, per_learner);
    return hipGetLastError();
}

hipError_t launch_conv_step(uint16_t* whi, uint16_t* wlo, uint16_t* bhi, uint16_t* blo, size_t lstride, const float* partial,
                            const float* pbias, int P, int S, int n_w, int n_b, float lr, hipStream_t st) {
    hipLaunchKernelGGL(conv_step_kernel, dim3(blocks((size_t)n_w + n_b), P), dim3(256), 0, st, whi, wlo, bhi, blo, lstride,
                       partial, pbias, S, n_w, n_b, lr);
    return hipGetLastError();
}

}  // namespace kavg
