// fp32 path of the learner step (KAVG_FP32): forward, backward-data and the
// fused weight-gradient + SGD update, batched over learners (grid.z).
//
// One generic LDS-tiled kernel computes   O[r][c] = sum_k R(r,k) * Cm(c,k)
// for operands given by (row stride, contraction stride, optional row gather),
// with three epilogues.  Products and sums are plain fp32 FMAs (no reduced
// precision matrix path), contraction in ascending k inside each thread, so
// results are deterministic and independent of the grid.
//
//   forward        r = sample, c = output unit, k = input unit
//                  O = act(A_{l-1} W_l^T + b_l)
//   backward-data  r = sample, c = input unit,  k = output unit
//                  dZ_{l-1} = (dZ_l W_l) * [A_{l-1} > 0]
//   update         r = output unit, c = input unit, k = sample
//                  W_l <- W_l - lr * dZ_l^T A_{l-1};  b_l <- b_l - lr * colsum(dZ_l)
//                  (the learner update of Algorithm 1; 1/B already sits in dZ_L)
#include "kavg_internal.h"

namespace kavg {

namespace {

constexpr int TILE = 64;   // output tile is TILE x TILE
constexpr int BK = 16;     // contraction slice
constexpr int PADW = TILE + 4;

enum { EPI_FWD = 0, EPI_BWD = 1, EPI_UPD = 2 };

struct Operand {
    const float* base;      // learner 0
    size_t learner_stride;  // elements between learners
    long ld_x;              // stride of the row (r or c) index
    long ld_k;              // stride of the contraction index
    const int32_t* gather;  // optional: replaces the strided index by a looked-up row
    long gather_stride;     // per learner
    int gather_on_k;        // 0: gather applies to x, 1: to k
};

struct Args {
    Operand R, C;
    int nR, nC, nK;
    // epilogue
    float* out;  size_t out_stride;  int ld_out;       // FWD/BWD output, UPD: master weights
    const float* bias; size_t bias_stride;             // FWD: bias; UPD: unused
    float* bias_rw;                                    // UPD: bias to update (stride = bias_stride)
    const float* mask; size_t mask_stride; int ld_mask;// BWD: previous activations
    const float* dz; size_t dz_stride; int ld_dz;      // UPD: dZ for the bias gradient [B][ld_dz]
    int relu;
    float lr;
};

__device__ __forceinline__ float fetch(const Operand& o, int learner, int x, int k) {
    const float* p = o.base + (size_t)learner * o.learner_stride;
    if (o.gather) {
        const int32_t* g = o.gather + (long)learner * o.gather_stride;
        if (o.gather_on_k) return p[(long)g[k] * o.ld_k + (long)x * o.ld_x];
        return p[(long)g[x] * o.ld_x + (long)k * o.ld_k];
    }
    return p[(long)x * o.ld_x + (long)k * o.ld_k];
}

template <int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(Args a) {
    __shared__ float Rs[BK][PADW];
    __shared__ float Cs[BK][PADW];
    const int tid = threadIdx.x;
    const int learner = blockIdx.z;
    const int r0 = blockIdx.y * TILE, c0 = blockIdx.x * TILE;
    const int tx = tid & 15, ty = tid >> 4;
    const bool r_kfast = (a.R.ld_k == 1 && !(a.R.gather && a.R.gather_on_k));
    const bool c_kfast = (a.C.ld_k == 1 && !(a.C.gather && a.C.gather_on_k));

    float acc[4][4] = {};
    for (int k0 = 0; k0 < a.nK; k0 += BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + 256 * i;
            int x, k;
            if (r_kfast) { x = e / BK; k = e % BK; } else { x = e % TILE; k = e / TILE; }
            float val = 0.f;
            if (r0 + x < a.nR && k0 + k < a.nK) val = fetch(a.R, learner, r0 + x, k0 + k);
            Rs[k][x] = val;
            if (c_kfast) { x = e / BK; k = e % BK; } else { x = e % TILE; k = e / TILE; }
            val = 0.f;
            if (c0 + x < a.nC && k0 + k < a.nK) val = fetch(a.C, learner, c0 + x, k0 + k);
            Cs[k][x] = val;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float rv[4], cv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { rv[i] = Rs[k][ty * 4 + i]; cv[i] = Cs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(rv[i], cv[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + ty * 4 + i;
        if (r >= a.nR) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = c0 + tx * 4 + j;
            if (c >= a.nC) continue;
            if (EPI == EPI_FWD) {
                float z = acc[i][j] + a.bias[(size_t)learner * a.bias_stride + c];
                if (a.relu) z = fmaxf(z, 0.f);
                a.out[(size_t)learner * a.out_stride + (size_t)r * a.ld_out + c] = z;
            } else if (EPI == EPI_BWD) {
                const float m = a.mask[(size_t)learner * a.mask_stride + (size_t)r * a.ld_mask + c];
                a.out[(size_t)learner * a.out_stride + (size_t)r * a.ld_out + c] = m > 0.f ? acc[i][j] : 0.f;
            } else {
                float* w = a.out + (size_t)learner * a.out_stride + (size_t)r * a.ld_out + c;
                *w = *w - a.lr * acc[i][j];
            }
        }
    }

    if (EPI == EPI_UPD && blockIdx.x == 0 && tid < TILE) {
        // bias gradient of this tile's output units: column sums of dZ_l over the batch
        const int r = r0 + tid;
        if (r < a.nR) {
            const float* dz = a.dz + (size_t)learner * a.dz_stride;
            float s = 0.f;
            for (int m = 0; m < a.nK; ++m) s += dz[(size_t)m * a.ld_dz + r];
            float* b = a.bias_rw + (size_t)learner * a.bias_stride + r;
            *b = *b - a.lr * s;
        }
    }
}

template <int EPI>
hipError_t run(const Args& a, int P, hipStream_t st) {
    dim3 grid((a.nC + TILE - 1) / TILE, (a.nR + TILE - 1) / TILE, P);
    hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t f32_forward(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const float*)c.in, c.in_stride, c.ld_in, 1, c.gather, c.gather_stride, 0};
    if (c.gather) a.R.learner_stride = 0;               // all learners read the one data set
    a.C = {c.w, c.w_stride, c.d_in, 1, nullptr, 0, 0};
    a.nR = c.B; a.nC = c.d_out; a.nK = c.d_in;
    a.out = (float*)c.out; a.out_stride = c.out_stride; a.ld_out = c.ld_out;
    a.bias = c.b; a.bias_stride = c.w_stride;
    a.relu = c.relu;
    return run<EPI_FWD>(a, c.P, st);
}

hipError_t f32_backward_data(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const float*)c.dz, c.dz_stride, c.ld_dz, 1, nullptr, 0, 0};
    a.C = {c.w, c.w_stride, 1, c.d_in, nullptr, 0, 0};  // Cm(c = input unit, k = output unit) = W[k][c]
    a.nR = c.B; a.nC = c.d_in; a.nK = c.d_out;
    a.out = (float*)c.dz_prev; a.out_stride = c.dz_prev_stride; a.ld_out = c.ld_in;
    a.mask = (const float*)c.in; a.mask_stride = c.in_stride; a.ld_mask = c.ld_in;
    return run<EPI_BWD>(a, c.P, st);
}

hipError_t f32_update(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const float*)c.dz, c.dz_stride, 1, c.ld_dz, nullptr, 0, 0};        // R(r = unit, k = sample) = dZ[k][r]
    a.C = {(const float*)c.in, c.in_stride, 1, c.ld_in, c.gather, c.gather_stride, 1};  // Cm(c, k = sample) = A[k][c]
    if (c.gather) a.C.learner_stride = 0;
    a.nR = c.d_out; a.nC = c.d_in; a.nK = c.B;
    a.out = c.w; a.out_stride = c.w_stride; a.ld_out = c.d_in;
    a.bias_rw = c.b; a.bias_stride = c.w_stride;
    a.dz = (const float*)c.dz; a.dz_stride = c.dz_stride; a.ld_dz = c.ld_dz;
    a.lr = c.lr;
    return run<EPI_UPD>(a, c.P, st);
}

}  // namespace kavg
