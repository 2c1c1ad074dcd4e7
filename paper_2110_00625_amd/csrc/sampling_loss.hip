// Minibatch index stream, label / index validation, and the fused
// softmax-cross-entropy + gradient kernel of the learner step.
#include "kavg_internal.h"

namespace kavg {

// ---------------------------------------------------------------------------
// Index stream.  Algorithm 1 only says "randomly sample a mini-batch of size
// B"; the draws are taken i.i.d. uniform with replacement (the xi_{k,s}^j of
// the Notations paragraph are i.i.d.).  Draw (j, t, s) is output number c+1,
// c = j*2^40 + t*2^16 + s, of SplitMix64 (Steele, Lea, Flood 2014) seeded
// with `seed`: because that generator's state is seed + i*gamma after i
// steps, any draw is computed directly from its counter.  Integer only.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t splitmix64_mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ void index_stream_kernel(int32_t* __restrict__ idx, int P, int K, int B,
                                    uint64_t seed, uint32_t t0, uint32_t N) {
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)P * K * B;
    if (e >= total) return;
    uint32_t s = (uint32_t)(e % B);
    uint32_t k = (uint32_t)((e / B) % K);
    uint64_t j = e / ((size_t)B * K);
    uint64_t c = (j << 40) | ((uint64_t)(t0 + k) << 16) | s;
    uint64_t z = splitmix64_mix(seed + (c + 1) * 0x9E3779B97F4A7C15ull);
    idx[e] = (int32_t)(z % (uint64_t)N);
}

hipError_t launch_index_stream(int32_t* idx, int P, int K, int B, uint64_t seed,
                               uint32_t t0, uint32_t N, hipStream_t st) {
    size_t total = (size_t)P * K * B;
    unsigned grid = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(index_stream_kernel, dim3(grid), dim3(256), 0, st, idx, P, K, B, seed, t0, N);
    return hipGetLastError();
}

__global__ void index_import_kernel(int32_t* __restrict__ idx, const int32_t* __restrict__ user,
                                    size_t count, uint32_t N, int* __restrict__ flag) {
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    int32_t v = user[e];
    if (v < 0 || (uint32_t)v >= N) {
        *flag = 1;                       // benign race: every writer stores the same value
        v = v < 0 ? 0 : (int32_t)(N - 1);
    }
    idx[e] = v;
}

hipError_t launch_index_import(int32_t* idx, const int32_t* user, size_t count, uint32_t N,
                               int* flag, hipStream_t st) {
    unsigned grid = (unsigned)((count + 255) / 256);
    hipLaunchKernelGGL(index_import_kernel, dim3(grid), dim3(256), 0, st, idx, user, count, N, flag);
    return hipGetLastError();
}

__global__ void label_check_kernel(const int32_t* __restrict__ y, size_t N, int C, int* __restrict__ flag) {
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    for (; e < N; e += step) {
        int32_t v = y[e];
        if (v < 0 || v >= C) *flag = 1;
    }
}

hipError_t launch_label_check(const int32_t* y, size_t N, int C, int* flag, hipStream_t st) {
    size_t want = (N + 255) / 256;
    unsigned grid = (unsigned)(want > 4096 ? 4096 : want);
    hipLaunchKernelGGL(label_check_kernel, dim3(grid), dim3(256), 0, st, y, N, C, flag);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Softmax cross-entropy and its gradient for the MEAN minibatch loss (the
// 1/B_n factor of the learner update in Algorithm 1 is applied here):
//   dZ[m][c] = (softmax(z_m)[c] - [c == y_m]) / B,   loss_m = -log softmax(z_m)[y_m].
// One 64-lane wavefront per row; lanes stride over the classes; max and sum
// are wavefront butterfly reductions, so every lane ends with the same value
// and the result does not depend on launch shape.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float x) {
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// NPL > 0: C <= 64*NPL, the row is read once and stays in NPL registers per lane (logit c = lane + 64*i);
// NPL == 0: any C, the row is read once per pass.
template <bool BF16, int NPL>
__global__ void __launch_bounds__(256)
softmax_ce_kernel(const float* __restrict__ logits, int ldz, int C, const int32_t* __restrict__ y,
                  const int32_t* __restrict__ idx, long idx_learner_stride, int B, int P,
                  void* __restrict__ dz, long dz_learner_stride, float* __restrict__ rowloss) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long)P * B) return;                       // whole wavefront leaves together
    const int j = (int)(row / B), m = (int)(row % B);
    int label = y[idx[(long)j * idx_learner_stride + m]];
    label = label < 0 ? 0 : (label >= C ? C - 1 : label); // labels were validated; never index outside
    const float* z = logits + row * ldz;
    const long dz_row = (long)j * dz_learner_stride + (long)m * ldz;
    const float invB = 1.0f / (float)B;
    auto store = [&](int c, float g) {
        if (BF16) {
            __bf16 h = (__bf16)g;
            ((uint16_t*)dz)[dz_row + c] = __builtin_bit_cast(uint16_t, h);
        } else {
            ((float*)dz)[dz_row + c] = g;
        }
    };
    if constexpr (NPL > 0) {
        float zr[NPL];
#pragma unroll
        for (int i = 0; i < NPL; ++i) { const int c = lane + 64 * i; zr[i] = c < C ? z[c] : -INFINITY; }
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NPL; ++i) mx = fmaxf(mx, zr[i]);
        mx = wave_max(mx);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < NPL; ++i) { zr[i] = lane + 64 * i < C ? expf(zr[i] - mx) : 0.f; sum += zr[i]; }
        sum = wave_sum(sum);
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int c = lane + 64 * i;
            if (c < ldz) store(c, c < C ? (zr[i] / sum - (c == label ? 1.0f : 0.0f)) * invB : 0.f);
        }
        if (lane == 0) rowloss[row] = -(z[label] - mx - logf(sum));
        return;
    }
    float mx = -INFINITY;
    for (int c = lane; c < C; c += 64) mx = fmaxf(mx, z[c]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int c = lane; c < C; c += 64) sum += expf(z[c] - mx);
    sum = wave_sum(sum);
    for (int c = lane; c < ldz; c += 64) {
        float g = 0.f;
        if (c < C) {
            float p = expf(z[c] - mx) / sum;
            g = (p - (c == label ? 1.0f : 0.0f)) * invB;
        }
        store(c, g);
    }
    if (lane == 0) rowloss[row] = -(z[label] - mx - logf(sum));
}

hipError_t launch_softmax_ce(const float* logits, int ldz, int C, const int32_t* y,
                             const int32_t* idx, long idx_learner_stride, int B, int P,
                             void* dz, long dz_learner_stride, int dz_bf16, float* rowloss, hipStream_t st) {
    long rows = (long)P * B;
    unsigned grid = (unsigned)((rows + 3) / 4);
#define KAVG_SOFTMAX(BF, NPL)                                                                             \
    hipLaunchKernelGGL((softmax_ce_kernel<BF, NPL>), dim3(grid), dim3(256), 0, st, logits, ldz, C, y, idx,  \
                       idx_learner_stride, B, P, dz, dz_learner_stride, rowloss)
    const int per_lane = (ldz + 63) / 64;
    if (dz_bf16) {
        if (per_lane <= 2) KAVG_SOFTMAX(true, 2); else if (per_lane <= 16) KAVG_SOFTMAX(true, 16); else KAVG_SOFTMAX(true, 0);
    } else {
        if (per_lane <= 2) KAVG_SOFTMAX(false, 2); else if (per_lane <= 16) KAVG_SOFTMAX(false, 16); else KAVG_SOFTMAX(false, 0);
    }
#undef KAVG_SOFTMAX
    return hipGetLastError();
}

// losses[r] = (1/B) sum_m rowloss[r][m], r = k*P + j; one wavefront per r, fixed order.
__global__ void __launch_bounds__(64)
loss_mean_kernel(const float* __restrict__ rowloss, float* __restrict__ losses, int B) {
    const int lane = threadIdx.x;
    const float* p = rowloss + (long)blockIdx.x * B;
    float s = 0.f;
    for (int m = lane; m < B; m += 64) s += p[m];
    s = wave_sum(s);
    if (lane == 0) losses[blockIdx.x] = s / (float)B;
}

hipError_t launch_loss_mean(const float* rowloss, float* losses, int KP, int B, hipStream_t st) {
    hipLaunchKernelGGL(loss_mean_kernel, dim3(KP), dim3(64), 0, st, rowloss, losses, B);
    return hipGetLastError();
}

}  // namespace kavg
