// The meta level of Algorithm 1 as one bandwidth-bound pass:
//     a = (1/P) sum_j w^j;  d = a - w~;  v <- mu v + d;  w~ <- w~ + v;  w^j <- w~ for all j.
// a and d never reach memory.  The displacement is formed as
//     d = (1/P) sum_j (w^j - w~),
// which equals a - w~ in exact arithmetic, keeps the small quantity d at full
// fp32 precision, and is exactly zero when all replicas equal w~ (so lr = 0
// leaves every parameter bit-identical for any P).
//
// Traffic per parameter and pass: read P replicas + w~ + v, write w~ + v + P
// replicas = (2P+4)*4 bytes (+2P bytes when bf16 shadows are refreshed).
// Each lane owns four consecutive parameters (16-byte accesses); the P replica
// loads are issued UNROLL at a time so that many are in flight per lane.
// Replica loads and stores are streaming (non-temporal): nothing is reused.
#include "kavg_internal.h"

namespace kavg {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t to_bf16_bits(float x) {
    __bf16 h = (__bf16)x;                 // round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ void meta_scalar_element(float* w_tilde, float* v, float* reps, size_t stride,
                                                    uint16_t* shadow, size_t sstride, int P, size_t e,
                                                    float mu, float invP) {
    const float wt = w_tilde[e];
    float acc = 0.f;
    for (int j = 0; j < P; ++j) acc += reps[(size_t)j * stride + e] - wt;
    const float vn = mu * v[e] + acc * invP;
    const float wn = wt + vn;
    v[e] = vn;
    w_tilde[e] = wn;
    for (int j = 0; j < P; ++j) reps[(size_t)j * stride + e] = wn;
    if (shadow) {
        const uint16_t h = to_bf16_bits(wn);
        for (int j = 0; j < P; ++j) shadow[(size_t)j * sstride + e] = h;
    }
}

template <bool SHADOW, int UNROLL, bool SHADOW_CACHED>
__global__ void __launch_bounds__(256)
meta_update_vec_kernel(float* __restrict__ w_tilde, float* __restrict__ v, float* __restrict__ reps,
                       size_t stride, uint16_t* __restrict__ shadow, size_t sstride, int P,
                       size_t n4, size_t n, float mu, float invP) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const f32x4 wt = ((const f32x4*)w_tilde)[i];
        const f32x4 vo = ((const f32x4*)v)[i];
        const f32x4* r = (const f32x4*)reps + i;
        const size_t s4 = stride / 4;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        int j = 0;
        for (; j + UNROLL <= P; j += UNROLL) {
            f32x4 t[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) t[u] = __builtin_nontemporal_load(r + (size_t)(j + u) * s4);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) acc += t[u] - wt;
        }
        for (; j < P; ++j) acc += __builtin_nontemporal_load(r + (size_t)j * s4) - wt;
        const f32x4 vn = mu * vo + acc * invP;
        const f32x4 wn = wt + vn;
        ((f32x4*)v)[i] = vn;
        ((f32x4*)w_tilde)[i] = wn;
        f32x4* o = (f32x4*)reps + i;
        for (int jj = 0; jj < P; ++jj) __builtin_nontemporal_store(wn, o + (size_t)jj * s4);
        if (SHADOW) {
            u16x4 h = {to_bf16_bits(wn.x), to_bf16_bits(wn.y), to_bf16_bits(wn.z), to_bf16_bits(wn.w)};
            u16x4* so = (u16x4*)shadow + i;
            const size_t ss4 = sstride / 4;
            // The shadows are what the next forward pass reads: when they all fit in the memory-side
            // cache they are written with ordinary stores and stay there (the replicas above, read
            // again only by the updates, always bypass it).
            if (SHADOW_CACHED) { for (int jj = 0; jj < P; ++jj) so[(size_t)jj * ss4] = h; }
            else { for (int jj = 0; jj < P; ++jj) __builtin_nontemporal_store(h, so + (size_t)jj * ss4); }
        }
    } else {
        const size_t e = 4 * n4 + (i - n4);               // ragged tail: at most 3 parameters
        if (e < n) meta_scalar_element(w_tilde, v, reps, stride, SHADOW ? shadow : nullptr, sstride, P, e, mu, invP);
    }
}

__global__ void __launch_bounds__(256)
meta_update_scalar_kernel(float* w_tilde, float* v, float* reps, size_t stride, uint16_t* shadow,
                          size_t sstride, int P, size_t n, float mu, float invP) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n) meta_scalar_element(w_tilde, v, reps, stride, shadow, sstride, P, e, mu, invP);
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

hipError_t launch_meta_update(float* w_tilde, float* v, float* reps, size_t stride,
                              uint16_t* shadow, size_t sstride, int P, size_t n, float mu,
                              int shadow_cached, hipStream_t st) {
    const float invP = 1.0f / (float)P;
    bool vec = aligned16(w_tilde) && aligned16(v) && aligned16(reps) && (stride % 4 == 0);
    if (shadow) vec = vec && (((uintptr_t)shadow & 7) == 0) && (sstride % 4 == 0);
    if (vec) {
        const size_t n4 = n / 4;
        const size_t threads = n4 + (n - 4 * n4);
        const unsigned grid = (unsigned)((threads + 255) / 256);
        if (shadow && shadow_cached)
            hipLaunchKernelGGL((meta_update_vec_kernel<true, 16, true>), dim3(grid), dim3(256), 0, st, w_tilde, v,
                               reps, stride, shadow, sstride, P, n4, n, mu, invP);
        else if (shadow)
            hipLaunchKernelGGL((meta_update_vec_kernel<true, 16, false>), dim3(grid), dim3(256), 0, st, w_tilde, v,
                               reps, stride, shadow, sstride, P, n4, n, mu, invP);
        else
            hipLaunchKernelGGL((meta_update_vec_kernel<false, 16, false>), dim3(grid), dim3(256), 0, st, w_tilde, v,
                               reps, stride, shadow, sstride, P, n4, n, mu, invP);
    } else {
        const unsigned grid = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(meta_update_scalar_kernel, dim3(grid), dim3(256), 0, st, w_tilde, v, reps,
                           stride, shadow, sstride, P, n, mu, invP);
    }
    return hipGetLastError();
}

// "set w^j = w~_n" for every learner (first round, or after a state restore).
__global__ void __launch_bounds__(256)
broadcast_kernel(const float* __restrict__ w_tilde, float* __restrict__ reps, size_t stride,
                 uint16_t* __restrict__ shadow, size_t sstride, int P, size_t n) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const float w = w_tilde[e];
    for (int j = 0; j < P; ++j) reps[(size_t)j * stride + e] = w;
    if (shadow) {
        const uint16_t h = to_bf16_bits(w);
        for (int j = 0; j < P; ++j) shadow[(size_t)j * sstride + e] = h;
    }
}

hipError_t launch_broadcast(const float* w_tilde, float* reps, size_t stride, uint16_t* shadow,
                            size_t sstride, int P, size_t n, hipStream_t st) {
    const unsigned grid = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(broadcast_kernel, dim3(grid), dim3(256), 0, st, w_tilde, reps, stride, shadow,
                       sstride, P, n);
    return hipGetLastError();
}

}  // namespace kavg
