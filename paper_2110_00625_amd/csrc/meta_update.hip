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
// Each lane owns four consecutive parameters (16-byte accesses), on long vectors
// eight such pieces 4 KB apart; the replica loads are issued sixteen at a time so
// that many are in flight per lane.
// Replica loads and stores are streaming (non-temporal): nothing is reused.
#include "kavg_internal.h"
#include "split.h"

namespace kavg {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t to_bf16_bits(float x) {     // weights: nearest, ties away from zero
    return (uint16_t)split_hi(__builtin_bit_cast(uint32_t, x));
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

// V: 16-byte pieces per lane, 256 lanes apart, so that a workgroup covers V*4 KB of consecutive
// addresses in every replica (longer runs inside one DRAM row per stream).
template <bool SHADOW, int UNROLL, bool SHADOW_CACHED, int V>
__global__ void __launch_bounds__(256)
meta_update_vec_kernel(float* __restrict__ w_tilde, float* __restrict__ v, float* __restrict__ reps,
                       size_t stride, uint16_t* __restrict__ shadow, size_t sstride, int P,
                       size_t n4, size_t n, float mu, float invP) {
    const size_t i0 = (size_t)blockIdx.x * (256 * V) + threadIdx.x;
    const size_t s4 = stride / 4;
    if (i0 + (size_t)(V - 1) * 256 < n4) {                  // all V pieces are whole vectors
        f32x4 wt[V], acc[V];
#pragma unroll
        for (int q = 0; q < V; ++q) { wt[q] = ((const f32x4*)w_tilde)[i0 + q * 256]; acc[q] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
        const f32x4* r = (const f32x4*)reps + i0;
        int j = 0;
        for (; j + UNROLL <= P; j += UNROLL) {
            f32x4 t[UNROLL][V];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int q = 0; q < V; ++q) t[u][q] = __builtin_nontemporal_load(r + (size_t)(j + u) * s4 + q * 256);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int q = 0; q < V; ++q) acc[q] += t[u][q] - wt[q];
        }
        for (; j < P; ++j)
#pragma unroll
            for (int q = 0; q < V; ++q) acc[q] += __builtin_nontemporal_load(r + (size_t)j * s4 + q * 256) - wt[q];
        f32x4 wn[V];
#pragma unroll
        for (int q = 0; q < V; ++q) {
            const f32x4 vn = mu * ((const f32x4*)v)[i0 + q * 256] + acc[q] * invP;
            wn[q] = wt[q] + vn;
            ((f32x4*)v)[i0 + q * 256] = vn;
            ((f32x4*)w_tilde)[i0 + q * 256] = wn[q];
        }
        f32x4* o = (f32x4*)reps + i0;
        for (int jj = 0; jj < P; ++jj)
#pragma unroll
            for (int q = 0; q < V; ++q) __builtin_nontemporal_store(wn[q], o + (size_t)jj * s4 + q * 256);
        if (SHADOW) {
            const size_t ss4 = sstride / 4;
#pragma unroll
            for (int q = 0; q < V; ++q) {
                u16x4 h = {to_bf16_bits(wn[q].x), to_bf16_bits(wn[q].y), to_bf16_bits(wn[q].z), to_bf16_bits(wn[q].w)};
                u16x4* so = (u16x4*)shadow + i0 + q * 256;
                // The shadows are what the next forward pass reads: when they all fit in the memory-side
                // cache they are written with ordinary stores and stay there (the replicas above, read
                // again only by the updates, always bypass it).
                if (SHADOW_CACHED) { for (int jj = 0; jj < P; ++jj) so[(size_t)jj * ss4] = h; }
                else { for (int jj = 0; jj < P; ++jj) __builtin_nontemporal_store(h, so + (size_t)jj * ss4); }
            }
        }
        return;
    }
    // the last workgroups: piece by piece, whole vectors first, then the ragged tail of at most 3 parameters
    for (int q = 0; q < V; ++q) {
        const size_t i = i0 + (size_t)q * 256;
        if (i < n4) {
            for (int e = 0; e < 4; ++e)
                meta_scalar_element(w_tilde, v, reps, stride, SHADOW ? shadow : nullptr, sstride, P, 4 * i + e, mu, invP);
        } else {
            const size_t e = 4 * n4 + (i - n4);
            if (e < n) meta_scalar_element(w_tilde, v, reps, stride, SHADOW ? shadow : nullptr, sstride, P, e, mu, invP);
        }
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
        // Long vectors: eight pieces per lane, so that a workgroup reads and writes 32 KB of consecutive
        // addresses per replica (meta-only workload, 64 replicas: 0.665 -> 0.70 of the HBM peak); short
        // ones keep one piece per lane and more workgroups.
        const bool wide = threads >= (size_t)256 * 8 * 1024;
        const unsigned grid = (unsigned)((threads + (wide ? 2048 : 256) - 1) / (wide ? 2048 : 256));
#define KAVG_META_LAUNCH(SH, SC)                                                                              \
        do {                                                                                                  \
            if (wide) hipLaunchKernelGGL((meta_update_vec_kernel<SH, 2, SC, 8>), dim3(grid), dim3(256), 0, st, w_tilde, \
                                         v, reps, stride, shadow, sstride, P, n4, n, mu, invP);              \
            else hipLaunchKernelGGL((meta_update_vec_kernel<SH, 16, SC, 1>), dim3(grid), dim3(256), 0, st, w_tilde, v, \
                                    reps, stride, shadow, sstride, P, n4, n, mu, invP);                      \
        } while (0)
        if (shadow && shadow_cached) KAVG_META_LAUNCH(true, true);
        else if (shadow) KAVG_META_LAUNCH(true, false);
        else KAVG_META_LAUNCH(false, false);
#undef KAVG_META_LAUNCH
    } else {
        const unsigned grid = (unsigned)((n + 255) / 256);
        hipLaunchKernelGGL(meta_update_scalar_kernel, dim3(grid), dim3(256), 0, st, w_tilde, v, reps,
                           stride, shadow, sstride, P, n, mu, invP);
    }
    return hipGetLastError();
}

// ---- the same step on replicas stored as hi / lo planes -------------------------------------
// Each lane owns eight consecutive parameters: 16 bytes of either plane per learner.  Traffic per
// parameter and pass: P*(2+2) bytes read, P*(2+2) written, plus w~ and v: (2P+4)*4 bytes -- the
// refreshed bf16 values are part of the replicas, not an extra copy.  The hi planes are what the
// next forward pass reads (ordinary stores when they fit the memory-side cache); the lo planes
// are only read again by the updates and are streamed.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void meta_split_scalar_element(float* w_tilde, float* v, uint16_t* hi, uint16_t* lo,
                                                          size_t stride, int P, size_t e, float mu, float invP) {
    const float wt = w_tilde[e];
    float acc = 0.f;
    for (int j = 0; j < P; ++j) {
        const size_t at = (size_t)j * stride + e;
        acc += __builtin_bit_cast(float, split_join(hi[at], lo[at])) - wt;
    }
    const float vn = mu * v[e] + acc * invP;
    const float wn = wt + vn;
    v[e] = vn;
    w_tilde[e] = wn;
    const uint32_t b = __builtin_bit_cast(uint32_t, wn);
    for (int j = 0; j < P; ++j) {
        const size_t at = (size_t)j * stride + e;
        hi[at] = (uint16_t)split_hi(b);
        lo[at] = (uint16_t)split_lo(b);
    }
}

template <int UNROLL, bool HI_CACHED>
__global__ void __launch_bounds__(256)
meta_update_split_kernel(float* __restrict__ w_tilde, float* __restrict__ v, uint16_t* __restrict__ hi,
                         uint16_t* __restrict__ lo, size_t stride, int P, size_t n8, size_t n, float mu,
                         float invP) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n8) {
        float wt[8], acc[8];
        {
            const f32x4 a = ((const f32x4*)w_tilde)[2 * i], b = ((const f32x4*)w_tilde)[2 * i + 1];
            wt[0] = a.x; wt[1] = a.y; wt[2] = a.z; wt[3] = a.w; wt[4] = b.x; wt[5] = b.y; wt[6] = b.z; wt[7] = b.w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        const u32x4* ph = (const u32x4*)hi + i;
        const u32x4* pl = (const u32x4*)lo + i;
        const size_t s8 = stride / 8;
        auto add = [&](const u32x4& h, const u32x4& l) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t b0, b1;
                split_join2(h[q], l[q], b0, b1);
                acc[2 * q] += __builtin_bit_cast(float, b0) - wt[2 * q];
                acc[2 * q + 1] += __builtin_bit_cast(float, b1) - wt[2 * q + 1];
            }
        };
        int j = 0;
        for (; j + UNROLL <= P; j += UNROLL) {
            u32x4 th[UNROLL], tl[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                th[u] = HI_CACHED ? ph[(size_t)(j + u) * s8] : __builtin_nontemporal_load(ph + (size_t)(j + u) * s8);
                tl[u] = __builtin_nontemporal_load(pl + (size_t)(j + u) * s8);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) add(th[u], tl[u]);
        }
        for (; j < P; ++j)
            add(HI_CACHED ? ph[(size_t)j * s8] : __builtin_nontemporal_load(ph + (size_t)j * s8),
                __builtin_nontemporal_load(pl + (size_t)j * s8));
        const f32x4 vo0 = ((const f32x4*)v)[2 * i], vo1 = ((const f32x4*)v)[2 * i + 1];
        const float vo[8] = {vo0.x, vo0.y, vo0.z, vo0.w, vo1.x, vo1.y, vo1.z, vo1.w};
        float vn[8], wn[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { vn[e] = mu * vo[e] + acc[e] * invP; wn[e] = wt[e] + vn[e]; }
        ((f32x4*)v)[2 * i] = (f32x4){vn[0], vn[1], vn[2], vn[3]};
        ((f32x4*)v)[2 * i + 1] = (f32x4){vn[4], vn[5], vn[6], vn[7]};
        ((f32x4*)w_tilde)[2 * i] = (f32x4){wn[0], wn[1], wn[2], wn[3]};
        ((f32x4*)w_tilde)[2 * i + 1] = (f32x4){wn[4], wn[5], wn[6], wn[7]};
        u32x4 oh, ol;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t h2, l2;
            split_pack2(__builtin_bit_cast(uint32_t, wn[2 * q]), __builtin_bit_cast(uint32_t, wn[2 * q + 1]), h2, l2);
            oh[q] = h2; ol[q] = l2;
        }
        u32x4* qh = (u32x4*)hi + i;
        u32x4* ql = (u32x4*)lo + i;
        if (HI_CACHED) { for (int jj = 0; jj < P; ++jj) qh[(size_t)jj * s8] = oh; }
        else { for (int jj = 0; jj < P; ++jj) __builtin_nontemporal_store(oh, qh + (size_t)jj * s8); }
        for (int jj = 0; jj < P; ++jj) __builtin_nontemporal_store(ol, ql + (size_t)jj * s8);
    } else {
        const size_t e = 8 * n8 + (i - n8);               // ragged tail: at most 7 parameters
        if (e < n) meta_split_scalar_element(w_tilde, v, hi, lo, stride, P, e, mu, invP);
    }
}

hipError_t launch_meta_update_split(float* w_tilde, float* v, uint16_t* hi, uint16_t* lo, size_t stride,
                                    int P, size_t n, float mu, int hi_cached, hipStream_t st) {
    // planes and vectors come out of the 256-byte aligned workspace; stride is a multiple of 64
    const float invP = 1.0f / (float)P;
    const size_t n8 = n / 8;
    const size_t threads = n8 + (n - 8 * n8);
    const unsigned grid = (unsigned)((threads + 255) / 256);
    if (hi_cached)
        hipLaunchKernelGGL((meta_update_split_kernel<8, true>), dim3(grid), dim3(256), 0, st, w_tilde, v, hi, lo,
                           stride, P, n8, n, mu, invP);
    else
        hipLaunchKernelGGL((meta_update_split_kernel<8, false>), dim3(grid), dim3(256), 0, st, w_tilde, v, hi, lo,
                           stride, P, n8, n, mu, invP);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256)
broadcast_split_kernel(const float* __restrict__ w_tilde, uint16_t* __restrict__ hi, uint16_t* __restrict__ lo,
                       size_t stride, int P, size_t n) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const uint32_t b = __builtin_bit_cast(uint32_t, w_tilde[e]);
    for (int j = 0; j < P; ++j) {
        hi[(size_t)j * stride + e] = (uint16_t)split_hi(b);
        lo[(size_t)j * stride + e] = (uint16_t)split_lo(b);
    }
}

hipError_t launch_broadcast_split(const float* w_tilde, uint16_t* hi, uint16_t* lo, size_t stride, int P,
                                  size_t n, hipStream_t st) {
    const unsigned grid = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(broadcast_split_kernel, dim3(grid), dim3(256), 0, st, w_tilde, hi, lo, stride, P, n);
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
