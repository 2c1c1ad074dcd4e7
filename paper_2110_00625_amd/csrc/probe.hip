// Ceilings of the device under the access patterns the M-AVG kernels use: what one GPU can stream
// (read-only, write-only, read and write in equal parts) with 16-byte non-temporal accesses laid out
// like the meta step's (each lane owns one 16-byte piece of each of U interleaved rows), and what
// the matrix cores deliver on v_mfma_f32_32x32x16_bf16 with nothing to fetch.  Measurement aid for
// the benchmark: the fused meta step of Algorithm 1 moves equal amounts in both directions, so the
// 1:1 figure is the one it can be held against.
#include "kavg_internal.h"

namespace kavg {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int U = 16;        // rows per lane in flight, as in the meta kernel

// buffer viewed as [U][row16] pieces of 16 bytes; thread i handles piece i of every row
template <int KIND>
__global__ void __launch_bounds__(256) stream_probe_kernel(f32x4* __restrict__ a, f32x4* __restrict__ b, size_t row16,
                                                            float* sink) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= row16) return;
    if (KIND == KAVG_PROBE_WRITE) {
        const f32x4 val = {1.f, 2.f, 3.f, (float)i};
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(val, a + (size_t)u * row16 + i);
        return;
    }
    f32x4 t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) t[u] = __builtin_nontemporal_load(a + (size_t)u * row16 + i);
    if (KIND == KAVG_PROBE_READ) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < U; ++u) acc += t[u];
        // never true for finite data; keeps the loads alive without a store per lane
        if (acc.x + acc.y + acc.z + acc.w == 1.2345678e38f) *sink = acc.x;
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(t[u], b + (size_t)u * row16 + i);
    }
}

// four independent accumulator chains per wavefront, operands held in registers
__global__ void __launch_bounds__(256) mfma_probe_kernel(int iters, float* sink) {
    bf16x8 x, y;
#pragma unroll
    for (int e = 0; e < 8; ++e) { x[e] = (__bf16)(0.001f * (float)(threadIdx.x + e)); y[e] = (__bf16)(0.002f * (float)e); }
    f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[c][e];
    if (s == 1.2345678e38f) *sink = s;
}

}  // namespace

size_t probe_stream_bytes(size_t bytes) { return bytes / (16 * U) * (16 * U); }

hipError_t launch_probe(int kind, void* a, void* b, size_t bytes, int iters, float* sink, hipStream_t st,
                        double* work_out) {
    if (kind == KAVG_PROBE_MFMA) {
        const int wgs = 256 * 8;                     // 8 workgroups of 4 wavefronts per compute unit
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(wgs), dim3(256), 0, st, iters, sink);
        *work_out = 2.0 * 32 * 32 * 16 * 4.0 * (double)iters * 4.0 * wgs;      // flops
        return hipGetLastError();
    }
    const size_t row16 = bytes / (16 * U);
    const unsigned grid = (unsigned)((row16 + 255) / 256);
    f32x4* pa = (f32x4*)a;
    f32x4* pb = (f32x4*)b;
    if (kind == KAVG_PROBE_READ) hipLaunchKernelGGL((stream_probe_kernel<KAVG_PROBE_READ>), dim3(grid), dim3(256), 0, st, pa, pb, row16, sink);
    else if (kind == KAVG_PROBE_WRITE) hipLaunchKernelGGL((stream_probe_kernel<KAVG_PROBE_WRITE>), dim3(grid), dim3(256), 0, st, pa, pb, row16, sink);
    else hipLaunchKernelGGL((stream_probe_kernel<KAVG_PROBE_COPY>), dim3(grid), dim3(256), 0, st, pa, pb, row16, sink);
    *work_out = (double)(row16 * 16 * U) * (kind == KAVG_PROBE_COPY ? 2.0 : 1.0);   // bytes moved
    return hipGetLastError();
}

}  // namespace kavg
