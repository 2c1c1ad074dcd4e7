// fp32 path of the learner step (KAVG_FP32): forward, backward-data and the
// fused weight-gradient + SGD update, batched over learners.
//
// One generic LDS-tiled kernel computes   O[r][c] = sum_k R(r,k) * Cm(c,k)
// for operands given by (row stride, contraction stride, optional row gather),
// with three epilogues.  The contraction runs on the matrix cores in full fp32
// (v_mfma_f32_32x32x2_f32: exact fp32 products, fp32 accumulation; no reduced
// precision), each of the four wavefronts owning one 32x32 quarter of the 64x64
// tile, k ascending, so results are deterministic and independent of timing.
//
//   forward        r = sample, c = output unit, k = input unit
//                  O = act(A_{l-1} W_l^T + b_l)
//   backward-data  r = sample, c = input unit,  k = output unit
//                  dZ_{l-1} = (dZ_l W_l) * [A_{l-1} > 0]
//   update         r = output unit, c = input unit, k = sample
//                  W_l <- W_l - lr * dZ_l^T A_{l-1};  b_l <- b_l - lr * colsum(dZ_l)
//                  (the learner update of Algorithm 1; 1/B already sits in dZ_L)
//
// The fp32 workloads are small (a few output tiles per learner, long
// contractions), so the forward pass may split the contraction over several
// workgroups: each writes its partial tile to a scratch buffer and a second
// small kernel adds the partials in ascending split order, then applies bias
// and ReLU.  The number of splits depends only on the shapes.
#include "kavg_internal.h"

namespace kavg {

namespace {

constexpr int TILE = 64;   // output tile is TILE x TILE
constexpr int BK = 32;     // contraction slice
constexpr int PADW = TILE + 4;
constexpr int NPER = TILE * BK / 256;   // elements of a slice each thread moves per operand

typedef float f32x16 __attribute__((ext_vector_type(16)));

enum { EPI_FWD = 0, EPI_BWD = 1, EPI_UPD = 2, EPI_PARTIAL = 3 };

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
    int k_chunk;            // contraction range of one split (multiple of BK); nK when not split
    // epilogue
    float* out;  size_t out_stride;  int ld_out;       // FWD/BWD output, UPD: master weights, PARTIAL: scratch
    size_t split_stride;                               // PARTIAL: elements between splits
    const float* bias; size_t bias_stride;             // FWD: bias
    float* bias_rw;                                    // UPD: bias to update (stride = bias_stride)
    const float* mask; size_t mask_stride; int ld_mask;// BWD: previous activations
    const float* dz; size_t dz_stride; int ld_dz;      // UPD: dZ for the bias gradient [B][ld_dz]
    int relu;
    float lr;
    float* u; float* ub; float beta;                   // UPD: velocities of weights / bias (null: plain SGD)
};

// Where thread `tid` finds its NPER elements of a slice: element i is (x, k) with the memory-
// contiguous index running fastest over the threads.
struct Mover {
    const float* p[NPER];   // address for k = 0 of the (clamped) row x
    int x[NPER], k[NPER];
    bool ok[NPER];          // x lies inside the operand
};

__device__ __forceinline__ void mover_init(Mover& m, const Operand& o, int learner, int x0, int nX, int tid) {
    const float* base = o.base + (size_t)learner * o.learner_stride;
    const int32_t* g = o.gather ? o.gather + (long)learner * o.gather_stride : nullptr;
    const bool kfast = (o.ld_k == 1 && !(g && o.gather_on_k));
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
        const int e = tid + 256 * i;
        if (kfast) { m.x[i] = e / BK; m.k[i] = e % BK; } else { m.x[i] = e % TILE; m.k[i] = e / TILE; }
        const int x = x0 + m.x[i];
        m.ok[i] = x < nX;
        const int xc = m.ok[i] ? x : nX - 1;
        const long row = (g && !o.gather_on_k) ? (long)g[xc] : (long)xc;
        m.p[i] = base + row * o.ld_x;
    }
}

// The thread's NPER elements of the slice starting at k0.  No load is predicated: positions outside
// the operand or beyond k_end are read from clamped addresses and replaced by zeros, so that all
// loads of the slice are in flight together; with a gather on the contraction index, all row
// indices are requested first, then all elements (one wait, not one per element).
__device__ __forceinline__ void mover_load_all(const Mover& m, const Operand& o, int learner, int k0, int k_end,
                                               float (&out)[NPER]) {
    long off[NPER];
    if (o.gather && o.gather_on_k) {
        const int32_t* g = o.gather + (long)learner * o.gather_stride;
        int32_t row[NPER];
#pragma unroll
        for (int i = 0; i < NPER; ++i) row[i] = g[min(k0 + m.k[i], k_end - 1)];
#pragma unroll
        for (int i = 0; i < NPER; ++i) off[i] = (long)row[i] * o.ld_k;
    } else {
#pragma unroll
        for (int i = 0; i < NPER; ++i) off[i] = (long)min(k0 + m.k[i], k_end - 1) * o.ld_k;
    }
    float v[NPER];
#pragma unroll
    for (int i = 0; i < NPER; ++i) v[i] = m.p[i][off[i]];
#pragma unroll
    for (int i = 0; i < NPER; ++i) out[i] = (m.ok[i] && k0 + m.k[i] < k_end) ? v[i] : 0.f;
}

template <int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(Args a) {
    __shared__ float Rs[BK][PADW];
    __shared__ float Cs[BK][PADW];
    const int tid = threadIdx.x;
    const int split = blockIdx.z % ((a.nK + a.k_chunk - 1) / a.k_chunk);
    const int learner = blockIdx.z / ((a.nK + a.k_chunk - 1) / a.k_chunk);
    const int r0 = blockIdx.y * TILE, c0 = blockIdx.x * TILE;
    const int lane = tid & 63, wave = tid >> 6;
    const int rq = (wave >> 1) * 32, cq = (wave & 1) * 32;    // this wavefront's quarter of the tile
    const int k_begin = split * a.k_chunk;
    const int k_end = k_begin + a.k_chunk < a.nK ? k_begin + a.k_chunk : a.nK;

    Mover mr, mc;
    mover_init(mr, a.R, learner, r0, a.nR, tid);
    mover_init(mc, a.C, learner, c0, a.nC, tid);

    f32x16 acc = {};
    float rv_next[NPER], cv_next[NPER];
    mover_load_all(mr, a.R, learner, k_begin, k_end, rv_next);
    mover_load_all(mc, a.C, learner, k_begin, k_end, cv_next);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
#pragma unroll
        for (int i = 0; i < NPER; ++i) {
            Rs[mr.k[i]][mr.x[i]] = rv_next[i];
            Cs[mc.k[i]][mc.x[i]] = cv_next[i];
        }
        __syncthreads();
        if (k0 + BK < k_end) {
            mover_load_all(mr, a.R, learner, k0 + BK, k_end, rv_next);      // next slice in flight during the FMAs
            mover_load_all(mc, a.C, learner, k0 + BK, k_end, cv_next);
        }
        // A step of the matrix instruction takes two k: lane l supplies R(row l%32, k l/32) and Cm(col l%32, k l/32);
        // consecutive lanes read consecutive LDS words.
#pragma unroll
        for (int k = 0; k < BK; k += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Rs[k + (lane >> 5)][rq + (lane & 31)], Cs[k + (lane >> 5)][cq + (lane & 31)],
                                                       acc, 0, 0, 0);
        __syncthreads();
    }

    // accumulator v of lane l is the output (row 8*(v/4) + 4*(l/32) + v%4, column l%32) of the quarter
    const int c = c0 + cq + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = r0 + rq + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (r >= a.nR || c >= a.nC) continue;
        if (EPI == EPI_FWD) {
            float z = acc[v] + a.bias[(size_t)learner * a.bias_stride + c];
            if (a.relu) z = fmaxf(z, 0.f);
            a.out[(size_t)learner * a.out_stride + (size_t)r * a.ld_out + c] = z;
        } else if (EPI == EPI_PARTIAL) {
            a.out[(size_t)split * a.split_stride + (size_t)learner * a.out_stride + (size_t)r * a.ld_out + c] = acc[v];
        } else if (EPI == EPI_BWD) {
            const float m = a.mask[(size_t)learner * a.mask_stride + (size_t)r * a.ld_mask + c];
            a.out[(size_t)learner * a.out_stride + (size_t)r * a.ld_out + c] = m > 0.f ? acc[v] : 0.f;
        } else {
            const size_t at = (size_t)learner * a.out_stride + (size_t)r * a.ld_out + c;
            float g = acc[v];
            if (a.u) { g = a.beta * a.u[at] + g; a.u[at] = g; }
            a.out[at] = a.out[at] - a.lr * g;
        }
    }

    if (EPI == EPI_UPD && blockIdx.x == 0 && tid < TILE) {
        // bias gradient of this tile's output units: column sums of dZ_l over the batch
        const int r = r0 + tid;
        if (r < a.nR) {
            const float* dz = a.dz + (size_t)learner * a.dz_stride;
            // eight rows requested together, added in ascending order
            float s = 0.f;
            int m = 0;
            for (; m + 8 <= a.nK; m += 8) {
                float t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = dz[(size_t)(m + u) * a.ld_dz + r];
#pragma unroll
                for (int u = 0; u < 8; ++u) s += t[u];
            }
            for (; m < a.nK; ++m) s += dz[(size_t)m * a.ld_dz + r];
            const size_t at = (size_t)learner * a.bias_stride + r;
            if (a.ub) { s = a.beta * a.ub[at] + s; a.ub[at] = s; }
            a.bias_rw[at] = a.bias_rw[at] - a.lr * s;
        }
    }
}

// out[j][r][c] = act(sum_s partial[s][j][r][c] + bias[j][c]), splits added in ascending order
__global__ void __launch_bounds__(256)
finish_forward_kernel(const float* __restrict__ partial, size_t split_stride, int splits, const float* __restrict__ bias,
                      size_t bias_stride, float* __restrict__ out, int P, int B, int ld_out, int nC, int relu) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t per_learner = (size_t)B * ld_out;
    if (e >= (size_t)P * per_learner) return;
    const int c = (int)(e % ld_out);
    if (c >= nC) return;
    const int learner = (int)(e / per_learner);
    // eight partials are requested together, then added in ascending order (same sum, one round trip
    // to memory per eight splits instead of one per split)
    float z = 0.f;
    int s = 0;
    for (; s + 8 <= splits; s += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = partial[(size_t)(s + u) * split_stride + e];
#pragma unroll
        for (int u = 0; u < 8; ++u) z += t[u];
    }
    for (; s < splits; ++s) z += partial[(size_t)s * split_stride + e];
    z += bias[(size_t)learner * bias_stride + c];
    if (relu) z = fmaxf(z, 0.f);
    out[e] = z;
}

template <int EPI>
hipError_t run(const Args& a, int P, int splits, hipStream_t st) {
    dim3 grid((a.nC + TILE - 1) / TILE, (a.nR + TILE - 1) / TILE, P * splits);
    hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace

// How the forward pass of a layer splits its contraction: returns the number of splits and the
// contraction range of each (a multiple of the slice length).  Depends on the shapes only.
int f32_forward_plan(int P, int B, int d_in, int d_out, int* chunk_out) {
    const long tiles = (long)((B + TILE - 1) / TILE) * ((d_out + TILE - 1) / TILE) * P;
    long s = 1;
    if (tiles < 256 && d_in > 4 * BK) {
        s = (512 + tiles - 1) / tiles;               // aim at ~512 workgroups
        const long max_s = d_in / (2 * BK);          // at least two slices per split
        if (s > max_s) s = max_s;
        if (s > 64) s = 64;
        if (s < 1) s = 1;
    }
    int chunk = (int)((d_in + s - 1) / s);
    chunk = (chunk + BK - 1) / BK * BK;
    if (chunk_out) *chunk_out = chunk;
    return (d_in + chunk - 1) / chunk;               // splits that actually receive work
}

hipError_t f32_forward(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const float*)c.in, c.in_stride, c.ld_in, 1, c.gather, c.gather_stride, 0};
    if (c.gather) a.R.learner_stride = 0;               // all learners read the one data set
    a.C = {c.w, c.w_stride, c.d_in, 1, nullptr, 0, 0};
    a.nR = c.B; a.nC = c.d_out; a.nK = c.d_in;
    a.out = (float*)c.out; a.out_stride = c.out_stride; a.ld_out = c.ld_out;
    a.bias = c.b; a.bias_stride = c.w_stride;
    a.relu = c.relu;
    int chunk = 0;
    const int splits = f32_forward_plan(c.P, c.B, c.d_in, c.d_out, &chunk);
    if (splits == 1 || !c.scratch) {
        a.k_chunk = a.nK;
        return run<EPI_FWD>(a, c.P, 1, st);
    }
    a.k_chunk = chunk;
    a.out = (float*)c.scratch;
    a.split_stride = (size_t)c.P * c.out_stride;
    hipError_t e = run<EPI_PARTIAL>(a, c.P, splits, st);
    if (e != hipSuccess) return e;
    const size_t total = (size_t)c.P * c.out_stride;
    hipLaunchKernelGGL(finish_forward_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const float*)c.scratch, a.split_stride, splits, c.b, c.w_stride, (float*)c.out, c.P, c.B,
                       c.ld_out, c.d_out, c.relu);
    return hipGetLastError();
}

hipError_t f32_backward_data(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const float*)c.dz, c.dz_stride, c.ld_dz, 1, nullptr, 0, 0};
    a.C = {c.w, c.w_stride, 1, c.d_in, nullptr, 0, 0};  // Cm(c = input unit, k = output unit) = W[k][c]
    a.nR = c.B; a.nC = c.d_in; a.nK = c.d_out; a.k_chunk = a.nK;
    a.out = (float*)c.dz_prev; a.out_stride = c.dz_prev_stride; a.ld_out = c.ld_in;
    a.mask = (const float*)c.in; a.mask_stride = c.in_stride; a.ld_mask = c.ld_in;
    return run<EPI_BWD>(a, c.P, 1, st);
}

hipError_t f32_update(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const float*)c.dz, c.dz_stride, 1, c.ld_dz, nullptr, 0, 0};        // R(r = unit, k = sample) = dZ[k][r]
    a.C = {(const float*)c.in, c.in_stride, 1, c.ld_in, c.gather, c.gather_stride, 1};  // Cm(c, k = sample) = A[k][c]
    if (c.gather) a.C.learner_stride = 0;
    a.nR = c.d_out; a.nC = c.d_in; a.nK = c.B; a.k_chunk = a.nK;
    a.out = c.w; a.out_stride = c.w_stride; a.ld_out = c.d_in;
    a.bias_rw = c.b; a.bias_stride = c.w_stride;
    a.dz = (const float*)c.dz; a.dz_stride = c.dz_stride; a.ld_dz = c.ld_dz;
    a.lr = c.lr; a.u = c.u; a.ub = c.ub; a.beta = c.beta;
    return run<EPI_UPD>(a, c.P, 1, st);
}

}  // namespace kavg
