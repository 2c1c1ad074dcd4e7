// bf16 MFMA path of the learner step (KAVG_BF16), batched over learners.
//
// All three dense products of a layer are instances of
//        O[r][c] = sum_k R(r,k) * Cm(c,k)          (fp32 accumulation)
// on bf16 operands staged through LDS and contracted with
// v_mfma_f32_32x32x16_bf16 on 64-lane wavefronts:
//
//   forward        r = sample, c = output unit, k = input unit
//                  A_l = bf16(relu(A_{l-1} W_l^T + b_l))      (last layer: fp32 logits)
//   backward-data  r = sample, c = input unit,  k = output unit
//                  dZ_{l-1} = bf16((dZ_l W_l) * [A_{l-1} > 0])
//   update         r = output unit, c = input unit, k = sample
//                  W_l <- W_l - lr * dZ_l^T A_{l-1}  on the fp32 master, bf16 shadow refreshed,
//                  b_l <- b_l - lr * colsum(dZ_l)
//                  (the learner update of Algorithm 1; the 1/B factor already sits in dZ_L)
//
// Operand roles are chosen so that the MFMA "row" index i runs along the
// memory-contiguous output dimension c: a lane then owns groups of four
// consecutive output columns and the epilogue uses 16-byte (fp32) / 8-byte
// (bf16) accesses.  i <- Cm rows, j <- R rows.
//
// An operand whose contraction index is contiguous in memory ("direct": the
// activations and weights of the forward pass, dZ of backward-data) is copied
// to LDS in 16-byte pieces.  An operand whose contraction index is the row
// index in memory ("transposed": W in backward-data, dZ and A in the update,
// whose contraction runs over the samples) is loaded as 4x8 blocks with
// coalesced 16-byte row reads, transposed in registers, and written as 8-byte
// pieces, so that LDS always holds [row][k] with k contiguous.
//
// Rows beyond an extent are zero-filled on load and masked on store; every
// memory-contiguous extent is a multiple of 8 elements (hidden widths are
// required to be, the class count is padded in the logits / dZ_L buffers).
#include "kavg_internal.h"

namespace kavg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;          // contraction slice held in LDS
constexpr int BKP = BK + 8;     // padded LDS row (bf16 elements): 144 bytes, keeps 16-byte alignment

enum { MODE_FWD = 0, MODE_BWD = 1, MODE_UPD = 2 };

struct Operand {
    const uint16_t* base;    // learner 0
    size_t lstride;          // elements between learners (0: shared by all learners)
    int ld;                  // elements between consecutive memory rows
    int trans;               // 0: memory row = x, contiguous = k;  1: memory row = k, contiguous = x
    const int32_t* gather;   // optional: memory row = gather[row]
    long gstride;            // per learner
    int n_rows;              // valid memory rows (exact)
    int n_cont;              // readable contiguous extent (multiple of 8)
};

struct Args {
    Operand R, C;
    int nR, nC, nK;
    // forward
    const float* bias; size_t bias_lstride;
    void* out; size_t out_lstride; int ld_out;   // bf16 activations or fp32 logits
    int relu;                                    // 1: hidden layer (bf16 out), 0: last layer (fp32 out)
    // backward-data
    const uint16_t* act_prev; size_t act_lstride; int ld_act;
    // update
    float* w; size_t w_lstride; uint16_t* ws; size_t ws_lstride; float* b;
    float lr;
};

__device__ __forceinline__ uint16_t bf16_bits(float x) {
    __bf16 h = (__bf16)x;                         // round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)bf16_bits(lo) | ((uint32_t)bf16_bits(hi) << 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
    return __builtin_bit_cast(float, (uint32_t)h << 16);
}

// ---- staging: global -> registers -> LDS ------------------------------------
template <int X> struct DirectRegs { u32x4 v[X / 32]; };
template <int X> struct TransRegs  { u32x4 v[4]; };     // four memory rows (k), eight x each

template <int X>
__device__ __forceinline__ void load_direct(DirectRegs<X>& g, const Operand& o, const uint16_t* base,
                                            const int32_t* gather, int x0, int k0, int tid) {
#pragma unroll
    for (int i = 0; i < X / 32; ++i) {
        const int e = tid + 256 * i;
        const int x = x0 + (e >> 3), k = k0 + (e & 7) * 8;
        u32x4 val = {0u, 0u, 0u, 0u};
        if (x < o.n_rows && k < o.n_cont) {
            const long row = gather ? (long)gather[x] : (long)x;
            val = *(const u32x4*)(base + row * o.ld + k);
        }
        g.v[i] = val;
    }
}

template <int X>
__device__ __forceinline__ void store_direct(const DirectRegs<X>& g, uint16_t* lds, int tid) {
#pragma unroll
    for (int i = 0; i < X / 32; ++i) {
        const int e = tid + 256 * i;
        *(u32x4*)(lds + (e >> 3) * BKP + (e & 7) * 8) = g.v[i];
    }
}

// thread u of X/8 * 16 handles memory rows k0 + 4*(u / (X/8)) .. +3 and columns x0 + 8*(u % (X/8)) .. +7
template <int X>
__device__ __forceinline__ void load_trans(TransRegs<X>& g, const Operand& o, const uint16_t* base,
                                           const int32_t* gather, int x0, int k0, int tid) {
    constexpr int XB = X / 8;
    const int xb = tid % XB, kb = tid / XB;
    const int x = x0 + xb * 8;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int k = k0 + kb * 4 + r;
        u32x4 val = {0u, 0u, 0u, 0u};
        if (kb < 16 && k < o.n_rows && x < o.n_cont) {
            const long row = gather ? (long)gather[k] : (long)k;
            val = *(const u32x4*)(base + row * o.ld + x);
        }
        g.v[r] = val;
    }
}

template <int X>
__device__ __forceinline__ void store_trans(const TransRegs<X>& g, uint16_t* lds, int tid) {
    constexpr int XB = X / 8;
    const int xb = tid % XB, kb = tid / XB;
    if (kb >= 16) return;
#pragma unroll
    for (int xi = 0; xi < 8; ++xi) {
        const int w = xi >> 1;
        uint32_t lo, hi;
        if (xi & 1) {
            lo = (g.v[0][w] >> 16) | (g.v[1][w] & 0xFFFF0000u);
            hi = (g.v[2][w] >> 16) | (g.v[3][w] & 0xFFFF0000u);
        } else {
            lo = (g.v[0][w] & 0xFFFFu) | (g.v[1][w] << 16);
            hi = (g.v[2][w] & 0xFFFFu) | (g.v[3][w] << 16);
        }
        u32x2 out = {lo, hi};
        *(u32x2*)(lds + (xb * 8 + xi) * BKP + kb * 4) = out;
    }
}

// ---- the kernel ----------------------------------------------------------------
// TR x TC output tile, 4 wavefronts arranged WR x WC, each owning MR x MC MFMA blocks of 32x32.
template <int MODE, int TR, int TC, int WR, int WC, bool RTRANS, bool CTRANS>
__global__ void __launch_bounds__(256) gemm_bf16_kernel(Args a) {
    static_assert(WR * WC == 4, "four wavefronts per workgroup");
    constexpr int MR = TR / (32 * WR), MC = TC / (32 * WC);
    static_assert(MR >= 1 && MC >= 1, "tile too small for the wave grid");
    __shared__ __attribute__((aligned(16))) uint16_t Rs[TR * BKP];
    __shared__ __attribute__((aligned(16))) uint16_t Cs[TC * BKP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave / WC, wc = wave % WC;
    const int learner = blockIdx.z;
    const int r0 = blockIdx.y * TR, c0 = blockIdx.x * TC;

    const uint16_t* Rbase = a.R.base + (size_t)learner * a.R.lstride;
    const uint16_t* Cbase = a.C.base + (size_t)learner * a.C.lstride;
    const int32_t* Rg = a.R.gather ? a.R.gather + (long)learner * a.R.gstride : nullptr;
    const int32_t* Cg = a.C.gather ? a.C.gather + (long)learner * a.C.gstride : nullptr;

    f32x16 acc[MR][MC];
#pragma unroll
    for (int i = 0; i < MR; ++i)
#pragma unroll
        for (int j = 0; j < MC; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    DirectRegs<TR> rd; TransRegs<TR> rt;
    DirectRegs<TC> cd; TransRegs<TC> ct;
    float bias_sum = 0.f;                       // update: column sum of dZ for row r0 + tid

    auto fetch = [&](int k0) {
        if (RTRANS) load_trans<TR>(rt, a.R, Rbase, Rg, r0, k0, tid); else load_direct<TR>(rd, a.R, Rbase, Rg, r0, k0, tid);
        if (CTRANS) load_trans<TC>(ct, a.C, Cbase, Cg, c0, k0, tid); else load_direct<TC>(cd, a.C, Cbase, Cg, c0, k0, tid);
    };
    auto stash = [&]() {
        if (RTRANS) store_trans<TR>(rt, Rs, tid); else store_direct<TR>(rd, Rs, tid);
        if (CTRANS) store_trans<TC>(ct, Cs, tid); else store_direct<TC>(cd, Cs, tid);
    };

    fetch(0);
    for (int k0 = 0; k0 < a.nK; k0 += BK) {
        stash();
        __syncthreads();
        if (k0 + BK < a.nK) fetch(k0 + BK);     // next slice in flight during the MFMAs
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 cf[MC], rf[MR];
            const int koff = kk * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int j = 0; j < MC; ++j)
                cf[j] = *(const bf16x8*)(Cs + (wc * MC * 32 + j * 32 + (lane & 31)) * BKP + koff);
#pragma unroll
            for (int i = 0; i < MR; ++i)
                rf[i] = *(const bf16x8*)(Rs + (wr * MR * 32 + i * 32 + (lane & 31)) * BKP + koff);
#pragma unroll
            for (int i = 0; i < MR; ++i)
#pragma unroll
                for (int j = 0; j < MC; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf[j], rf[i], acc[i][j], 0, 0, 0);
        }
        if (MODE == MODE_UPD && blockIdx.x == 0 && tid < TR) {
            const uint16_t* row = Rs + tid * BKP;
#pragma unroll 8
            for (int k = 0; k < BK; ++k) bias_sum += bf16_to_f32(row[k]);
        }
        __syncthreads();
    }

    // ---- epilogue: lane owns, per block, row r = l%32 and columns 8q + 4(l/32) + 0..3, q = 0..3
#pragma unroll
    for (int i = 0; i < MR; ++i) {
        const int r = r0 + (wr * MR + i) * 32 + (lane & 31);
        if (r >= a.nR) continue;
#pragma unroll
        for (int j = 0; j < MC; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c0 + (wc * MC + j) * 32 + q * 8 + (lane >> 5) * 4;
                float v0 = acc[i][j][4 * q + 0], v1 = acc[i][j][4 * q + 1];
                float v2 = acc[i][j][4 * q + 2], v3 = acc[i][j][4 * q + 3];
                if (MODE == MODE_FWD) {
                    if (c >= a.ld_out) continue;
                    const float* bias = a.bias + (size_t)learner * a.bias_lstride;
                    v0 += c + 0 < a.nC ? bias[c + 0] : 0.f;
                    v1 += c + 1 < a.nC ? bias[c + 1] : 0.f;
                    v2 += c + 2 < a.nC ? bias[c + 2] : 0.f;
                    v3 += c + 3 < a.nC ? bias[c + 3] : 0.f;
                    if (a.relu) {
                        u32x2 o = {pack2(fmaxf(v0, 0.f), fmaxf(v1, 0.f)), pack2(fmaxf(v2, 0.f), fmaxf(v3, 0.f))};
                        *(u32x2*)((uint16_t*)a.out + (size_t)learner * a.out_lstride + (size_t)r * a.ld_out + c) = o;
                    } else {
                        f32x4 o = {v0, v1, v2, v3};
                        *(f32x4*)((float*)a.out + (size_t)learner * a.out_lstride + (size_t)r * a.ld_out + c) = o;
                    }
                } else if (MODE == MODE_BWD) {
                    if (c >= a.nC) continue;
                    const u32x2 m = *(const u32x2*)(a.act_prev + (size_t)learner * a.act_lstride + (size_t)r * a.ld_act + c);
                    // stored activations are relu outputs (never negative): positive <=> non-zero magnitude
                    v0 = (m.x & 0x7FFFu) ? v0 : 0.f;
                    v1 = (m.x & 0x7FFF0000u) ? v1 : 0.f;
                    v2 = (m.y & 0x7FFFu) ? v2 : 0.f;
                    v3 = (m.y & 0x7FFF0000u) ? v3 : 0.f;
                    u32x2 o = {pack2(v0, v1), pack2(v2, v3)};
                    *(u32x2*)((uint16_t*)a.out + (size_t)learner * a.out_lstride + (size_t)r * a.ld_out + c) = o;
                } else {
                    if (c >= a.nC) continue;
                    float* wp = a.w + (size_t)learner * a.w_lstride + (size_t)r * a.nC + c;
                    f32x4 w = *(const f32x4*)wp;
                    w.x -= a.lr * v0; w.y -= a.lr * v1; w.z -= a.lr * v2; w.w -= a.lr * v3;
                    *(f32x4*)wp = w;
                    u32x2 o = {pack2(w.x, w.y), pack2(w.z, w.w)};
                    *(u32x2*)(a.ws + (size_t)learner * a.ws_lstride + (size_t)r * a.nC + c) = o;
                }
            }
        }
    }
    if (MODE == MODE_UPD && blockIdx.x == 0 && tid < TR && r0 + tid < a.nR) {
        float* b = a.b + (size_t)learner * a.w_lstride + r0 + tid;
        *b = *b - a.lr * bias_sum;
    }
}

template <int MODE, int TR, int TC, int WR, int WC, bool RT, bool CT>
hipError_t launch(const Args& a, int P, hipStream_t st) {
    dim3 grid((a.nC + TC - 1) / TC, (a.nR + TR - 1) / TR, P);
    hipLaunchKernelGGL((gemm_bf16_kernel<MODE, TR, TC, WR, WC, RT, CT>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

int round8(int x) { return (x + 7) / 8 * 8; }

}  // namespace

hipError_t bf16_forward(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.in, c.gather ? 0 : c.in_stride, c.ld_in, 0, c.gather, c.gather_stride, c.B, c.d_in};
    a.C = {c.ws, c.ws_stride, c.d_in, 0, nullptr, 0, c.d_out, c.d_in};
    a.nR = c.B; a.nC = c.d_out; a.nK = c.d_in;
    a.bias = c.b; a.bias_lstride = c.w_stride;
    a.out = c.out; a.out_lstride = c.out_stride; a.ld_out = c.ld_out; a.relu = c.relu;
    if (c.B <= 64) return launch<MODE_FWD, 64, 128, 2, 2, false, false>(a, c.P, st);
    return launch<MODE_FWD, 128, 128, 2, 2, false, false>(a, c.P, st);
}

hipError_t bf16_backward_data(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.dz, c.dz_stride, c.ld_dz, 0, nullptr, 0, c.B, round8(c.d_out)};
    a.C = {c.ws, c.ws_stride, c.d_in, 1, nullptr, 0, c.d_out, c.d_in};   // Cm(c, k) = W[k][c]
    a.nR = c.B; a.nC = c.d_in; a.nK = c.d_out;
    a.act_prev = (const uint16_t*)c.in; a.act_lstride = c.in_stride; a.ld_act = c.ld_in;
    a.out = c.dz_prev; a.out_lstride = c.dz_prev_stride; a.ld_out = c.ld_in;
    if (c.B <= 64) return launch<MODE_BWD, 64, 128, 2, 2, false, true>(a, c.P, st);
    return launch<MODE_BWD, 128, 128, 2, 2, false, true>(a, c.P, st);
}

hipError_t bf16_update(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.dz, c.dz_stride, c.ld_dz, 1, nullptr, 0, c.B, c.ld_dz};      // R(r, k) = dZ[k][r]
    a.C = {(const uint16_t*)c.in, c.gather ? 0 : c.in_stride, c.ld_in, 1, c.gather, c.gather_stride, c.B, c.d_in};
    a.nR = c.d_out; a.nC = c.d_in; a.nK = c.B;
    a.w = c.w; a.w_lstride = c.w_stride; a.ws = c.ws; a.ws_lstride = c.ws_stride; a.b = c.b;
    a.lr = c.lr;
    return launch<MODE_UPD, 128, 128, 2, 2, true, true>(a, c.P, st);
}

}  // namespace kavg
