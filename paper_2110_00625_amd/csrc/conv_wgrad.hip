// Weight gradient of a 3x3 convolution (stride 1, zero padding 1) for images 32 pixels wide, all nine taps
// from one pass over the images:
//
//     dW[o][tap][c] = sum over positions p of dZ[p][o] * A[p + (dy, dx)][c],   tap = 3 (dy+1) + (dx+1)
//
// (the learner update of Algorithm 1 for a convolutional layer: the contraction runs over the positions of
// the minibatch).  The generic kernel treats the nine taps as nine column tiles of a patch matrix, and each
// of them reads dZ and a shifted copy of the images again; here a workgroup walks over whole images two
// rows (64 positions) at a time, keeps those rows of dZ and the four image rows around them (with a zero
// column on either side) in LDS, and every tap's operand is the same LDS tile read at a shifted pixel.
// Per 64 positions a compute unit then takes in 16 KB + 16 KB instead of nine times 24 KB.
//
// Workgroup = (learner, range of whole images); 3 * c_out/32 wavefronts: a wavefront owns the taps with
// dx = tl - 1 (dy = -1, 0, 1) for 32 output channels and all input channels (or, see the kernel, 64 output
// channels and 32 input channels), i.e. 3 * c_in/32 accumulator blocks of 32x32.  MFMA 32x32x16 bf16 with M = output channel, N = input channel, K = position; both operands lie
// in LDS as [position][channel] and their fragments come from the transpose read, as in the generic update
// kernel.  Slices are double-buffered in LDS (one barrier per slice), the next one waits in registers.
// The fp32 sums of a workgroup go to partial[learner * splits + range][o][9 c_in] and the column sums of dZ
// to partial_bias, which conv_step_kernel adds up and applies to the master.
#include "kavg_internal.h"
#include "conv_wgrad.h"
#include "conv_pool.h"

namespace kavg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int IMG_W = 32;                    // image width the tiling is built for
constexpr int SLP = 2 * IMG_W;               // positions per slice: two image rows
constexpr int HALO_W = IMG_W + 2;            // pixels of a halo row: a zero pixel on either side
constexpr int HALO_PX = 4 * HALO_W;          // the slice's two rows, one above, one below

template <int C_IN, int C_OUT>
struct WgradShape {
    static constexpr int OB = C_OUT / 32, NB = C_IN / 32, NW = 3 * OB, NT = 64 * NW;
    static constexpr int ZP = C_OUT + 32, AP = C_IN + 32;      // LDS rows: channels plus 64 bytes (transpose reads stay off each other's banks)
    static constexpr int Z_ELEMS = SLP * ZP, A_ELEMS = HALO_PX * AP, BUF = Z_ELEMS + A_ELEMS;
    static constexpr int SMEM = 2 * BUF * 2;
    static constexpr int Z_PIECES = SLP * C_OUT / 8, A_PIECES = 4 * IMG_W * C_IN / 8;
    static constexpr int ZN = (Z_PIECES + NT - 1) / NT, AN = (A_PIECES + NT - 1) / NT;
};

struct WgradArgs {
    const uint16_t* dz; size_t dz_lstride;       // [learner][B*H*W][C_OUT]
    const uint16_t* in; size_t in_lstride;       // [learner][B*H*W][C_IN]
    float* partial; float* partial_bias;
    int H, images, splits;                       // images per workgroup; ranges per learner
    // dpool != null: dz holds this layer's activations, and the gradient is formed from them and
    // dpool[learner][image][C_OUT] while loading (conv_pool.h)
    const uint16_t* dpool; size_t dpool_lstride; float inv;
};

// Fragment of a [position][channel] LDS tile for one 16-position slab: lane l receives channel x0 + l%32 at
// positions 8 (l/32) .. +7 of the slab (row0 = LDS row of the slab's first position).  In its 16-lane group,
// lane t = 4a + b fetches channels 4b .. 4b+3 of row a and receives the four rows of channel t.
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t* tile, int pitch, int row0, int x0, int lane) {
    const int t = lane & 15, grp = lane >> 4;
    const uint16_t* p = tile + (row0 + (grp >> 1) * 8 + (t >> 2)) * pitch + x0 + (grp & 1) * 16 + (t & 3) * 4;
    typedef bf16x4 __attribute__((address_space(3))) * lds_ptr;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)p);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(p + 4 * pitch));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

constexpr int POOL_IMAGES_MAX = 64;          // images of a workgroup whose dpool rows are kept in LDS

// POOL: dZ is formed from the layer's activations and dpool while the slice is written to LDS
template <int C_IN, int C_OUT, bool POOL>
__global__ void __launch_bounds__(64 * 3 * (C_OUT / 32)) conv_wgrad_halo_kernel(WgradArgs a) {
    typedef WgradShape<C_IN, C_OUT> SH;
    constexpr int OB = SH::OB, NB = SH::NB, NT = SH::NT, ZP = SH::ZP, AP = SH::AP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* const lds = (uint16_t*)smem;       // buffer b: dZ rows at lds + b*BUF, halo at + Z_ELEMS
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // A wavefront owns the taps with dx = tl - 1 and, of the OB x NB blocks (output channels x input channels), either
    // one output block and all input blocks or -- when there are two input blocks and an even number of output
    // blocks -- two output blocks and one input block: the same six accumulator blocks, five fragment reads per
    // slab instead of seven.
    constexpr bool PAIR = NB == 2 && OB % 2 == 0;
    constexpr int OI = PAIR ? 2 : 1, NI = PAIR ? 1 : NB;
    const int tl = wave / OB;
    const int ob0 = PAIR ? ((wave % OB) >> 1) * 2 : wave % OB, nb0 = PAIR ? (wave % OB) & 1 : 0;
    const int lp = blockIdx.x, learner = lp / a.splits, range = lp - learner * a.splits;
    const int H = a.H, half = H / 2;
    const size_t pos0 = (size_t)range * a.images * H * IMG_W;
    const uint16_t* dz = a.dz + (size_t)learner * a.dz_lstride + pos0 * C_OUT;
    const uint16_t* in = a.in + (size_t)learner * a.in_lstride + pos0 * C_IN;
    const int slices = a.images * half;

    // the zero pixels left and right of every halo row, both buffers: never written again
    for (int e = tid; e < 2 * 4 * 2 * (C_IN / 8); e += NT) {
        const int ch8 = e % (C_IN / 8), side = (e / (C_IN / 8)) % 2, row = (e / (C_IN / 8) / 2) % 4, b = e / (C_IN / 8) / 8;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *(u32x4*)(lds + b * SH::BUF + SH::Z_ELEMS + (row * HALO_W + side * (HALO_W - 1)) * AP + ch8 * 8) = zero;
    }

    // the dpool rows of this workgroup's images: behind the two slice buffers
    uint16_t* const gl = lds + 2 * SH::BUF;
    if constexpr (POOL) {
        const uint16_t* dpool = a.dpool + (size_t)learner * a.dpool_lstride + (size_t)range * a.images * C_OUT;
        for (int e = tid; e < a.images * (C_OUT / 8); e += NT) *(u32x4*)(gl + e * 8) = *(const u32x4*)(dpool + (size_t)e * 8);
    }
    u32x4 zr[SH::ZN], ar[SH::AN];
    unsigned a_ok = 0;                           // bit i: piece i of the halo in the registers lies inside the image
    auto fetch = [&](int s) {
        const int b = s / half, h0 = (s - b * half) * 2;
        const uint16_t* zsrc = dz + ((size_t)b * H + h0) * IMG_W * C_OUT;        // 64 positions, contiguous
#pragma unroll
        for (int i = 0; i < SH::ZN; ++i) {
            const int e = min(tid + NT * i, SH::Z_PIECES - 1);
            zr[i] = *(const u32x4*)(zsrc + (size_t)e * 8);
        }
        a_ok = 0;
#pragma unroll
        for (int i = 0; i < SH::AN; ++i) {
            const int e = min(tid + NT * i, SH::A_PIECES - 1);
            const int row = e / (IMG_W * C_IN / 8), rest = e - row * (IMG_W * C_IN / 8);     // rest = pixel * (C_IN/8) + chunk
            const int h = h0 - 1 + row;
            const bool ok = h >= 0 && h < H;
            if (ok) a_ok |= 1u << i;
            ar[i] = *(const u32x4*)(in + (((size_t)b * H + (ok ? h : h0)) * IMG_W) * C_IN + (size_t)rest * 8);
        }
    };
    auto stash = [&](int buf, int s) {           // s: the slice in the registers
        const int b = s / half;
        uint16_t* Z = lds + buf * SH::BUF;
        uint16_t* A = Z + SH::Z_ELEMS;
#pragma unroll
        for (int i = 0; i < SH::ZN; ++i) {
            const int e = tid + NT * i;
            if (e < SH::Z_PIECES) {
                u32x4 v = zr[i];
                if constexpr (POOL) v = pool_grad_piece(v, *(const u32x4*)(gl + b * C_OUT + (e % (C_OUT / 8)) * 8), a.inv);
                *(u32x4*)(Z + (e / (C_OUT / 8)) * ZP + (e % (C_OUT / 8)) * 8) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < SH::AN; ++i) {
            const int e = tid + NT * i;
            if (e < SH::A_PIECES) {
                const int row = e / (IMG_W * C_IN / 8), rest = e - row * (IMG_W * C_IN / 8);
                const int px = rest / (C_IN / 8), ch8 = rest - px * (C_IN / 8);
                const u32x4 zero = {0u, 0u, 0u, 0u};
                *(u32x4*)(A + (row * HALO_W + px + 1) * AP + ch8 * 8) = ((a_ok >> i) & 1u) ? ar[i] : zero;
            }
        }
    };

    f32x16 acc[3][OI][NI];
#pragma unroll
    for (int ty = 0; ty < 3; ++ty)
#pragma unroll
        for (int oi = 0; oi < OI; ++oi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[ty][oi][ni][e] = 0.f;
    // column sums of dZ: the workgroup has 6 threads per output channel (NT = 6 C_OUT); thread (g, ch) adds the
    // positions g, g + 6, ... of every slice, and the six partial sums are joined in fixed order at the end
    static_assert(NT == 6 * C_OUT, "six threads per output channel");
    const int bch = tid % C_OUT, bg = tid / C_OUT;
    float bias_sum = 0.f;

    fetch(0);
    if constexpr (POOL) __syncthreads();         // the dpool rows are in LDS
    stash(0, 0);
    __syncthreads();
    for (int s = 0; s < slices; ++s) {
        const int buf = s & 1;
        if (s + 1 < slices) fetch(s + 1);        // in flight during the MFMAs
        const uint16_t* Z = lds + buf * SH::BUF;
        const uint16_t* A = Z + SH::Z_ELEMS;
#pragma unroll
        for (int kq = 0; kq < SLP / 16; ++kq) {
            // slab kq: positions 16 kq .. +15 = image row kq/2 of the slice, pixels 16 (kq%2) .. +15
            bf16x8 zf[OI];
#pragma unroll
            for (int oi = 0; oi < OI; ++oi) zf[oi] = frag_tr(Z, ZP, kq * 16, (ob0 + oi) * 32, lane);
            const int r = kq >> 1, w0 = (kq & 1) * 16;
#pragma unroll
            for (int ty = 0; ty < 3; ++ty) {
                // tap (dy, dx) = (ty - 1, tl - 1): halo row r + 1 + dy, halo pixel w0 + 1 + dx
                const int row0 = (r + ty) * HALO_W + w0 + tl;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const bf16x8 af = frag_tr(A, AP, row0, (nb0 + ni) * 32, lane);
#pragma unroll
                    for (int oi = 0; oi < OI; ++oi)
                        acc[ty][oi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zf[oi], af, acc[ty][oi][ni], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < SLP; k += 6)
            if (k + bg < SLP) bias_sum += __builtin_bit_cast(float, (uint32_t)Z[(k + bg) * ZP + bch] << 16);
        if (s + 1 < slices) stash(buf ^ 1, s + 1);   // the other buffer: last read before the previous barrier
        __syncthreads();
    }

    // accumulator e of a block: output channel 8 (e/4) + 4 (lane/32) + e%4, input channel lane%32
    float* out = a.partial + (size_t)lp * C_OUT * 9 * C_IN;
#pragma unroll
    for (int ty = 0; ty < 3; ++ty)
#pragma unroll
        for (int oi = 0; oi < OI; ++oi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int o = (ob0 + oi) * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    out[(size_t)o * 9 * C_IN + (ty * 3 + tl) * C_IN + (nb0 + ni) * 32 + (lane & 31)] = acc[ty][oi][ni][e];
                }
    float* red = (float*)smem;                   // (the tiles are dead: the loop ended with a barrier)
    red[bg * C_OUT + bch] = bias_sum;
    __syncthreads();
    if (tid < C_OUT) {
        float b = 0.f;
#pragma unroll
        for (int g = 0; g < 6; ++g) b += red[g * C_OUT + tid];
        a.partial_bias[(size_t)lp * C_OUT + tid] = b;
    }
}

template <int C_IN, int C_OUT, bool POOL>
hipError_t launch_wgrad_as(const WgradArgs& a, int P, hipStream_t st) {
    typedef WgradShape<C_IN, C_OUT> SH;
    constexpr int SMEM = SH::SMEM + (POOL ? POOL_IMAGES_MAX * C_OUT * 2 : 0);
    static_assert(SMEM <= 160 * 1024, "more LDS than a compute unit has");
    static_assert(3 * SH::NB * 16 <= 96, "accumulators leave room for three wavefronts per SIMD");
    if (SMEM > 64 * 1024) {
        static hipError_t raised = hipFuncSetAttribute((const void*)conv_wgrad_halo_kernel<C_IN, C_OUT, POOL>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        if (raised != hipSuccess) return raised;
    }
    hipLaunchKernelGGL((conv_wgrad_halo_kernel<C_IN, C_OUT, POOL>), dim3(P * a.splits), dim3(SH::NT), SMEM, st, a);
    return hipGetLastError();
}
template <int C_IN, int C_OUT>
hipError_t launch_wgrad(const WgradArgs& a, int P, hipStream_t st) {
    return a.dpool ? launch_wgrad_as<C_IN, C_OUT, true>(a, P, st) : launch_wgrad_as<C_IN, C_OUT, false>(a, P, st);
}

}  // namespace

int conv_wgrad_halo_pool_images() { return POOL_IMAGES_MAX; }

int conv_wgrad_halo_splits(int P, int B, int H, int W, int c_in, int c_out) {
    if (W != IMG_W || H < 2 || H % 2 != 0 || P < 1 || B < 1) return 0;
    if (!(c_in == 32 || c_in == 64) || !(c_out == 32 || c_out == 64 || c_out == 128)) return 0;
    // ranges of whole images, enough of them for one workgroup per compute unit where the batch allows -- two
    // where two fit (LDS: up to 64 input and output channels)
    const int target = (c_in <= 64 && c_out <= 64) ? 512 : 256;
    int S = 1;
    while (P * S < target && B % (2 * S) == 0) S *= 2;
    return S;
}

hipError_t conv_wgrad_halo(const ConvCall& c, const void* dpool, hipStream_t st) {
    if (conv_wgrad_halo_splits(c.P, c.B, c.H, c.W, c.c_in, c.c_out) == 0 || c.splits < 1 || c.B % c.splits != 0 || !c.partial || (dpool && (!c.out || c.B / c.splits > POOL_IMAGES_MAX)) ||
        !c.partial_bias)
        return hipErrorInvalidValue;
    WgradArgs a;
    const size_t rows = (size_t)c.B * c.H * c.W;
    a.dz = (const uint16_t*)(dpool ? c.out : c.dz); a.dz_lstride = rows * c.c_out;
    a.in = (const uint16_t*)c.in; a.in_lstride = rows * c.c_in;
    a.partial = c.partial; a.partial_bias = c.partial_bias;
    a.H = c.H; a.images = c.B / c.splits; a.splits = c.splits;
    a.dpool = (const uint16_t*)dpool; a.dpool_lstride = (size_t)c.B * c.c_out; a.inv = 1.0f / (float)(c.H * c.W);
    if (c.c_in == 32) {
        if (c.c_out == 32) return launch_wgrad<32, 32>(a, c.P, st);
        if (c.c_out == 64) return launch_wgrad<32, 64>(a, c.P, st);
        return launch_wgrad<32, 128>(a, c.P, st);
    }
    if (c.c_out == 32) return launch_wgrad<64, 32>(a, c.P, st);
    if (c.c_out == 64) return launch_wgrad<64, 64>(a, c.P, st);
    return launch_wgrad<64, 128>(a, c.P, st);
}

}  // namespace kavg
