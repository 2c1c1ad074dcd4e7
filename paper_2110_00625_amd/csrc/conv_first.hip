// The first 3x3 convolution of the learner (stride 1, zero padding 1): 8 input channels, images 32 pixels
// wide that are gathered out of the data set by the step's minibatch indices.  Forward pass and weight
// gradient (there is no data gradient below the first layer) without a patch matrix:
//
//   forward          out[p][o] = relu( b[o] + sum over (tap, c) of x[p + (dy, dx)][c] * W[o][tap][c] )
//   weight gradient  dW[o][tap][c] = sum over positions p of dZ[p][o] * x[p + (dy, dx)][c]
//
// (the learner's forward pass and update of Algorithm 1; tap = 3 (dy+1) + (dx+1)).  With 8 channels a
// pixel is one 16-byte piece and the whole contraction of the forward pass, 9 x 8 = 72, is five k slabs
// of the 32x32x16 matrix instruction: slab kq holds taps 2 kq and 2 kq + 1, one per half of the
// wavefront, so a lane's operand is the pixel its own tap points at in the image tile in LDS (eight rows
// plus one above and below, a zero pixel on either side); the tenth tap has zero weights.  The weight
// gradient runs over 8-row slices of whole images like the all-taps kernel of the later layers, with the
// 72 columns (tap, channel) spread over three 32-column blocks (24 of the 96 columns are never stored).
#include "kavg_internal.h"
#include "conv_first.h"
#include "split.h"

namespace kavg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int IMG_W = 32, CH = 8;            // image width and input channels this file is built for
constexpr int ROWS = 8;                      // image rows per tile / slice
constexpr int HALO_W = IMG_W + 2;
constexpr int HALO_PX = (ROWS + 2) * HALO_W;
constexpr int KW = 9 * CH;                   // 72 columns (tap, channel)
constexpr int WPITCH = 88;                   // LDS row of the forward weights: 80 (five slabs) plus 16 bytes
constexpr int OPITCH = 32 + 8;               // output patch of a wavefront: [32 pixels][32 channels + 16 bytes]

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;          // round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

struct FirstArgs {
    const uint16_t* X; const int32_t* idx; long idx_lstride;     // data set [N][H][32][8]; the step's rows per learner
    int H, B;
    // forward
    const uint16_t* w; size_t w_lstride;                 // hi plane of W [c_out][9][8]
    const uint16_t* bhi; const uint16_t* blo;            // bias planes (learner stride w_lstride)
    uint16_t* out; size_t out_lstride;                   // [learner][B*H*32][c_out]
    // weight gradient
    const uint16_t* dz; size_t dz_lstride;               // [learner][B*H*32][c_out]
    float* partial; float* partial_bias; int splits, images;
};

// the tile rows h0 - 1 .. h0 + 8 of one image: one 16-byte piece per pixel, zeros outside the image
__device__ __forceinline__ u32x4 tile_piece(const uint16_t* img, int H, int h0, int e) {
    const int row = e / IMG_W, px = e - row * IMG_W;
    const int h = h0 - 1 + row;
    const bool ok = h >= 0 && h < H;
    const u32x4 x = *(const u32x4*)(img + ((size_t)(ok ? h : h0) * IMG_W + px) * CH);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    return ok ? x : zero;
}

template <int CN>
__global__ void __launch_bounds__(64 * ROWS) conv_first_forward_kernel(FirstArgs a) {
    constexpr int NT = 64 * ROWS, NB = CN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* const IN = (uint16_t*)smem;                    // [HALO_PX][8]
    uint16_t* const WT = IN + HALO_PX * CH;                  // [CN][WPITCH]
    uint16_t* const PATCH = WT + CN * WPITCH;                // [ROWS][32][OPITCH]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles_per_image = a.H / ROWS, tiles = a.B * tiles_per_image;
    const int learner = blockIdx.x / tiles, tile = blockIdx.x - learner * tiles;
    const int b = tile / tiles_per_image, row0 = (tile - b * tiles_per_image) * ROWS;
    const uint16_t* img = a.X + (size_t)a.idx[(long)learner * a.idx_lstride + b] * a.H * IMG_W * CH;
    const uint16_t* w = a.w + (size_t)learner * a.w_lstride;

    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int e = tid; e < (ROWS + 2) * IMG_W; e += NT)
        *(u32x4*)(IN + ((e / IMG_W) * HALO_W + e % IMG_W + 1) * CH) = tile_piece(img, a.H, row0, e);
    for (int e = tid; e < (ROWS + 2) * 2; e += NT)               // the zero pixels left and right
        *(u32x4*)(IN + ((e >> 1) * HALO_W + (e & 1) * (HALO_W - 1)) * CH) = zero;
    for (int e = tid; e < CN * 10; e += NT) {                    // W[o][72] and the zero tenth tap
        const int o = e / 10, t = e - o * 10;
        *(u32x4*)(WT + o * WPITCH + t * CH) = t < 9 ? *(const u32x4*)(w + (size_t)o * KW + t * CH) : zero;
    }
    __syncthreads();

    f32x16 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
#pragma unroll
    for (int kq = 0; kq < 5; ++kq) {
        const int tap = min(2 * kq + (lane >> 5), 8);            // (the tenth tap meets zero weights: any pixel will do)
        const int dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
        const bf16x8 xf = *(const bf16x8*)(IN + ((wave + 1 + dy) * HALO_W + (lane & 31) + 1 + dx) * CH);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const bf16x8 wf = *(const bf16x8*)(WT + (j * 32 + (lane & 31)) * WPITCH + kq * 16 + (lane >> 5) * 8);
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[j], 0, 0, 0);
        }
    }

    // accumulator e of block j = output channel 32 j + 8 (e/4) + 4 (lane/32) + e%4 at pixel lane%32 of row `wave`
    uint16_t* out = a.out + (size_t)learner * a.out_lstride + (((size_t)b * a.H + row0 + wave) * IMG_W) * CN;
    uint16_t* patch = PATCH + wave * 32 * OPITCH;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = j * 32 + q * 8 + (lane >> 5) * 4;
            const u32x2 h2 = *(const u32x2*)(a.bhi + (size_t)learner * a.w_lstride + n);
            const u32x2 l2 = *(const u32x2*)(a.blo + (size_t)learner * a.w_lstride + n);
            uint32_t b0, b1, b2, b3;
            split_join2(h2.x, l2.x, b0, b1);
            split_join2(h2.y, l2.y, b2, b3);
            const float v0 = fmaxf(acc[j][4 * q + 0] + __builtin_bit_cast(float, b0), 0.f);
            const float v1 = fmaxf(acc[j][4 * q + 1] + __builtin_bit_cast(float, b1), 0.f);
            const float v2 = fmaxf(acc[j][4 * q + 2] + __builtin_bit_cast(float, b2), 0.f);
            const float v3 = fmaxf(acc[j][4 * q + 3] + __builtin_bit_cast(float, b3), 0.f);
            *(u32x2*)(patch + (lane & 31) * OPITCH + q * 8 + (lane >> 5) * 4) = (u32x2){pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
        }
        // (the patch is this wavefront's own, and a wavefront's LDS accesses complete in order)
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int id = pass * 64 + lane, px = id >> 2, ch = id & 3;
            *(u32x4*)(out + (size_t)px * CN + j * 32 + ch * 8) = *(const u32x4*)(patch + px * OPITCH + ch * 8);
        }
    }
}

// Weight gradient.  Workgroup = (learner, range of whole images); 3 * C_OUT/32 wavefronts: wavefront (ob, nbk)
// owns output channels 32 ob .. +31 and columns 32 nbk .. +31 of the 72 (tap, channel) columns.
template <int C_OUT>
struct FirstWgradShape {
    static constexpr int OB = C_OUT / 32, NW = 3 * OB, NT = 64 * NW;
    static constexpr int SLP = ROWS * IMG_W;                 // positions per slice
    static constexpr int ZP = C_OUT + 32;                    // dZ rows in LDS: channels plus 64 bytes
    static constexpr int Z_ELEMS = SLP * ZP, A_ELEMS = HALO_PX * CH, BUF = Z_ELEMS + A_ELEMS;
    static constexpr int SMEM = 2 * BUF * 2;
    static constexpr int Z_PIECES = SLP * C_OUT / 8, A_PIECES = (ROWS + 2) * IMG_W;
    static constexpr int ZN = (Z_PIECES + NT - 1) / NT, AN = (A_PIECES + NT - 1) / NT;
};

template <int C_OUT>
__global__ void __launch_bounds__(64 * 3 * (C_OUT / 32)) conv_first_wgrad_kernel(FirstArgs a) {
    typedef FirstWgradShape<C_OUT> SH;
    constexpr int OB = SH::OB, NT = SH::NT, ZP = SH::ZP, SLP = SH::SLP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* const lds = (uint16_t*)smem;       // buffer b: dZ rows at lds + b*BUF, image tile at + Z_ELEMS
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ob = wave % OB, nbk = wave / OB;
    const int lp = blockIdx.x, learner = lp / a.splits, range = lp - learner * a.splits;
    const int H = a.H, per_image = H / ROWS;
    const int img0 = range * a.images;
    const uint16_t* dz = a.dz + (size_t)learner * a.dz_lstride + (size_t)img0 * H * IMG_W * C_OUT;
    const int32_t* idx = a.idx + (long)learner * a.idx_lstride + img0;
    const int slices = a.images * per_image;

    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int e = tid; e < 2 * (ROWS + 2) * 2; e += NT) {         // the zero pixels left and right, both buffers
        const int b = e / ((ROWS + 2) * 2), r = e - b * (ROWS + 2) * 2;
        *(u32x4*)(lds + b * SH::BUF + SH::Z_ELEMS + ((r >> 1) * HALO_W + (r & 1) * (HALO_W - 1)) * CH) = zero;
    }

    u32x4 zr[SH::ZN], ar[SH::AN];
    auto fetch = [&](int s) {
        const int b = s / per_image, h0 = (s - b * per_image) * ROWS;
        const uint16_t* zsrc = dz + ((size_t)b * H + h0) * IMG_W * C_OUT;        // SLP positions, contiguous
#pragma unroll
        for (int i = 0; i < SH::ZN; ++i) zr[i] = *(const u32x4*)(zsrc + (size_t)min(tid + NT * i, SH::Z_PIECES - 1) * 8);
        const uint16_t* img = a.X + (size_t)idx[b] * H * IMG_W * CH;
#pragma unroll
        for (int i = 0; i < SH::AN; ++i) ar[i] = tile_piece(img, H, h0, min(tid + NT * i, SH::A_PIECES - 1));
    };
    auto stash = [&](int buf) {
        uint16_t* Z = lds + buf * SH::BUF;
        uint16_t* A = Z + SH::Z_ELEMS;
#pragma unroll
        for (int i = 0; i < SH::ZN; ++i) {
            const int e = tid + NT * i;
            if (e < SH::Z_PIECES) *(u32x4*)(Z + (e / (C_OUT / 8)) * ZP + (e % (C_OUT / 8)) * 8) = zr[i];
        }
#pragma unroll
        for (int i = 0; i < SH::AN; ++i) {
            const int e = tid + NT * i;
            if (e < SH::A_PIECES) *(u32x4*)(A + ((e / IMG_W) * HALO_W + e % IMG_W + 1) * CH) = ar[i];
        }
    };

    // This lane's part of the transpose reads: in its 16-lane group, lane t = 4a + b fetches columns 4b .. 4b+3 of
    // position a (four channels of one tap's pixel) and receives the four positions of column t.
    const int t16 = lane & 15, grp = lane >> 4;
    const int xn = nbk * 32 + (grp & 1) * 16 + (t16 & 3) * 4;       // first of the four columns this lane fetches
    const int tap = min(xn / CH, 8);                                 // (columns 72 .. 95 are never stored)
    const int dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
    const int a_lane = ((1 + dy) * HALO_W + 1 + dx + (grp >> 1) * 8 + (t16 >> 2)) * CH + xn % CH;
    const int z_lane = ((grp >> 1) * 8 + (t16 >> 2)) * ZP + ob * 32 + (grp & 1) * 16 + (t16 & 3) * 4;
    typedef bf16x4 __attribute__((address_space(3))) * lds_ptr;

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    static_assert(NT == 6 * C_OUT, "six threads per output channel");
    const int bch = tid % C_OUT, bg = tid / C_OUT;
    float bias_sum = 0.f;

    fetch(0);
    stash(0);
    __syncthreads();
    for (int s = 0; s < slices; ++s) {
        const int buf = s & 1;
        if (s + 1 < slices) fetch(s + 1);
        const uint16_t* Z = lds + buf * SH::BUF;
        const uint16_t* A = Z + SH::Z_ELEMS;
#pragma unroll 4
        for (int kq = 0; kq < SLP / 16; ++kq) {
            // slab kq: image row kq/2 of the slice, pixels 16 (kq%2) .. +15
            const uint16_t* zp = Z + kq * 16 * ZP + z_lane;
            const bf16x4 zlo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)zp);
            const bf16x4 zhi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(zp + 4 * ZP));
            const uint16_t* ap = A + ((kq >> 1) * HALO_W + (kq & 1) * 16) * CH + a_lane;
            const bf16x4 alo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)ap);
            const bf16x4 ahi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(ap + 4 * CH));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_shufflevector(zlo, zhi, 0, 1, 2, 3, 4, 5, 6, 7),
                                                          __builtin_shufflevector(alo, ahi, 0, 1, 2, 3, 4, 5, 6, 7), acc, 0, 0, 0);
        }
        for (int k = bg; k < SLP; k += 6) bias_sum += __builtin_bit_cast(float, (uint32_t)Z[k * ZP + bch] << 16);
        if (s + 1 < slices) stash(buf ^ 1);
        __syncthreads();
    }

    // accumulator e: output channel 32 ob + 8 (e/4) + 4 (lane/32) + e%4, column 32 nbk + lane%32
    const int col = nbk * 32 + (lane & 31);
    if (col < KW) {
        float* out = a.partial + (size_t)lp * C_OUT * KW;
#pragma unroll
        for (int e = 0; e < 16; ++e) out[(size_t)(ob * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)) * KW + col] = acc[e];
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

template <int CN>
hipError_t launch_first_forward(const FirstArgs& a, int P, hipStream_t st) {
    constexpr int SMEM = (HALO_PX * CH + CN * WPITCH + ROWS * 32 * OPITCH) * 2;
    static_assert(SMEM <= 64 * 1024, "within the default LDS limit");
    hipLaunchKernelGGL((conv_first_forward_kernel<CN>), dim3(P * a.B * (a.H / ROWS)), dim3(64 * ROWS), SMEM, st, a);
    return hipGetLastError();
}

template <int C_OUT>
hipError_t launch_first_wgrad(const FirstArgs& a, int P, hipStream_t st) {
    typedef FirstWgradShape<C_OUT> SH;
    static_assert(SH::SMEM <= 160 * 1024, "more LDS than a compute unit has");
    if (SH::SMEM > 64 * 1024) {
        static hipError_t raised = hipFuncSetAttribute((const void*)conv_first_wgrad_kernel<C_OUT>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, SH::SMEM);
        if (raised != hipSuccess) return raised;
    }
    hipLaunchKernelGGL((conv_first_wgrad_kernel<C_OUT>), dim3(P * a.splits), dim3(SH::NT), SH::SMEM, st, a);
    return hipGetLastError();
}

}  // namespace

int conv_first_splits(int P, int B, int H, int W, int c_in, int c_out) {
    if (W != IMG_W || c_in != CH || H < ROWS || H % ROWS != 0 || P < 1 || B < 1 || !(c_out == 32 || c_out == 64)) return 0;
    // two workgroups per compute unit where the batch allows: a slice is short, and one workgroup alone would
    // wait out the latency of every slice's loads
    int S = 1;
    while (P * S < 512 && B % (2 * S) == 0) S *= 2;
    return S;
}

hipError_t conv_first_forward(const ConvCall& c, const void* X, const int32_t* idx, long idx_lstride, hipStream_t st) {
    if (conv_first_splits(c.P, c.B, c.H, c.W, c.c_in, c.c_out) == 0 || !X || !idx || !c.out) return hipErrorInvalidValue;
    FirstArgs a = {};
    a.X = (const uint16_t*)X; a.idx = idx; a.idx_lstride = idx_lstride; a.H = c.H; a.B = c.B;
    a.w = c.ws; a.w_lstride = c.ws_stride; a.bhi = c.bhi; a.blo = c.blo;
    a.out = (uint16_t*)c.out; a.out_lstride = (size_t)c.B * c.H * c.W * c.c_out;
    return c.c_out == 32 ? launch_first_forward<32>(a, c.P, st) : launch_first_forward<64>(a, c.P, st);
}

hipError_t conv_first_wgrad(const ConvCall& c, const void* X, const int32_t* idx, long idx_lstride, hipStream_t st) {
    if (conv_first_splits(c.P, c.B, c.H, c.W, c.c_in, c.c_out) == 0 || !X || !idx || !c.dz || !c.partial || !c.partial_bias ||
        c.splits < 1 || c.B % c.splits != 0)
        return hipErrorInvalidValue;
    FirstArgs a = {};
    a.X = (const uint16_t*)X; a.idx = idx; a.idx_lstride = idx_lstride; a.H = c.H; a.B = c.B;
    a.dz = (const uint16_t*)c.dz; a.dz_lstride = (size_t)c.B * c.H * c.W * c.c_out;
    a.partial = c.partial; a.partial_bias = c.partial_bias; a.splits = c.splits; a.images = c.B / c.splits;
    return c.c_out == 32 ? launch_first_wgrad<32>(a, c.P, st) : launch_first_wgrad<64>(a, c.P, st);
}

}  // namespace kavg
