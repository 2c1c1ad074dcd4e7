// 3x3 convolution (stride 1, zero padding 1) on channels-last bf16 images 32 pixels wide, forward and data
// gradient, with the image rows a workgroup needs held in LDS once:
//
//   forward        out[p][o] = relu( b[o] + sum over (tap, c) of in[p + (dy, dx)][c] * W[o][tap][c] )
//   data gradient  din[p][c] = [act[p][c] > 0] * sum over (tap, o) of dz[p - (dy, dx)][o] * W[o][tap][c]
//
// (the learner's forward and backward pass of Algorithm 1 through a convolutional layer; tap = 3 (dy+1) +
// (dx+1)).  The generic kernel forms the patch matrix in its operand loaders, which reads every input
// pixel nine times out of L2; here a workgroup owns eight image rows (256 positions) and all output
// channels, loads those rows plus one above and one below (a zero pixel on either side) into LDS, and
// every tap reads the same tile at a shifted pixel.  Only the weights still stream: one slice of
// [channels out][channels in] per tap, one to three taps per step (as many as leave LDS for two workgroups
// per compute unit), single LDS buffer, the slices of the next two steps waiting in registers.
//
// Eight wavefronts, one per image row: wavefront w holds the 32 positions of row w times all N output
// channels (N/32 accumulator blocks).  MFMA 32x32x16 bf16 with the weights as the first operand
// (accumulator registers run over output channels) and the pixels as the second (lanes run over the
// positions of the row).  Contraction channels are taken in groups of at most 64 (a layer with 128 of them
// runs the nine taps twice, reloading the tile with the other half), so the tile stays below 50 KB and two
// workgroups share a compute unit.  Outputs leave through a per-wavefront LDS patch as 64-byte row segments.
#include "kavg_internal.h"
#include "conv_direct.h"
#include "split.h"
#include "conv_pool.h"
#include <type_traits>

namespace kavg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int IMG_W = 32;                    // image width the tiling is built for
constexpr int ROWS = 8;                      // image rows per workgroup, one per wavefront
constexpr int NT = 64 * ROWS;
constexpr int HALO_W = IMG_W + 2;            // pixels of a tile row: a zero pixel on either side
constexpr int HALO_PX = (ROWS + 2) * HALO_W;
constexpr int OPITCH = 32 + 8;               // output patch of a wavefront: [32 pixels][32 channels + 16 bytes]

// CK: contraction channels per group (32 or 64); CN: output channels; BWD: data gradient
template <int CK, int CN, bool BWD>
struct DirectShape {
    static constexpr int IP = CK + 8;                            // LDS pixel: its channels plus 16 bytes
    static constexpr int IN_ELEMS = HALO_PX * IP;
    static constexpr int WP = BWD ? CN + 32 : CK + 8;            // weight slice rows: [k][n] for the data gradient (transpose reads), [n][k] forward
    static constexpr int W_ROWS = BWD ? CK : CN, W_COLS = BWD ? CN : CK;
    static constexpr int W_ELEMS = W_ROWS * WP;                  // one tap's slice
    // taps per step (one weight buffer, two barriers per step): as many as leave room for two workgroups per compute unit
    static constexpr int TPS = 2 * (IN_ELEMS + 3 * W_ELEMS) * 2 <= 160 * 1024 ? 3 : 2 * (IN_ELEMS + 2 * W_ELEMS) * 2 <= 160 * 1024 ? 2 : 1;
    static constexpr int STEPS = (9 + TPS - 1) / TPS;            // per channel group
    static constexpr int SMEM = (IN_ELEMS + TPS * W_ELEMS) * 2;
    static constexpr int W_PIECES = W_ROWS * W_COLS / 8, WN = (W_PIECES + NT - 1) / NT;
    static constexpr int IN_PIECES = (ROWS + 2) * IMG_W * CK / 8, INN = (IN_PIECES + NT - 1) / NT;
    static constexpr int NB = CN / 32;
};

struct DirectArgs {
    const uint16_t* in; size_t in_lstride; int c_k;      // images of c_k contraction channels
    const uint16_t* w; size_t w_lstride;                 // hi plane of W [c_out][9][c_in]
    const uint16_t* bhi; const uint16_t* blo; size_t b_lstride;      // forward: bias planes
    const uint16_t* act;                                 // data gradient: activations of the layer below (CN channels, same strides as out)
    uint16_t* out; size_t out_lstride;
    int H, tiles;                                        // tiles (of 8 rows) per learner
    // data gradient of the last convolution: dpool != null means `in` holds that layer's activations and the
    // gradient images are formed from them and dpool[learner][image][c_k] while loading (conv_pool.h)
    const uint16_t* dpool; size_t dpool_lstride; float inv;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;          // round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

// fragment of a [k][x] LDS tile by transpose reads: lane l receives x0 + l%32 at k = row0 + 8 (l/32) .. +7
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t* tile, int pitch, int row0, int x0, int lane) {
    const int t = lane & 15, grp = lane >> 4;
    const uint16_t* p = tile + (row0 + (grp >> 1) * 8 + (t >> 2)) * pitch + x0 + (grp & 1) * 16 + (t & 3) * 4;
    typedef bf16x4 __attribute__((address_space(3))) * lds_ptr;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)p);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(p + 4 * pitch));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// POOL (data gradient only): the gradient images are formed from activations and dpool while the tile is loaded
template <int CK, int CN, bool BWD, bool POOL = false>
__global__ void __launch_bounds__(NT, 4) conv_direct_kernel(DirectArgs a) {
    typedef DirectShape<CK, CN, BWD> SH;
    constexpr int IP = SH::IP, WP = SH::WP, NB = SH::NB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* const IN = (uint16_t*)smem;
    uint16_t* const WT = IN + SH::IN_ELEMS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int learner = blockIdx.x / a.tiles, tile = blockIdx.x - learner * a.tiles;
    const int H = a.H, tiles_per_image = H / ROWS;
    const int b = tile / tiles_per_image, row0 = (tile - b * tiles_per_image) * ROWS;
    const uint16_t* in = a.in + (size_t)learner * a.in_lstride + (size_t)b * H * IMG_W * a.c_k;
    const uint16_t* w = a.w + (size_t)learner * a.w_lstride;
    const int c_in = BWD ? CN : a.c_k;                   // W [c_out][9][c_in]
    const int groups = a.c_k / CK;

    // the zero pixels left and right of every tile row: never written again
    for (int e = tid; e < (ROWS + 2) * 2 * (CK / 8); e += NT) {
        const int ch8 = e % (CK / 8), side = (e / (CK / 8)) % 2, row = e / (CK / 8) / 2;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *(u32x4*)(IN + (row * HALO_W + side * (HALO_W - 1)) * IP + ch8 * 8) = zero;
    }

    // weight slice of (group g, tap): forward [n = o][k = c of the group], data gradient [k = o of the group][n = c]
    // Two slices wait in registers (sets 0 and 1 in turn): a slice is requested two taps before it is used,
    // which is about what a read out of L2 takes.
    constexpr int TPS = SH::TPS, STEPS = SH::STEPS;
    u32x4 wr[2][TPS][SH::WN];
    auto wfetch = [&](auto set, int s) {         // step s = (group, taps TPS*st .. ), taps beyond the ninth clamped (never used)
        const int g = s / STEPS, tap0 = (s - g * STEPS) * TPS;
#pragma unroll
        for (int tt = 0; tt < TPS; ++tt) {
            const int tap = min(tap0 + tt, 8);
#pragma unroll
            for (int i = 0; i < SH::WN; ++i) {
                const int e = min(tid + NT * i, SH::W_PIECES - 1);
                const int r = e / (SH::W_COLS / 8), c8 = e - r * (SH::W_COLS / 8);
                const int o = BWD ? g * CK + r : r;
                const int c = BWD ? c8 * 8 : g * CK + c8 * 8;
                wr[set][tt][i] = *(const u32x4*)(w + ((size_t)o * 9 + tap) * c_in + c);
            }
        }
    };
    auto wstash = [&](auto set) {
#pragma unroll
        for (int tt = 0; tt < TPS; ++tt)
#pragma unroll
            for (int i = 0; i < SH::WN; ++i) {
                const int e = tid + NT * i;
                if (e < SH::W_PIECES)
                    *(u32x4*)(WT + tt * SH::W_ELEMS + (e / (SH::W_COLS / 8)) * WP + (e % (SH::W_COLS / 8)) * 8) = wr[set][tt][i];
            }
    };
    // the tile's rows row0 - 1 .. row0 + 8 of channel group g: global -> registers -> LDS
    auto load_tile = [&](int g) {
        u32x4 v[SH::INN], gp[POOL ? SH::INN : 1];
        if constexpr (POOL) {                    // requested first, all at once
#pragma unroll
            for (int i = 0; i < SH::INN; ++i) {
                const int e = min(tid + NT * i, SH::IN_PIECES - 1);
                gp[i] = *(const u32x4*)(a.dpool + (size_t)learner * a.dpool_lstride + (size_t)b * a.c_k + g * CK + (e % (CK / 8)) * 8);
            }
        }
#pragma unroll
        for (int i = 0; i < SH::INN; ++i) {
            const int e = min(tid + NT * i, SH::IN_PIECES - 1);
            const int row = e / (IMG_W * CK / 8), rest = e - row * (IMG_W * CK / 8);
            const int px = rest / (CK / 8), ch8 = rest - px * (CK / 8);
            const int h = row0 - 1 + row;
            const bool ok = h >= 0 && h < H;
            const u32x4 x = *(const u32x4*)(in + ((size_t)(ok ? h : row0) * IMG_W + px) * a.c_k + g * CK + ch8 * 8);
            const u32x4 zero = {0u, 0u, 0u, 0u};
            v[i] = ok ? x : zero;                // (zero activations give a zero gradient below)
        }
        if constexpr (POOL) {
#pragma unroll
            for (int i = 0; i < SH::INN; ++i) v[i] = pool_grad_piece(v[i], gp[i], a.inv);
        }
#pragma unroll
        for (int i = 0; i < SH::INN; ++i) {
            const int e = tid + NT * i;
            if (e < SH::IN_PIECES) {
                const int row = e / (IMG_W * CK / 8), rest = e - row * (IMG_W * CK / 8);
                const int px = rest / (CK / 8), ch8 = rest - px * (CK / 8);
                *(u32x4*)(IN + (row * HALO_W + px + 1) * IP + ch8 * 8) = v[i];
            }
        }
    };

    f32x16 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

    const int steps = STEPS * groups;            // (channel group, TPS taps) in order
    auto step = [&](auto set, int s) {
        const int g = s / STEPS, tap0 = (s - g * STEPS) * TPS;
        if (tap0 == 0) load_tile(g);             // (the previous group's last step ended with a barrier)
        wstash(set);
        __syncthreads();                         // the slices (and, at the group's first step, the tile) are in LDS
        if (s + 2 < steps) wfetch(set, s + 2);
#pragma unroll
        for (int tt = 0; tt < TPS; ++tt) {
            const int tap = tap0 + tt;
            if (tap < 9) {
                const int dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
                // pixel this lane's position reads for the tap: forward p + (dy, dx), data gradient p - (dy, dx)
                const int pix = (wave + 1 + (BWD ? -dy : dy)) * HALO_W + (lane & 31) + 1 + (BWD ? -dx : dx);
                const uint16_t* ip = IN + pix * IP + (lane >> 5) * 8;
                const uint16_t* wt = WT + tt * SH::W_ELEMS;
#pragma unroll
                for (int kq = 0; kq < CK / 16; ++kq) {
                    const bf16x8 xf = *(const bf16x8*)(ip + kq * 16);
#pragma unroll
                    for (int j = 0; j < NB; ++j) {
                        bf16x8 wf;
                        if constexpr (BWD) wf = frag_tr(wt, WP, kq * 16, j * 32, lane);
                        else wf = *(const bf16x8*)(wt + (j * 32 + (lane & 31)) * WP + kq * 16 + (lane >> 5) * 8);
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[j], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();                         // everyone is done with the slices (and, after the last step, with the tile)
    };
    constexpr std::integral_constant<int, 0> set0;
    constexpr std::integral_constant<int, 1> set1;
    wfetch(set0, 0);
    if (steps > 1) wfetch(set1, 1);
    for (int s = 0; s < steps; s += 2) {
        step(set0, s);
        if (s + 1 < steps) step(set1, s + 1);
    }

    // epilogue: accumulator e of block j = output channel 32 j + 8 (e/4) + 4 (lane/32) + e%4 at pixel lane%32 of row `wave`
    const size_t pos_row = ((size_t)b * H + row0 + wave) * IMG_W;            // first position of this wavefront's row
    uint16_t* out = a.out + (size_t)learner * a.out_lstride + pos_row * CN;
    const uint16_t* act = BWD ? a.act + (size_t)learner * a.out_lstride + pos_row * CN : nullptr;
    uint16_t* patch = (uint16_t*)smem + wave * 32 * OPITCH;                  // (the tile is dead)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = j * 32 + q * 8 + (lane >> 5) * 4;
            float v0 = acc[j][4 * q + 0], v1 = acc[j][4 * q + 1], v2 = acc[j][4 * q + 2], v3 = acc[j][4 * q + 3];
            if constexpr (BWD) {
                const u32x2 m = *(const u32x2*)(act + (size_t)(lane & 31) * CN + n);
                // stored activations are ReLU outputs (never negative): positive <=> non-zero magnitude
                v0 = (m.x & 0x7FFFu) ? v0 : 0.f;
                v1 = (m.x & 0x7FFF0000u) ? v1 : 0.f;
                v2 = (m.y & 0x7FFFu) ? v2 : 0.f;
                v3 = (m.y & 0x7FFF0000u) ? v3 : 0.f;
            } else {
                const u32x2 h2 = *(const u32x2*)(a.bhi + (size_t)learner * a.b_lstride + n);
                const u32x2 l2 = *(const u32x2*)(a.blo + (size_t)learner * a.b_lstride + n);
                uint32_t b0, b1, b2, b3;
                split_join2(h2.x, l2.x, b0, b1);
                split_join2(h2.y, l2.y, b2, b3);
                v0 = fmaxf(v0 + __builtin_bit_cast(float, b0), 0.f);
                v1 = fmaxf(v1 + __builtin_bit_cast(float, b1), 0.f);
                v2 = fmaxf(v2 + __builtin_bit_cast(float, b2), 0.f);
                v3 = fmaxf(v3 + __builtin_bit_cast(float, b3), 0.f);
            }
            *(u32x2*)(patch + (lane & 31) * OPITCH + q * 8 + (lane >> 5) * 4) = (u32x2){pack_bf16x2(v0, v1), pack_bf16x2(v2, v3)};
        }
        // (the patch is this wavefront's own, and a wavefront's LDS accesses complete in order)
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int id = pass * 64 + lane, px = id >> 2, ch = id & 3;
            const u32x4 v = *(const u32x4*)(patch + px * OPITCH + ch * 8);
            *(u32x4*)(out + (size_t)px * CN + j * 32 + ch * 8) = v;
        }
    }
}

template <int CK, int CN, bool BWD, bool POOL = false>
hipError_t launch_direct(const DirectArgs& a, int P, hipStream_t st) {
    typedef DirectShape<CK, CN, BWD> SH;
    static_assert(2 * SH::SMEM <= 160 * 1024, "two workgroups per compute unit");
    static_assert(ROWS * 32 * OPITCH * 2 <= SH::IN_ELEMS * 2, "output patches fit the tile's LDS");
    if (SH::SMEM > 64 * 1024) {
        static hipError_t raised = hipFuncSetAttribute((const void*)conv_direct_kernel<CK, CN, BWD, POOL>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, SH::SMEM);
        if (raised != hipSuccess) return raised;
    }
    hipLaunchKernelGGL((conv_direct_kernel<CK, CN, BWD, POOL>), dim3(P * a.tiles), dim3(NT), SH::SMEM, st, a);
    return hipGetLastError();
}

bool shape_ok(const ConvCall& c) { return c.P >= 1 && c.B >= 1 && c.W == IMG_W && c.H >= ROWS && c.H % ROWS == 0; }

}  // namespace

bool conv_direct_ok(int H, int W, int c_in, int c_out, bool backward) {
    if (W != IMG_W || H < ROWS || H % ROWS != 0) return false;
    const int k = backward ? c_out : c_in, n = backward ? c_in : c_out;
    if (!(k == 32 || k == 64 || k == 128)) return false;
    return backward ? (n == 32 || n == 64) : (n == 32 || n == 64 || n == 128);
}

hipError_t conv_direct_forward(const ConvCall& c, hipStream_t st) {
    if (!shape_ok(c) || !conv_direct_ok(c.H, c.W, c.c_in, c.c_out, false)) return hipErrorInvalidValue;
    const size_t rows = (size_t)c.B * c.H * c.W;
    DirectArgs a = {};
    a.in = (const uint16_t*)c.in; a.in_lstride = rows * c.c_in; a.c_k = c.c_in;
    a.w = c.ws; a.w_lstride = c.ws_stride;
    a.bhi = c.bhi; a.blo = c.blo; a.b_lstride = c.ws_stride;
    a.out = (uint16_t*)c.out; a.out_lstride = rows * c.c_out;
    a.H = c.H; a.tiles = c.B * (c.H / ROWS);
    if (c.c_in == 32) {
        if (c.c_out == 32) return launch_direct<32, 32, false>(a, c.P, st);
        if (c.c_out == 64) return launch_direct<32, 64, false>(a, c.P, st);
        return launch_direct<32, 128, false>(a, c.P, st);
    }
    if (c.c_out == 32) return launch_direct<64, 32, false>(a, c.P, st);
    if (c.c_out == 64) return launch_direct<64, 64, false>(a, c.P, st);
    return launch_direct<64, 128, false>(a, c.P, st);
}

hipError_t conv_direct_backward_data(const ConvCall& c, const void* dpool, hipStream_t st) {
    if (!shape_ok(c) || !conv_direct_ok(c.H, c.W, c.c_in, c.c_out, true)) return hipErrorInvalidValue;
    const size_t rows = (size_t)c.B * c.H * c.W;
    DirectArgs a = {};
    if (dpool && !c.out) return hipErrorInvalidValue;
    a.in = (const uint16_t*)(dpool ? c.out : c.dz); a.in_lstride = rows * c.c_out; a.c_k = c.c_out;
    a.dpool = (const uint16_t*)dpool; a.dpool_lstride = (size_t)c.B * c.c_out; a.inv = 1.0f / (float)(c.H * c.W);
    a.w = c.ws; a.w_lstride = c.ws_stride;
    a.act = (const uint16_t*)c.in;
    a.out = (uint16_t*)c.dz_in; a.out_lstride = rows * c.c_in;
    a.H = c.H; a.tiles = c.B * (c.H / ROWS);
    if (dpool) {
        if (c.c_out == 32) {
            if (c.c_in == 32) return launch_direct<32, 32, true, true>(a, c.P, st);
            return launch_direct<32, 64, true, true>(a, c.P, st);
        }
        if (c.c_in == 32) return launch_direct<64, 32, true, true>(a, c.P, st);
        return launch_direct<64, 64, true, true>(a, c.P, st);
    }
    if (c.c_out == 32) {
        if (c.c_in == 32) return launch_direct<32, 32, true>(a, c.P, st);
        return launch_direct<32, 64, true>(a, c.P, st);
    }
    if (c.c_in == 32) return launch_direct<64, 32, true>(a, c.P, st);
    return launch_direct<64, 64, true>(a, c.P, st);
}

}  // namespace kavg
