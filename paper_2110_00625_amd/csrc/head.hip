// Classifier head for small class counts (C <= 16), both precisions.
//
// With ten classes the last layer is a sliver: its forward product, the
// softmax cross-entropy, its data gradient and its weight update together
// move a few hundred KB per learner, and as four generic launches they cost
// four launch-plus-pipeline latencies.  Two kernels replace them:
//
//  head_forward_backward   one wavefront per sample row:
//        z = A_{L-1}[s] W_L^T + b_L                     (lanes split the contraction, butterfly sum)
//        loss_s = -log softmax(z)[y_s],  dZ_L[s] = (softmax(z) - onehot(y_s)) / B   (the 1/B_n of Algorithm 1)
//        dZ_{L-1}[s] = (dZ_L[s] W_L) * [A_{L-1}[s] > 0]
//  head_update             W_L <- W_L - lr * dZ_L^T A_{L-1},  b_L <- b_L - lr * colsum(dZ_L)
//        (the learner update of Algorithm 1 for the last layer; runs after the kernel above
//        because that one reads the weights of before the step)
//
// Mixed precision follows the same rounding points as the generic kernels:
// products of bf16 operands accumulated in fp32, dZ_L and dZ_{L-1} rounded to
// bf16 (round to nearest even) before any use, logits / softmax / loss / bias
// / master update in fp32; the master is read and written as its two 16-bit
// planes (split.h), of which the bf16 one is the operand of the products.
#include "kavg_internal.h"
#include "split.h"

namespace kavg {

namespace {

constexpr int CMAX = 16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Data-parallel-primitive moves inside a row of 16 lanes: no LDS round trip, unlike a general shuffle.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
// Sum over the 64 lanes, the same value in every lane.  Inside a row: neighbours, pairs, mirrored halves,
// mirrored row (every lane then holds its row's sum); across the four rows: their last lanes are read
// as scalars and added in a fixed order.
__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_move<0xB1>(x);        // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);        // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);       // row_half_mirror
    x += dpp_move<0x140>(x);       // row_mirror
    const int xi = __builtin_bit_cast(int, x);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 15));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 31));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 47));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 63));
    return (r0 + r1) + (r2 + r3);
}
// Sum over the 16 lanes that differ in bits 2..5 of the lane index (same low two bits), in every lane:
// rotations by 4 and 8 inside a row keep the low bits; the rows are joined by two shuffles.
__device__ __forceinline__ float groups_sum(float x) {
    x += dpp_move<0x124>(x);       // row_ror:4
    x += dpp_move<0x128>(x);       // row_ror:8
    x += __shfl_xor(x, 16, 64);
    x += __shfl_xor(x, 32, 64);
    return x;
}
__device__ __forceinline__ uint16_t bf16_bits(float x) {
    __bf16 h = (__bf16)x;                         // round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float bf16_round(float x) {
    return __builtin_bit_cast(float, (uint32_t)bf16_bits(x) << 16);
}

// A "piece" is what one lane loads at once: 8 bf16 or 1 float.  It is kept as loaded (r) and unpacked
// into floats (v) only where it is used, so that pieces can stay in registers cheaply.
template <bool BF16> struct Piece;
template <> struct Piece<true> {
    static constexpr int N = 8;
    u32x4 r;
    float v[8];
    __device__ __forceinline__ void fetch(const void* base, size_t elem) { r = *(const u32x4*)((const uint16_t*)base + elem); }
    __device__ __forceinline__ void clear() { r = (u32x4){0u, 0u, 0u, 0u}; }
    __device__ __forceinline__ void unpack() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __builtin_bit_cast(float, r[i] << 16);
            v[2 * i + 1] = __builtin_bit_cast(float, r[i] & 0xFFFF0000u);
        }
    }
    __device__ __forceinline__ void load(const void* base, size_t elem) { fetch(base, elem); unpack(); }
};
template <> struct Piece<false> {
    static constexpr int N = 1;
    float r;
    float v[1];
    __device__ __forceinline__ void fetch(const void* base, size_t elem) { r = ((const float*)base)[elem]; }
    __device__ __forceinline__ void clear() { r = 0.f; }
    __device__ __forceinline__ void unpack() { v[0] = r; }
    __device__ __forceinline__ void load(const void* base, size_t elem) { fetch(base, elem); unpack(); }
};

struct HeadArgs {
    const void* act; int ld_act; size_t act_lstride;      // A_{L-1} [P][B][ld_act], or the data set when gather != null
    const int32_t* gather; long gather_lstride;           // row s of learner j is data row gather[j*gather_lstride + s]
    const void* wmul; size_t wmul_lstride;                // weights as multiplied: bf16 (hi) plane or fp32, [C][d]
    float* wmaster; size_t w_lstride;                     // fp32 mode: the layer's weights
    float* bias;                                          // fp32 mode: its bias (stride w_lstride)
    uint16_t* whi; uint16_t* wlo; size_t ws_lstride;      // bf16 mode: hi / lo planes of the weights (split.h)
    uint16_t* bhi; uint16_t* blo;                         // bf16 mode: hi / lo planes of the bias (stride ws_lstride)
    const int32_t* y;                                     // labels of the data set
    void* dz; int ldz; size_t dz_lstride;                 // dZ_L [P][B][ldz]
    void* dz_prev; size_t dz_prev_lstride;                // dZ_{L-1} [P][B][d], null for a single-layer model
    float* rowloss;                                       // [P][B]
    int P, B, d, C;
    float lr;
    float* u; float* ub; float beta;                      // velocities of W_L / b_L (stride w_lstride), null: plain SGD
};

// CT = compile-time bound on the class count (4, 8, 12 or 16): every loop over classes is fully
// unrolled and its loads are issued unconditionally (rows beyond C re-read row C-1 and are ignored),
// so that a lane's loads of a step go out together instead of one round trip per class.
// KEEP: the row has at most 128 pieces (two per lane); they are fetched once and stay in registers for
// the second pass (the data gradient) instead of being fetched again.
template <bool BF16, int CT, bool KEEP>
__global__ void __launch_bounds__(256) head_forward_backward_kernel(HeadArgs a) {
    constexpr int N = Piece<BF16>::N;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);      // one wavefront per sample row
    const int learner = blockIdx.y;
    if (row >= a.B) return;                                   // whole wavefront leaves together
    const int32_t* g = a.gather + (long)learner * a.gather_lstride;
    const int sample = g[row];                                // data row of this sample (labels; inputs when L = 1)
    const size_t arow = a.act_lstride ? (size_t)learner * a.act_lstride + (size_t)row * a.ld_act
                                      : (size_t)sample * a.ld_act;
    const void* W = BF16 ? (const void*)((const uint16_t*)a.wmul + (size_t)learner * a.wmul_lstride)
                         : (const void*)((const float*)a.wmul + (size_t)learner * a.wmul_lstride);
    const int pieces = a.d / N;
    const int label_raw = a.y[sample];
    float bias_c[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const int cc = c < a.C ? c : a.C - 1;
        if (BF16) {
            const size_t at = (size_t)learner * a.ws_lstride + cc;
            bias_c[c] = __builtin_bit_cast(float, split_join(a.bhi[at], a.blo[at]));
        } else {
            bias_c[c] = a.bias[(size_t)learner * a.w_lstride + cc];
        }
    }
    size_t wrow[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) wrow[c] = (size_t)(c < a.C ? c : a.C - 1) * a.d;

    float acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[c] = 0.f;
    Piece<BF16> xs[KEEP ? 2 : 1], ws[CT][KEEP ? 2 : 1];
    if constexpr (KEEP) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int q = lane + 64 * it;
            const size_t qq = (size_t)(q < pieces ? q : pieces - 1) * N;      // clamped: no predicated loads
            xs[it].fetch(a.act, arow + qq);
#pragma unroll
            for (int c = 0; c < CT; ++c) ws[c][it].fetch(W, wrow[c] + qq);
        }
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            if (lane + 64 * it >= pieces) xs[it].clear();                      // contributes nothing to either pass
            xs[it].unpack();
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                ws[c][it].unpack();
#pragma unroll
                for (int e = 0; e < N; ++e) acc[c] = fmaf(xs[it].v[e], ws[c][it].v[e], acc[c]);
            }
        }
    } else {
        for (int q = lane; q < pieces; q += 64) {
            Piece<BF16> x, w[CT];
            x.load(a.act, arow + (size_t)q * N);
#pragma unroll
            for (int c = 0; c < CT; ++c) w[c].load(W, wrow[c] + (size_t)q * N);
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int e = 0; e < N; ++e) acc[c] = fmaf(x.v[e], w[c].v[e], acc[c]);
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        acc[c] = wave_sum(acc[c]) + bias_c[c];
        if (c < a.C) mx = fmaxf(mx, acc[c]);
    }
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < CT; ++c) if (c < a.C) sum += expf(acc[c] - mx);
    const int label = label_raw < 0 ? 0 : (label_raw >= a.C ? a.C - 1 : label_raw);   // validated; never index outside
    const float invB = 1.0f / (float)a.B;
    float gz[CT];
    float zy = 0.f;
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        gz[c] = 0.f;
        if (c < a.C) {
            const float p = expf(acc[c] - mx) / sum;
            gz[c] = (p - (c == label ? 1.0f : 0.0f)) * invB;
            if (BF16) gz[c] = bf16_round(gz[c]);
            if (c == label) zy = acc[c];
        }
    }
    if (lane == 0) a.rowloss[(size_t)learner * a.B + row] = -(zy - mx - logf(sum));
    if (lane < a.ldz) {                                       // dZ_L row, pad columns zero
        float mine = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) if (c == lane) mine = gz[c];
        const size_t at = (size_t)learner * a.dz_lstride + (size_t)row * a.ldz + lane;
        if (BF16) ((uint16_t*)a.dz)[at] = bf16_bits(mine); else ((float*)a.dz)[at] = mine;
    }
    if (!a.dz_prev) return;

    // dZ_{L-1}[s][k] = (sum_c dZ_L[s][c] W_L[c][k]) * [A_{L-1}[s][k] > 0]      (gz[c] = 0 beyond C)
    auto data_gradient = [&](int q, Piece<BF16>& x, Piece<BF16> (&w)[CT]) {
        float da[N];
#pragma unroll
        for (int e = 0; e < N; ++e) da[e] = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int e = 0; e < N; ++e) da[e] = fmaf(gz[c], w[c].v[e], da[e]);
#pragma unroll
        for (int e = 0; e < N; ++e) da[e] = x.v[e] > 0.f ? da[e] : 0.f;
        const size_t at = (size_t)learner * a.dz_prev_lstride + (size_t)row * a.d + (size_t)q * N;
        if (BF16) {
            u32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (uint32_t)bf16_bits(da[(2 * i) % N]) | ((uint32_t)bf16_bits(da[(2 * i + 1) % N]) << 16);
            *(u32x4*)((uint16_t*)a.dz_prev + at) = o;
        } else {
            ((float*)a.dz_prev)[at] = da[0];
        }
    };
    if constexpr (KEEP) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int q = lane + 64 * it;
            if (q < pieces) {
                Piece<BF16> w[CT];
#pragma unroll
                for (int c = 0; c < CT; ++c) { w[c] = ws[c][it]; w[c].unpack(); }
                xs[it].unpack();
                data_gradient(q, xs[it], w);
            }
        }
    } else {
        for (int q = lane; q < pieces; q += 64) {
            Piece<BF16> x, w[CT];
            x.load(a.act, arow + (size_t)q * N);
#pragma unroll
            for (int c = 0; c < CT; ++c) w[c].load(W, wrow[c] + (size_t)q * N);
            data_gradient(q, x, w);
        }
    }
}

// One row of dZ_L (ldz <= 16 values) as floats; entries beyond ldz are zero.
template <bool BF16>
__device__ __forceinline__ void load_dz_row(const void* dz, size_t at, int ldz, float* out /*[16]*/) {
#pragma unroll
    for (int i = 0; i < 16; ++i) out[i] = 0.f;
    if (BF16) {
        const u32x4 lo = *(const u32x4*)((const uint16_t*)dz + at);
        u32x4 hi = {0u, 0u, 0u, 0u};
        if (ldz > 8) hi = *(const u32x4*)((const uint16_t*)dz + at + 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __builtin_bit_cast(float, lo[i] << 16);
            out[2 * i + 1] = __builtin_bit_cast(float, lo[i] & 0xFFFF0000u);
            out[8 + 2 * i] = __builtin_bit_cast(float, hi[i] << 16);
            out[8 + 2 * i + 1] = __builtin_bit_cast(float, hi[i] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (4 * i < ldz) {                                // ldz is a multiple of 8
                const f32x4 v = *(const f32x4*)((const float*)dz + at + 4 * i);
                out[4 * i] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
            }
        }
    }
}

// 256 threads = 4 wavefronts.  Lane = 4*g + pl: sample group g (samples s = g mod 16) and piece
// blockIdx.x*16 + 4*wave + pl of the layer's input units.  Every lane sums dZ_L[s][c] * A[s][piece]
// over its samples in ascending order; a butterfly over the group bits of the lane index adds the
// sixteen groups, after which lane group g applies the update of class c = g.
constexpr int XCH_CS = 16 * 32 + 36;      // floats between classes in a wavefront's exchange patch (36: classes fall on different banks)

template <bool BF16, int CT>
__global__ void __launch_bounds__(256) head_update_kernel(HeadArgs a) {
    constexpr int N = Piece<BF16>::N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = lane >> 2, pl = lane & 3;
    const int q = blockIdx.x * 16 + wave * 4 + pl;
    const int learner = blockIdx.y;
    const int pieces = a.d / N;
    const bool live = q < pieces;
    const int qq = live ? q : pieces - 1;                     // out-of-range lanes shadow the last piece, never store
    const int32_t* g = a.gather + (long)learner * a.gather_lstride;

    float acc[CT][N], bsum[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        bsum[c] = 0.f;
#pragma unroll
        for (int e = 0; e < N; ++e) acc[c][e] = 0.f;
    }
#pragma unroll 4
    for (int s = grp; s < a.B; s += 16) {
        const size_t arow = a.act_lstride ? (size_t)learner * a.act_lstride + (size_t)s * a.ld_act
                                          : (size_t)g[s] * a.ld_act;
        Piece<BF16> x;
        x.load(a.act, arow + (size_t)qq * N);
        float gz[16];
        load_dz_row<BF16>(a.dz, (size_t)learner * a.dz_lstride + (size_t)s * a.ldz, a.ldz, gz);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            bsum[c] += gz[c];                                  // bias gradient: column sum of dZ_L
#pragma unroll
            for (int e = 0; e < N; ++e) acc[c][e] = fmaf(gz[c], x.v[e], acc[c][e]);
        }
    }
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        float b = bsum[c];
        bsum[c] = groups_sum(b);
    }
    float mine[N];
    if constexpr (BF16) {
        // Lane group g needs class g's gradient of the wavefront's four pieces, summed over the sixteen sample
        // groups: each lane leaves its CT x 8 partial sums in the wavefront's LDS patch and lane group g adds
        // the sixteen partials of class g in ascending group order (a butterfly would move every value four
        // times, this moves it twice).  A wavefront's LDS accesses complete in order: no barrier.
        extern __shared__ __align__(16) float head_xch[];
        float* patch = head_xch + wave * (CT * XCH_CS);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            *(f32x4*)(patch + c * XCH_CS + lane * 8) = (f32x4){acc[c][0], acc[c][1], acc[c][2], acc[c][3]};
            *(f32x4*)(patch + c * XCH_CS + lane * 8 + 4) = (f32x4){acc[c][4], acc[c][5], acc[c][6], acc[c][7]};
        }
#pragma unroll
        for (int e = 0; e < N; ++e) mine[e] = 0.f;
        const float* src = patch + min(grp, CT - 1) * XCH_CS + pl * 8;
#pragma unroll
        for (int g2 = 0; g2 < 16; ++g2) {
            const f32x4 lo4 = *(const f32x4*)(src + g2 * 32), hi4 = *(const f32x4*)(src + g2 * 32 + 4);
            mine[0] += lo4.x; mine[1 % N] += lo4.y; mine[2 % N] += lo4.z; mine[3 % N] += lo4.w;
            mine[4 % N] += hi4.x; mine[5 % N] += hi4.y; mine[6 % N] += hi4.z; mine[7 % N] += hi4.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int e = 0; e < N; ++e) {
                float v = acc[c][e];
                acc[c][e] = groups_sum(v);
            }
#pragma unroll
        for (int e = 0; e < N; ++e) mine[e] = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c)
            if (c == grp) {
#pragma unroll
                for (int e = 0; e < N; ++e) mine[e] = acc[c][e];
            }
    }
    if (live && grp < a.C) {
        const size_t uat = (size_t)learner * a.w_lstride + (size_t)grp * a.d + (size_t)q * N;   // velocity (fp32 layout)
        if (a.u) {                                            // heavy ball inside the learner
#pragma unroll
            for (int e = 0; e < N; ++e) { mine[e] = a.beta * a.u[uat + e] + mine[e]; a.u[uat + e] = mine[e]; }
        }
        if (BF16) {
            // the master lives in two 16-bit planes; the hi plane is what the next products read
            const size_t at = (size_t)learner * a.ws_lstride + (size_t)grp * a.d + (size_t)q * N;
            const u32x4 h = *(const u32x4*)(a.whi + at), l = *(const u32x4*)(a.wlo + at);
            u32x4 oh, ol;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t b0, b1;
                split_join2(h[i], l[i], b0, b1);
                const float w0 = __builtin_bit_cast(float, b0) - a.lr * mine[(2 * i) % N];
                const float w1 = __builtin_bit_cast(float, b1) - a.lr * mine[(2 * i + 1) % N];
                uint32_t h2, l2;
                split_pack2(__builtin_bit_cast(uint32_t, w0), __builtin_bit_cast(uint32_t, w1), h2, l2);
                oh[i] = h2; ol[i] = l2;
            }
            *(u32x4*)(a.whi + at) = oh;
            *(u32x4*)(a.wlo + at) = ol;
        } else {
            float* wm = a.wmaster + uat;
#pragma unroll
            for (int e = 0; e < N; ++e) wm[e] = wm[e] - a.lr * mine[e];
        }
    }
    if (blockIdx.x == 0 && wave == 0 && pl == 0 && grp < a.C) {   // every lane holds the full column sums
        float mine = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) if (c == grp) mine = bsum[c];
        const size_t at = (size_t)learner * a.w_lstride + grp;
        if (a.ub) { mine = a.beta * a.ub[at] + mine; a.ub[at] = mine; }
        if (BF16) {
            const size_t sat = (size_t)learner * a.ws_lstride + grp;
            const float b = __builtin_bit_cast(float, split_join(a.bhi[sat], a.blo[sat])) - a.lr * mine;
            a.bhi[sat] = (uint16_t)split_hi(__builtin_bit_cast(uint32_t, b));
            a.blo[sat] = (uint16_t)split_lo(__builtin_bit_cast(uint32_t, b));
        } else {
            a.bias[at] = a.bias[at] - a.lr * mine;
        }
    }
}

HeadArgs make_args(const LayerCall& c, const int32_t* y, const int32_t* idx, long idx_lstride, float* rowloss, bool bf16) {
    HeadArgs a = {};
    a.act = c.in; a.ld_act = c.ld_in; a.act_lstride = c.gather ? 0 : c.in_stride;
    a.gather = idx; a.gather_lstride = idx_lstride;
    a.wmul = bf16 ? (const void*)c.ws : (const void*)c.w;
    a.wmul_lstride = bf16 ? c.ws_stride : c.w_stride;
    a.wmaster = c.w; a.w_lstride = c.w_stride; a.bias = c.b;
    a.whi = c.ws; a.wlo = c.wlo; a.ws_lstride = c.ws_stride; a.bhi = c.bhi; a.blo = c.blo;
    a.y = y;
    a.dz = (void*)c.dz; a.ldz = c.ld_dz; a.dz_lstride = c.dz_stride;
    a.dz_prev = c.dz_prev; a.dz_prev_lstride = c.dz_prev_stride;
    a.rowloss = rowloss;
    a.P = c.P; a.B = c.B; a.d = c.d_in; a.C = c.d_out; a.lr = c.lr;
    a.u = c.u; a.ub = c.ub; a.beta = c.beta;
    return a;
}

}  // namespace

bool head_supported(int C) { return C <= CMAX; }

namespace {
template <bool BF16, bool KEEP>
void launch_fb2(const HeadArgs& a, dim3 grid, hipStream_t st) {
    if (a.C <= 4) hipLaunchKernelGGL((head_forward_backward_kernel<BF16, 4, KEEP>), grid, dim3(256), 0, st, a);
    else if (a.C <= 8) hipLaunchKernelGGL((head_forward_backward_kernel<BF16, 8, KEEP>), grid, dim3(256), 0, st, a);
    else if (a.C <= 12) hipLaunchKernelGGL((head_forward_backward_kernel<BF16, 12, KEEP>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((head_forward_backward_kernel<BF16, 16, KEEP && !BF16>), grid, dim3(256), 0, st, a);   // bf16 x 16 classes: too many registers to keep
}
template <bool BF16>
void launch_fb(const HeadArgs& a, dim3 grid, hipStream_t st) {
    const int pieces = a.d / Piece<BF16>::N;
    if (pieces <= 128) launch_fb2<BF16, true>(a, grid, st); else launch_fb2<BF16, false>(a, grid, st);
}
template <bool BF16, int CT>
hipError_t launch_upd_ct(const HeadArgs& a, dim3 grid, hipStream_t st) {
    constexpr int SMEM = BF16 ? 4 * CT * XCH_CS * 4 : 0;       // one exchange patch per wavefront
    if (SMEM > 64 * 1024) {
        static hipError_t raised = hipFuncSetAttribute((const void*)head_update_kernel<BF16, CT>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        if (raised != hipSuccess) return raised;
    }
    hipLaunchKernelGGL((head_update_kernel<BF16, CT>), grid, dim3(256), SMEM, st, a);
    return hipSuccess;
}
template <bool BF16>
hipError_t launch_upd(const HeadArgs& a, dim3 grid, hipStream_t st) {
    if (a.C <= 4) return launch_upd_ct<BF16, 4>(a, grid, st);
    if (a.C <= 8) return launch_upd_ct<BF16, 8>(a, grid, st);
    if (a.C <= 12) return launch_upd_ct<BF16, 12>(a, grid, st);
    return launch_upd_ct<BF16, 16>(a, grid, st);
}

}  // namespace

hipError_t head_forward_backward(const LayerCall& c, const int32_t* y, const int32_t* idx, long idx_lstride,
                                 float* rowloss, int bf16, hipStream_t st) {
    HeadArgs a = make_args(c, y, idx, idx_lstride, rowloss, bf16 != 0);
    dim3 grid((c.B + 3) / 4, c.P);
    if (bf16) launch_fb<true>(a, grid, st); else launch_fb<false>(a, grid, st);
    return hipGetLastError();
}

hipError_t head_update(const LayerCall& c, const int32_t* idx, long idx_lstride, int bf16, hipStream_t st) {
    HeadArgs a = make_args(c, nullptr, idx, idx_lstride, nullptr, bf16 != 0);
    const int pieces = c.d_in / (bf16 ? 8 : 1);
    dim3 grid((pieces + 15) / 16, c.P);
    const hipError_t e = bf16 ? launch_upd<true>(a, grid, st) : launch_upd<false>(a, grid, st);
    return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace kavg
