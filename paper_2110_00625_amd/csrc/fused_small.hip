// All K local steps of Algorithm 1 in ONE launch, for fp32 models small enough to live on chip:
// one hidden layer of at most 64 units, at most 16 classes, minibatches of at most 64 rows.
//
// Such a model (d_0 x 64 + 64 x C weights per learner) takes a few microseconds of arithmetic per
// step; run as a chain of generic kernels it is bound by ~6 dependent launches per step.  Here the
// learner's first-layer weights are cut into S column chunks of CW input features (CW a multiple of
// 64, at most 192); workgroup (j, s) keeps chunk s of learner j's W_1 in LDS for the whole call,
// together with private copies of b_1, W_2 and b_2.  (Where the device has the compute units for it and the
// layer has more than 32 units, two workgroups share a chunk, each with half of the hidden units: "its chunk"
// is then those units' rows of the chunk; everything else is unchanged.)  Per step
//   1. the workgroup multiplies its CW columns of the gathered rows X[idx] with its chunk of W_1
//      (fp32 matrix instructions) and writes the B x 64 partial pre-activations to device memory;
//   2. it collects the partials of all S workgroups of its learner and adds them in ascending chunk
//      order (bias, ReLU): every workgroup now holds the same A_1;
//   3. it runs the head -- logits, softmax cross-entropy, dZ_2, dZ_1, the SGD step on its copies of
//      W_2, b_2, b_1 -- redundantly: same inputs, same instruction sequence in every workgroup, so
//      the copies stay bit-identical without further communication;
//   4. and takes the SGD step on its own chunk of W_1 in LDS (dZ_1^T times its columns of X[idx]).
// Only after the K steps do the parameters go back to the replica in device memory.
//
// One exchange per step, without flags that anything depends on: a partial is written as a 64-bit word
// (value, tag) by one device-scope atomic store, the tag being the number of the step counted over all launches of the
// context.  A reader requests the S words of an element with device-scope atomic loads and asks again
// (a bounded number of times, after a device-scope acquire that discards cached copies of the lines)
// until every tag shows the current step; each word validates itself, so nothing depends on the order
// in which different addresses become visible.  (Each wavefront also raises a hint word after its stores, and
// wavefront 0 waits for the learner's hints before anyone gathers -- the other wavefronts finish the previous
// step's W_2, b_1, b_2 and loss meanwhile; the hints only time the first request, the tags decide.)  Partials
// alternate between two buffers: a workgroup overwrites the buffer of step k only when it computes step k+2,
// which it starts after it has read every partial of step k+1, each of which was written after its
// writer had read the partials of step k.  All workgroups must be resident at once: the host
// launches this kernel only when their number does not exceed the number of compute units.  A reader that
// runs out of polls raises an error word and carries on, so every wavefront reaches the end of the
// kernel whatever happens.
//
// The minibatch indices of the learner's K steps are produced here as well (same counter-based
// stream as index_stream_kernel; workgroup 0 of a learner also stores them for kavg_indices), unless
// the caller supplied its own.
#include "kavg_internal.h"

#include <type_traits>

namespace kavg {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int NT = 512;         // threads per workgroup (8 wavefronts)
constexpr int CWMAX = 192;      // input features per workgroup, at most
constexpr int HID = 64;         // hidden units (upper bound)
constexpr int CLS = 16;         // classes (upper bound)
constexpr int ROWS = 64;        // minibatch rows (upper bound)
// Row pitches of the LDS tiles, in words.  A matrix instruction reads a tile either as (16 rows) x (4 consecutive
// words) or as (4 rows) x (16 consecutive words); pitches of 12 or 4 modulo the 64 banks spread the first pattern
// over all banks (the hot one: the operands of the two big products) and the second over most.
constexpr int PW = CWMAX + 12;  // tiles CW wide
constexpr int PH = HID + 4;     // tiles 64 wide
constexpr int PD = CLS + 4;     // dZ_2
constexpr int TILE = ROWS * HID;
constexpr int KBMAX = 1024;     // K*B, at most

struct Smem {
    float W1[HID * PW];         // chunk of W_1: [unit][feature]
    float X[ROWS * PW];         // gathered rows, this chunk's columns: [row][feature]
    float A1[ROWS * PH];        // hidden activations [row][unit]
    float D1[ROWS * PH];        // dZ_1 [row][unit]
    float W2[CLS * PH];         // [class][unit]
    float D2[ROWS * PD];        // dZ_2 [row][class]
    float b1[HID], b2[CLS], rowloss[ROWS];
    int y[ROWS];
    int idx[KBMAX];             // the learner's minibatch indices [K][B]
    int gave_up;                // a wait ran out of polls
};

// a partial and its tag as one 64-bit word
__device__ __forceinline__ void st_tagged(uint64_t* p, float v, uint32_t tag) {
    __hip_atomic_store(p, ((uint64_t)tag << 32) | __builtin_bit_cast(uint32_t, v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_tagged(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t splitmix64_mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// value of lane (l ^ pattern) within rows of 16 lanes, by data-parallel primitives (no LDS round trip)
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
// sum / maximum over each row of 16 lanes, left in all 16 (same operand pairs in every lane: bit-identical)
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_move<0xB1>(x);        // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);        // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);       // row_half_mirror
    x += dpp_move<0x140>(x);       // row_mirror
    return x;
}
__device__ __forceinline__ float row16_max(float x) {
    x = fmaxf(x, dpp_move<0xB1>(x));
    x = fmaxf(x, dpp_move<0x4E>(x));
    x = fmaxf(x, dpp_move<0x141>(x));
    x = fmaxf(x, dpp_move<0x140>(x));
    return x;
}

__global__ void __launch_bounds__(NT)
fused_small_kernel(FusedSmallCall a, int S, int CW, int UH) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Smem& sm = *(Smem*)smem_raw;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // workgroup (j, s, h): learner j, column chunk s, and -- with UH = 2 -- half h of the hidden units (the chunk's
    // two products are then shared by two compute units; everything else is as if UH were 1)
    const int j = blockIdx.x / (S * UH), s = (blockIdx.x / UH) % S, h = blockIdx.x % UH;
    const int UN = HID / UH, ub = h * UN;                       // hidden units ub .. ub+UN-1 are this workgroup's
    const bool first = s == 0 && h == 0;                        // the learner's workgroup that writes what all of them hold
    const int c0 = s * CW;
    const int cw = min(CW, a.d0 - c0);                          // valid columns of this chunk (a multiple of 4)
    const int CW4 = CW / 4;
    float* rep = a.reps + (size_t)j * a.rep_stride;

    // ---- the learner's minibatch indices: draw (j, t0 + k, m) of the counter-based stream, or the caller's ----
    for (int e = tid; e < a.K * a.B; e += NT) {
        int32_t v;
        if (a.generate_idx) {
            const uint64_t c = ((uint64_t)j << 40) | ((uint64_t)(a.t0 + (uint32_t)(e / a.B)) << 16) | (uint32_t)(e % a.B);
            v = (int32_t)(splitmix64_mix(a.seed + (c + 1) * 0x9E3779B97F4A7C15ull) % (uint64_t)a.N);
            if (first) a.idx[(size_t)j * a.K * a.B + e] = v;
        } else {
            v = a.idx[(size_t)j * a.K * a.B + e];
        }
        sm.idx[e] = v;
    }

    // ---- parameters into LDS ----
    for (int e = tid; e < UN * CW4; e += NT) {                  // sm.W1 row r holds unit ub + r
        const int r = e / CW4, c = (e % CW4) * 4;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (ub + r < a.d1 && c < cw) v = *(const f32x4*)(rep + a.w1_off + (size_t)(ub + r) * a.d0 + c0 + c);
        *(f32x4*)(sm.W1 + r * PW + c) = v;
    }
    for (int e = tid; e < CLS * HID; e += NT) {
        const int c = e / HID, u = e % HID;
        sm.W2[c * PH + u] = (c < a.C && u < a.d1) ? rep[a.w2_off + (size_t)c * a.d1 + u] : 0.f;
    }
    if (tid == 0) sm.gave_up = 0;
    if (tid < HID) sm.b1[tid] = tid < a.d1 ? rep[a.b1_off + tid] : 0.f;
    if (tid < CLS) sm.b2[tid] = tid < a.C ? rep[a.b2_off + tid] : 0.f;
    for (int e = tid; e < ROWS * PH; e += NT) { sm.D1[e] = 0.f; sm.A1[e] = 0.f; }   // rows beyond B stay zero throughout
    for (int e = tid; e < ROWS * PD; e += NT) sm.D2[e] = 0.f;
    for (int e = tid; e < ROWS * PW; e += NT) sm.X[e] = 0.f;

    // The thread's 16-byte pieces of a step's X tile: piece i covers row (tid / CW4 + i * (NT / CW4)) ... laid
    // out so that consecutive threads read consecutive 16 bytes of a row.
    const int rows_per_pass = NT / CW4;                         // CW4 in {16, 32, 48}: 32, 16, 10 rows per pass
    const int xr = tid / CW4, xc = (tid % CW4) * 4;
    constexpr int XMAX = 7;                                     // passes: ceil(64 / 10)
    const int xpasses = (a.B + rows_per_pass - 1) / rows_per_pass;
    // the next step's pieces (and label) are requested one step ahead
    int ynext = 0;
    f32x4 xnext[XMAX];
    auto fetch_x = [&](int k) {
        const int* idx = sm.idx + k * a.B;
#pragma unroll
        for (int i = 0; i < XMAX; ++i) {
            const int m = xr + i * rows_per_pass;
            if (i < xpasses && xr < rows_per_pass) {
                const f32x4 x = *(const f32x4*)(a.X + (size_t)idx[min(m, a.B - 1)] * a.d0 + c0 + min(xc, cw - 4));
                xnext[i] = (m < a.B && xc < cw) ? x : (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
        ynext = a.y[idx[min(tid, a.B - 1)]];
    };
    __syncthreads();                                            // sm.idx is complete
    fetch_x(0);

    bool gave_up = false;                                       // a wait ran out of polls: the results are void, finish quickly
    const int Bk = (a.B + 7) & ~7;                              // rows as a contraction length (rows beyond B are zero)
    const int rblocks = (a.B + 15) / 16;                        // 16-row blocks of the minibatch
    const float invB = 1.f / (float)a.B;

    // The small parameters of step kk, from what its head left in LDS: W_2 <- W_2 - lr dZ_2^T A_1 as four 16x16 blocks
    // (wavefronts 1..4), b_1 (5), b_2 (6), the loss (7).  Runs while wavefront 0 waits for the next step's partials.
    auto small_updates = [&](int kk) {
        if (wave >= 1 && wave <= HID / 16) {
            const int u0 = (wave - 1) * 16;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const float* dp = sm.D2 + (lane >> 4) * PD + (lane & 15);           // dZ_2[m][c]: row c of the product
            const float* ap = sm.A1 + (lane >> 4) * PH + u0 + (lane & 15);
            for (int m = 0; m < Bk; m += 8) {
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(dp[m * PD], ap[m * PH], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(dp[(m + 4) * PD], ap[(m + 4) * PH], acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) sm.W2[(4 * (lane >> 4) + v) * PH + u0 + (lane & 15)] -= a.lr * acc[v];
        } else if (wave == 5) {                                 // b_1 <- b_1 - lr colsum(dZ_1)
            float g = 0.f;
#pragma unroll 8
            for (int m = 0; m < Bk; ++m) g += sm.D1[m * PH + lane];
            sm.b1[lane] -= a.lr * g;
        } else if (wave == 6) {                                 // b_2 <- b_2 - lr colsum(dZ_2)
            if (lane < CLS) {
                float g = 0.f;
#pragma unroll 8
                for (int m = 0; m < Bk; ++m) g += sm.D2[m * PD + lane];
                sm.b2[lane] -= a.lr * g;
            }
        } else if (wave == 7 && first && lane == 0) {           // mean loss of this learner's step
            float l = 0.f;
            for (int m = 0; m < a.B; ++m) l += sm.rowloss[m];
            a.losses[(size_t)kk * a.P + j] = l * invB;
        }
    };

    for (int k = 0; k < a.K; ++k) {
        __syncthreads();                                        // previous step is done with sm.X
#pragma unroll
        for (int i = 0; i < XMAX; ++i) {
            const int m = xr + i * rows_per_pass;
            if (i < xpasses && xr < rows_per_pass && m < ROWS) {
                *(f32x4*)(sm.X + m * PW + xc) = xnext[i];
            }
        }
        if (tid < ROWS) sm.y[tid] = tid < a.B ? ynext : 0;
        __syncthreads();
        if (k + 1 < a.K) fetch_x(k + 1);                        // the next step's rows: requested now, used a step later

        // 1. partial pre-activations of this chunk, Zp[m][u] = sum_c X[m][c] W1[u][c], in 16x16 blocks
        //    (matrix instruction 16x16x4: lane l supplies X[m0 + l%16][c + l/16] and W1[u0 + l%16][c + l/16],
        //     and receives Zp[m0 + 4*(l/16) + v][u0 + l%16] in accumulator v)
        const uint32_t tag = a.tag0 + (uint32_t)k + 1u;
        uint64_t* part = a.partial + (((size_t)(k & 1) * a.P + j) * S + s) * TILE;
        for (int blk = wave; blk < rblocks * (UN / 16); blk += NT / 64) {
            const int m0 = (blk / (UN / 16)) * 16, u0 = (blk % (UN / 16)) * 16;        // u0: row of sm.W1, unit ub + u0
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};   // two chains: the matrix pipeline never waits for its own result
            const float* xp = sm.X + (m0 + (lane & 15)) * PW + (lane >> 4);
            const float* wp = sm.W1 + (u0 + (lane & 15)) * PW + (lane >> 4);
#pragma unroll 4
            for (int c = 0; c < CW; c += 8) {
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xp[c], wp[c], acc, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(xp[c + 4], wp[c + 4], acc1, 0, 0, 0);
            }
            acc += acc1;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + 4 * (lane >> 4) + v;
                if (m < a.B) st_tagged(part + m * HID + ub + u0 + (lane & 15), acc[v], tag);
            }
        }

        // This wavefront's partials are on their way: say so in its hint word (a separate address: only a hint --
        // the words of the partials validate themselves).  Then, while wavefront 0 waits for the hints of all
        // wavefronts of the learner's S workgroups, the others finish the previous step's small parameters.
        uint32_t* hints = a.hints + ((size_t)(k & 1) * a.P + j) * S * UH * (NT / 64);
        if (lane == 0) __hip_atomic_store(hints + (s * UH + h) * (NT / 64) + wave, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (wave == 0) {
            unsigned spins = 0;
            for (;;) {
                bool ok = true;
                for (int i = lane; i < S * UH * (NT / 64); i += 64)
                    ok = ok && __hip_atomic_load(hints + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == tag;
                if (__builtin_amdgcn_ballot_w64(!ok) == 0 || gave_up) break;
                if (++spins >= a.spin_limit) { atomicOr(a.err, 1); sm.gave_up = 1; break; }
                __builtin_amdgcn_s_sleep(1);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");       // discard cached copies (see below)
            }
        } else if (k > 0) {
            small_updates(k - 1);
        }
        __syncthreads();
        gave_up = gave_up || sm.gave_up != 0;

        // 2. A_1 = relu(sum of the learner's S partials + b_1).  Element e = tid + i*NT of the B x 64 tile; eight
        //    partials of each of four elements are requested together and asked for again until all carry this
        //    step's tag; they are added in ascending chunk order.
        {
            const uint64_t* base = a.partial + ((size_t)(k & 1) * a.P + j) * S * TILE;
            const int n_el = a.B * HID;
            for (int g0 = 0; g0 * NT < n_el; g0 += 4) {
                float z[4] = {0.f, 0.f, 0.f, 0.f};
                for (int q0 = 0; q0 < S; q0 += 8) {
                    const int nq = min(8, S - q0);
                    uint64_t t[4][8];
                    unsigned spins = 0;
                    for (;;) {
                        bool ok = true;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int u = 0; u < 8; ++u)
                                t[i][u] = ld_tagged(base + (size_t)(q0 + min(u, nq - 1)) * TILE + min(tid + (g0 + i) * NT, n_el - 1));
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int u = 0; u < 8; ++u) ok = ok && (uint32_t)(t[i][u] >> 32) == tag;
                        if (ok || gave_up) break;
                        if (++spins >= a.spin_limit) { atomicOr(a.err, 1); gave_up = true; break; }   // and never wait again
                        __builtin_amdgcn_s_sleep(1);
                        // Without this a reader can be served the same cached copy of a line again and again (seen on
                        // the device: waits that never ended although the words had long been written); the acquire
                        // discards the cached copies, so the next request goes to memory.
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int u = 0; u < 8; ++u) z[i] += u < nq ? __builtin_bit_cast(float, (uint32_t)t[i][u]) : 0.f;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = tid + (g0 + i) * NT;
                    if (e < n_el) sm.A1[(e / HID) * PH + e % HID] = fmaxf(z[i] + sm.b1[e % HID], 0.f);
                }
            }
        }
        __syncthreads();

        // 3. the head, identically in every workgroup of the learner.  Logits in 16-row blocks, one per wavefront:
        //    lane l receives rows m0 + 4*(l/16) + v (v = 0..3) of class l%16, so the 16 classes of a row sit in the
        //    16 lanes of one row of the wavefront and its softmax is a reduction over that row.
        if (wave < rblocks) {
            const int m0 = wave * 16, c = lane & 15;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const float* ap = sm.A1 + (m0 + c) * PH + (lane >> 4);
            const float* wp = sm.W2 + c * PH + (lane >> 4);
#pragma unroll
            for (int u = 0; u < HID; u += 4) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[u], wp[u], acc, 0, 0, 0);
            const bool live = c < a.C;
            const float bias = sm.b2[c];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + 4 * (lane >> 4) + v;
                const float z = acc[v] + bias;
                const float mx = row16_max(live ? z : -INFINITY);
                const float ex = live ? expf(z - mx) : 0.f;
                const float den = row16_sum(ex);
                const int yy = sm.y[m];
                if (m < a.B) {
                    sm.D2[m * PD + c] = live ? (ex / den - (c == yy ? 1.f : 0.f)) * invB : 0.f;   // dZ_2 = (p - onehot) / B
                    if (c == yy) sm.rowloss[m] = logf(den) + mx - z;
                }
            }
        }
        __syncthreads();
        for (int blk = wave; blk < rblocks * (HID / 16); blk += NT / 64) {      // dZ_1 = (dZ_2 W_2) masked by the ReLU
            const int m0 = (blk / (HID / 16)) * 16, u0 = (blk % (HID / 16)) * 16;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const float* dp = sm.D2 + (m0 + (lane & 15)) * PD + (lane >> 4);
            const float* wp = sm.W2 + (lane >> 4) * PH + u0 + (lane & 15);
#pragma unroll
            for (int c = 0; c < CLS; c += 4) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(dp[c], wp[c * PH], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int at = (m0 + 4 * (lane >> 4) + v) * PH + u0 + (lane & 15);
                sm.D1[at] = sm.A1[at] > 0.f ? acc[v] : 0.f;      // rows beyond B: A_1 is zero there
            }
        }
        __syncthreads();

        // 4. W_1[u][c] <- W_1[u][c] - lr sum_m dZ_1[m][u] X[m][c] on this workgroup's units and columns.  A wavefront
        //    owns one 16-unit block and every G-th 16-column block (G = wavefronts per unit block): one dZ_1 operand
        //    feeds all its blocks.
        {
            const int nub = UN / 16, G = (NT / 64) / nub;       // 4 unit blocks x 2 column groups, or 2 x 4
            const int u0 = (wave % nub) * 16, cb0 = (wave / nub) * 16;
            const float* dp = sm.D1 + (lane >> 4) * PH + ub + u0 + (lane & 15);
            const float* xp = sm.X + (lane >> 4) * PW + cb0 + (lane & 15);
            const int cstep = 16 * G;
            auto update_w1 = [&](auto nb_tag) {
                constexpr int NB = decltype(nb_tag)::value;
                f32x4 acc[NB];
#pragma unroll
                for (int i = 0; i < NB; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
                for (int m = 0; m < Bk; m += 4) {
                    const float d = dp[m * PH];
#pragma unroll
                    for (int i = 0; i < NB; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(d, xp[m * PW + cstep * i], acc[i], 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < NB; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        sm.W1[(u0 + 4 * (lane >> 4) + v) * PW + cb0 + cstep * i + (lane & 15)] -= a.lr * acc[i][v];
            };
            switch ((CW / 16) / G) {                            // column blocks per wavefront
                case 1: update_w1(std::integral_constant<int, 1>{}); break;
                case 2: update_w1(std::integral_constant<int, 2>{}); break;
                case 3: update_w1(std::integral_constant<int, 3>{}); break;
                case 4: update_w1(std::integral_constant<int, 4>{}); break;
                default: update_w1(std::integral_constant<int, 6>{}); break;
            }
        }
    }
    __syncthreads();
    small_updates(a.K - 1);
    __syncthreads();

    // ---- parameters back to the replica ----
    for (int e = tid; e < UN * CW4; e += NT) {
        const int r = e / CW4, c = (e % CW4) * 4;
        if (ub + r < a.d1 && c < cw) {
            *(f32x4*)(rep + a.w1_off + (size_t)(ub + r) * a.d0 + c0 + c) = *(const f32x4*)(sm.W1 + r * PW + c);
        }
    }
    if (first) {
        for (int e = tid; e < a.C * a.d1; e += NT) rep[a.w2_off + e] = sm.W2[(e / a.d1) * PH + e % a.d1];
        if (tid < a.d1) rep[a.b1_off + tid] = sm.b1[tid];
        if (tid < a.C) rep[a.b2_off + tid] = sm.b2[tid];
    }
}

}  // namespace

// Columns per workgroup: the fewest multiples of 64 (at most 192) that leave at most 16 chunks, else 192.
int fused_small_chunk_width(int d0) {
    for (int cw = 64; cw < CWMAX; cw += 64)
        if ((d0 + cw - 1) / cw <= 16) return cw;
    return CWMAX;
}
int fused_small_chunks(int d0) { const int cw = fused_small_chunk_width(d0); return (d0 + cw - 1) / cw; }

bool fused_small_shape_ok(int P, int K, int B, int d0, int d1, int C, int compute_units) {
    if (d1 < 1 || d1 > HID || C < 1 || C > CLS || B < 1 || B > ROWS || d0 < 4 || d0 % 4 != 0) return false;
    if ((long)K * B > KBMAX) return false;
    return (long)P * fused_small_chunks(d0) <= compute_units;
}

// Workgroups per column chunk: two (each with half of the hidden units) when the layer is wider than 32 units and
// the device has the compute units for it.
int fused_small_unit_split(int P, int d0, int d1, int compute_units) {
    return d1 > HID / 2 && (long)2 * P * fused_small_chunks(d0) <= compute_units ? 2 : 1;
}

// two buffers of P x chunks tiles of (value, tag) words, then two of P x chunks x wavefronts hint words
size_t fused_small_partial_words(int P, int d0) { return (size_t)2 * P * fused_small_chunks(d0) * TILE; }
size_t fused_small_scratch_bytes(int P, int d0) {          // (hint words for a unit split of two)
    return fused_small_partial_words(P, d0) * 8 + (size_t)2 * P * fused_small_chunks(d0) * 2 * (NT / 64) * 4;
}

hipError_t launch_fused_small(const FusedSmallCall& c, hipStream_t st) {
    const int S = fused_small_chunks(c.d0), CW = fused_small_chunk_width(c.d0);
    const int UH = fused_small_unit_split(c.P, c.d0, c.d1, c.compute_units);
    static hipError_t raised = hipFuncSetAttribute((const void*)fused_small_kernel,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem));
    if (raised != hipSuccess) return raised;
    hipLaunchKernelGGL(fused_small_kernel, dim3(c.P * S * UH), dim3(NT), sizeof(Smem), st, c, S, CW, UH);
    return hipGetLastError();
}

}  // namespace kavg
