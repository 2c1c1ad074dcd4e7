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
//                  W_l <- W_l - lr * dZ_l^T A_{l-1}  on the fp32 master (stored as two 16-bit
//                  planes, split.h: the bf16 plane is what the other two products read),
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
// to LDS as [x][k] in 16-byte pieces and read back as 16-byte MFMA fragments.
// An operand whose contraction index is the row index in memory ("transposed":
// W in backward-data, dZ and A in the update, whose contraction runs over the
// samples) is copied to LDS unchanged as [k][x], again in 16-byte pieces, and
// its MFMA fragments are produced by the LDS transpose read
// (ds_read_b64_tr_b16): inside a 16-lane group the lanes fetch a 4(k) x 16(x)
// block, four consecutive x per lane, and each lane receives the four k of
// one x.  Both LDS layouts are padded so that fragment reads and tile writes
// spread over all banks.  The forward pass (both operands direct) skips the
// registers: its slices go from global memory straight into LDS
// (global_load_lds_dwordx4), unpadded, with the 16-byte chunks of a row permuted
// instead (DmaLoader).
//
// Rows beyond an extent are zero-filled on load and masked on store; every
// memory-contiguous extent is a multiple of 8 elements (hidden widths are
// required to be, the class count is padded in the logits / dZ_L buffers).
#include "kavg_internal.h"
#include "fastdiv.h"
#include "split.h"

namespace kavg {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

enum { MODE_FWD = 0, MODE_BWD = 1, MODE_UPD = 2 };
// Main-loop pipelines.  PLAIN: one LDS buffer, the next slice waits in registers.  LDS2: two LDS
// buffers, the next slice is written while the current one is read.  DMA: two LDS buffers filled by
// direct global->LDS loads (no registers, no LDS store instructions); k-contiguous operands only.
// RING: a ring of LDS buffers filled, slices ahead, by two extra wavefronts that do nothing else
// (the wavefronts that multiply never issue a memory load, so none of them stands in the queue of the
// memory pipeline while its MFMAs could run); whole slices only.
enum { PIPE_PLAIN = 0, PIPE_LDS2 = 1, PIPE_DMA = 2, PIPE_RING = 3 };
constexpr int RING_LOADERS = 2, RING_BYTES = 144 * 1024;

struct Operand {
    const uint16_t* base;    // learner 0
    size_t lstride;          // elements between learners (0: shared by all learners)
    int ld;                  // elements between consecutive memory rows
    const int32_t* gather;   // optional: memory row = gather[row]
    long gstride;            // per learner
    int n_rows;              // valid memory rows (exact)
    int n_cont;              // readable contiguous extent (multiple of 8)
    // Implicit patch matrix of a 3x3 convolution (cv_c > 0): `base` is then a channels-last image stack
    // [n][H][W][cv_c] per learner, memory row x is the position (n, h, w) and the contiguous index is
    // k = tap * cv_c + channel, tap = 3*kh + kw reading pixel (h + sign*(kh-1), w + sign*(kw-1)), zero outside
    // the image.  n_rows = positions, n_cont = 9 * cv_c.  div_* are multiply-shift divisors (FastDiv).
    int cv_c, cv_H, cv_W, cv_sign;
    uint32_t div_c_m, div_w_m, div_hw_m; int div_c_s, div_w_s, div_hw_s;
};

inline void operand_conv(Operand& o, int c, int H, int W, int sign) {
    o.cv_c = c; o.cv_H = H; o.cv_W = W; o.cv_sign = sign;
    fastdiv_make((uint32_t)c, &o.div_c_m, &o.div_c_s);
    fastdiv_make((uint32_t)W, &o.div_w_m, &o.div_w_s);
    fastdiv_make((uint32_t)(H * W), &o.div_hw_m, &o.div_hw_s);
}

struct Args {
    Operand R, C;
    int nR, nC, nK;
    int tiles_r, tiles_c, total_wg, chunk;       // workgroup -> tile map (set by launch)
    // forward: bias as hi / lo planes (split.h)
    const uint16_t* bias_hi; const uint16_t* bias_lo; size_t bias_lstride;
    void* out; size_t out_lstride; int ld_out;   // bf16 activations or fp32 logits
    int relu;                                    // 1: hidden layer (bf16 out), 0: last layer (fp32 out)
    // backward-data
    const uint16_t* act_prev; size_t act_lstride; int ld_act;
    // update: the fp32 master as two 16-bit planes (split.h): ws = hi (the bf16 operands of the other
    // products), wlo = lo; bias planes likewise; all with ws_lstride between learners
    uint16_t* ws; uint16_t* wlo; size_t ws_lstride; uint16_t* bhi; uint16_t* blo;
    size_t w_lstride;                            // between learners in the velocity arrays
    float lr;
    float* u; float* ub; float beta;             // velocities of weights / bias (stride w_lstride), null: plain SGD
    const int32_t* next_gather;                  // rows of C's data set that the next step gathers (stride C.gstride), or null
    // Variants of the epilogues used when weight updates are deferred (see kavg_internal.h, DeferredCall):
    //   forward mode:  EPI_GRAM   out = bf16(alpha * acc), no bias, no ReLU
    //   backward mode: EPI_RAW    out = fp32 acc (no mask)
    //                  EPI_RELU   out = bf16(relu(base + acc));  EPI_LOGITS  out = fp32 (base + acc)
    //                  EPI_STD with base != null: out = bf16(mask(base + acc))
    //   update mode:   skip_bias  leave the bias alone (it has been stepped already)
    int epi; float alpha;
    const float* base; size_t base_lstride; int ld_base;
    int skip_bias;
    //                  partial != null: store the fp32 accumulators (and column sums of R) instead of stepping
    //                  the master; "learners" are then ranges of rows of the real learners
    float* partial; float* partial_bias;
    int cv_splits;                               // implicit C operand with partial outputs: ranges per real learner
    int c_stream;                                // forward: the C operand (weights) is read once and does not stay in the memory-side cache
                                                 // (measured: noisy_wide forward 5.9 -> 5.5 ms per round; no gain on the transposed reads of backward-data)
};
enum { EPI_STD = 0, EPI_GRAM = 1, EPI_RAW = 2, EPI_RELU = 3, EPI_LOGITS = 4 };

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
// A slice is BK along the contraction.  Every thread of the NT-thread workgroup moves
// X*BK/8/NT pieces of 16 bytes per operand and slice.
template <int N> struct StageRegs { u32x4 v[N]; };

constexpr int dpitch(int BK) { return BK + 8; }    // [x][k] tile: row of BK bf16 plus 16 bytes
constexpr int tpitch(int X) { return X + 32; }     // [k][x] tile: row of X bf16 plus 64 bytes

// Direct operand: piece e covers memory row x0 + e/(BK/8), k0 + 8*(e%(BK/8)) .. +7.  The row a
// piece reads does not change from slice to slice, so its address (and gather lookup) is formed once.
template <int X, int BK, int NT>
struct DirectLoader {
    static constexpr int N = X * BK / 8 / NT;
    const uint16_t* rowp[N];     // null: row outside the operand
    int kc[N];
    __device__ __forceinline__ void init(const Operand& o, const uint16_t* base, const int32_t* gather, int x0, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int e = tid + NT * i;
            const int x = x0 + e / (BK / 8);
            kc[i] = (e % (BK / 8)) * 8;
            rowp[i] = nullptr;
            if (x < o.n_rows) rowp[i] = base + (gather ? (long)gather[x] : (long)x) * o.ld + kc[i];
        }
    }
    // STREAM: the operand is read once per launch and comes from memory (weights that do not fit the
    // memory-side cache): non-temporal loads
    template <bool STREAM>
    __device__ __forceinline__ void load_as(StageRegs<N>& g, const Operand& o, int k0) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            u32x4 val = {0u, 0u, 0u, 0u};
            if (rowp[i] && k0 + kc[i] < o.n_cont)
                val = STREAM ? __builtin_nontemporal_load((const u32x4*)(rowp[i] + k0)) : *(const u32x4*)(rowp[i] + k0);
            g.v[i] = val;
        }
    }
    __device__ __forceinline__ void load(StageRegs<N>& g, const Operand& o, int k0, bool stream = false) const {
        if (stream) load_as<true>(g, o, k0); else load_as<false>(g, o, k0);
    }
    __device__ __forceinline__ void store(const StageRegs<N>& g, uint16_t* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int e = tid + NT * i;
            *(u32x4*)(lds + (e / (BK / 8)) * dpitch(BK) + (e % (BK / 8)) * 8) = g.v[i];
        }
    }
};

// Transposed operand: piece e covers memory row k0 + e/(X/8), columns x0 + 8*(e%(X/8)) .. +7.
// GATHER is a compile-time property: the plain path then contains no index loads and no waits.
template <int X, int BK, int NT, bool GATHER>
struct TransLoader {
    static constexpr int N = X * BK / 8 / NT;
    const uint16_t* colp;        // base + this thread's (clamped) column offset
    const int32_t* gather;
    bool col_ok;                 // the thread's columns lie inside the operand
    unsigned row_ok;             // bit i: piece i of the slice in the registers lies inside the operand
    int32_t next_row[GATHER ? N : 1];   // gathered rows of the slice that the next load() fetches
    __device__ __forceinline__ void lookup(const Operand& o, int k0, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int k = k0 + (tid + NT * i) / (X / 8);
            if constexpr (GATHER) next_row[i] = gather[min(k, o.n_rows - 1)];
        }
    }
    __device__ __forceinline__ void init(const Operand& o, const uint16_t* base, const int32_t* g, int x0, int tid) {
        const int x = x0 + (tid % (X / 8)) * 8;      // NT is a multiple of X/8: same column for every piece
        col_ok = x < o.n_cont;
        colp = base + min(x, o.n_cont - 8);
        gather = g;
        row_ok = 0;
        lookup(o, 0, tid);
    }
    // No load is predicated: rows and columns outside the operand are clamped to valid addresses and
    // the piece is replaced by zeros on its way to LDS.  Without branches around the loads the
    // compiler can count how many are outstanding, so a wait for this slice does not have to be a
    // wait for every load issued since.  Gathered rows are looked up one slice ahead (init for the first
    // slice, each load() for the following one), so the wait for them is a wait for old loads only.
    // Slices are fetched in ascending order, BK apart.
    __device__ __forceinline__ void load(StageRegs<N>& g, const Operand& o, int k0, int tid) {
        long row[N];
        row_ok = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int k = k0 + (tid + NT * i) / (X / 8);
            if (k < o.n_rows) row_ok |= 1u << i;
            row[i] = GATHER ? (long)next_row[i] : (long)min(k, o.n_rows - 1);
        }
        lookup(o, k0 + BK, tid);
#pragma unroll
        for (int i = 0; i < N; ++i) g.v[i] = *(const u32x4*)(colp + row[i] * o.ld);
    }
    __device__ __forceinline__ void store(const StageRegs<N>& g, uint16_t* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int e = tid + NT * i;
            const u32x4 zero = {0u, 0u, 0u, 0u};
            const bool ok = col_ok && ((row_ok >> i) & 1u);
            *(u32x4*)(lds + (e / (X / 8)) * tpitch(X) + (e % (X / 8)) * 8) = ok ? g.v[i] : zero;
        }
    }
};

// Direct operand that is the implicit patch matrix of a convolution (Operand::cv_c): same pieces and the same LDS
// tile as DirectLoader; the 8 channels of a piece come from the pixel that the piece's tap points at.
template <int X, int BK, int NT>
struct ConvDirectLoader {
    static constexpr int N = X * BK / 8 / NT;
    const uint16_t* pixp[N];     // channel 0 of the row's own pixel; null: row outside the operand
    int h[N], w[N], kc[N];
    __device__ __forceinline__ void init(const Operand& o, const uint16_t* base, int x0, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int e = tid + NT * i;
            const int x = x0 + e / (BK / 8);
            kc[i] = (e % (BK / 8)) * 8;
            pixp[i] = nullptr; h[i] = 0; w[i] = 0;
            if (x < o.n_rows) {
                const uint32_t pos = (uint32_t)x - fastdiv((uint32_t)x, o.div_hw_m, o.div_hw_s) * (uint32_t)(o.cv_H * o.cv_W);
                h[i] = (int)fastdiv(pos, o.div_w_m, o.div_w_s);
                w[i] = (int)pos - h[i] * o.cv_W;
                pixp[i] = base + (size_t)x * o.cv_c;
            }
        }
    }
    __device__ __forceinline__ void load(StageRegs<N>& g, const Operand& o, int k0) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            u32x4 val = {0u, 0u, 0u, 0u};
            const int k = k0 + kc[i];
            if (pixp[i] && k < o.n_cont) {
                const int tap = (int)fastdiv((uint32_t)k, o.div_c_m, o.div_c_s);
                const int ch = k - tap * o.cv_c;
                const int kh = (tap * 11) >> 5;                  // tap / 3 for tap < 9
                const int dh = o.cv_sign * (kh - 1), dw = o.cv_sign * (tap - 3 * kh - 1);
                if ((unsigned)(h[i] + dh) < (unsigned)o.cv_H && (unsigned)(w[i] + dw) < (unsigned)o.cv_W)
                    val = *(const u32x4*)(pixp[i] + (long)(dh * o.cv_W + dw) * o.cv_c + ch);
            }
            g.v[i] = val;
        }
    }
    __device__ __forceinline__ void store(const StageRegs<N>& g, uint16_t* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int e = tid + NT * i;
            *(u32x4*)(lds + (e / (BK / 8)) * dpitch(BK) + (e % (BK / 8)) * 8) = g.v[i];
        }
    }
};

// Transposed operand that is the implicit patch matrix of a convolution: memory row = position k (offset by
// k_off inside the learner's image stack: the launch may hand a workgroup a range of positions), columns = (tap,
// channel).  A thread's pieces all have the same columns, hence one tap; invalid pieces (outside the image, the
// operand or the range) are loaded from a safe address and replaced by zeros on their way to LDS, so that no
// load is predicated.
template <int X, int BK, int NT>
struct ConvTransLoader {
    static constexpr int N = X * BK / 8 / NT;
    const uint16_t* base;
    const uint16_t* colp;        // base + (tap offset in pixels) * c + channel: add k * c for the pixel of row k
    int dh, dw, k_off;
    bool col_ok;
    unsigned row_ok;
    __device__ __forceinline__ void init(const Operand& o, const uint16_t* b, int koff, int x0, int tid) {
        const int x = x0 + (tid % (X / 8)) * 8;
        col_ok = x < o.n_cont;
        const int xx = min(x, o.n_cont - 8);
        const int tap = (int)fastdiv((uint32_t)xx, o.div_c_m, o.div_c_s);
        const int ch = xx - tap * o.cv_c;
        const int kh = (tap * 11) >> 5;
        dh = o.cv_sign * (kh - 1); dw = o.cv_sign * (tap - 3 * kh - 1);
        base = b; k_off = koff;
        colp = b + (long)(dh * o.cv_W + dw) * o.cv_c + ch;
        row_ok = 0;
    }
    __device__ __forceinline__ void load(StageRegs<N>& g, const Operand& o, int k0, int tid) {
        row_ok = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int kl = k0 + (tid + NT * i) / (X / 8);          // row inside this workgroup's range
            const uint32_t k = (uint32_t)(k_off + min(kl, o.n_rows - 1));
            const uint32_t pos = k - fastdiv(k, o.div_hw_m, o.div_hw_s) * (uint32_t)(o.cv_H * o.cv_W);
            const int h = (int)fastdiv(pos, o.div_w_m, o.div_w_s), w = (int)pos - h * o.cv_W;
            const bool ok = kl < o.n_rows && (unsigned)(h + dh) < (unsigned)o.cv_H && (unsigned)(w + dw) < (unsigned)o.cv_W;
            if (ok) row_ok |= 1u << i;
            g.v[i] = *(const u32x4*)(ok ? colp + (size_t)k * o.cv_c : base);
        }
    }
    __device__ __forceinline__ void store(const StageRegs<N>& g, uint16_t* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int e = tid + NT * i;
            const u32x4 zero = {0u, 0u, 0u, 0u};
            const bool ok = col_ok && ((row_ok >> i) & 1u);
            *(u32x4*)(lds + (e / (X / 8)) * tpitch(X) + (e % (X / 8)) * 8) = ok ? g.v[i] : zero;
        }
    }
};

// MFMA fragment (lane l: index l%32 of the 32-block, k = 8*(l/32) .. +7 of the 16-slab kk)
template <int BK>
__device__ __forceinline__ bf16x8 frag_direct(const uint16_t* tile, int block_row0, int kk, int lane) {
    return *(const bf16x8*)(tile + (block_row0 + (lane & 31)) * dpitch(BK) + kk * 16 + (lane >> 5) * 8);
}

// Same fragment out of a [k][x] tile with two transpose reads.  In its 16-lane group, lane t = 4a + b
// fetches x = 4b .. 4b+3 of row k = a and receives the four k (a = 0..3) of x = t.
template <int X>
__device__ __forceinline__ bf16x8 frag_trans(const uint16_t* tile, int block_x0, int kk, int lane) {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    const int t = lane & 15, grp = lane >> 4;
    const int krow = kk * 16 + (grp >> 1) * 8 + (t >> 2);
    const int xcol = block_x0 + (grp & 1) * 16 + (t & 3) * 4;
    const uint16_t* p = tile + krow * tpitch(X) + xcol;
    typedef bf16x4 __attribute__((address_space(3))) * lds_ptr;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)p);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(p + 4 * tpitch(X)));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Direct global -> LDS loads (global_load_lds_dwordx4): a wavefront instruction moves 64 pieces of
// 16 bytes into 1 KB of consecutive LDS, lane l to byte 16*l, so rows cannot be padded.  The tile
// is [x][BK] with rows of exactly BK bf16 and the 16-byte chunks of row x permuted by an XOR:
// LDS slot (x, c') holds memory chunk c' ^ s(x), s(x) = x mod 16 for rows of 256 bytes (BK = 128) and
// (x/2) mod 8 for rows of 128 bytes (BK = 64: two rows per 256-byte bank period).  Sixteen
// consecutive rows then put any one chunk index into sixteen different 16-byte bank groups, so
// fragment reads are conflict-free.  (Three or four LDS buffers were measured too: no faster.)  Piece i of a wavefront covers slots (wave*N + i)*64 .. +63.
// Rows outside the operand are clamped to its last row: they only reach outputs that are never
// stored.  A chunk beyond the contraction length is clamped too and zeroed in LDS after it has
// landed (fix_tail), by the lane that loaded it.
template <int BK> __device__ __forceinline__ int dma_swizzle(int x) {
    static_assert(BK == 128 || BK == 64 || BK == 32, "rows of 256 bytes (one per bank period), 128 bytes (two) or 64 bytes (four)");
    return BK == 128 ? (x & 15) : BK == 64 ? ((x >> 1) & 7) : ((x >> 2) & 3);
}

template <int X, int BK, int NT>
struct DmaLoader {
    static constexpr int N = X * BK / 8 / NT;
    static constexpr int CPR = BK / 8;           // chunks per row
    const uint16_t* row[N];      // start of the (clamped) memory row of piece i, plus the piece's chunk offset
    int chunk8[N];               // first element of the piece's memory chunk within a slice
    int wave;                    // wavefront index, uniform (kept in a scalar register)
    __device__ __forceinline__ void init(const Operand& o, const uint16_t* base, const int32_t* gather, int x0, int tid) {
        const int lane = tid & 63;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int slot = (wave * N + i) * 64 + lane;
            const int xr = slot / CPR;
            const int x = min(x0 + xr, o.n_rows - 1);
            chunk8[i] = ((slot % CPR) ^ dma_swizzle<BK>(xr)) * 8;
            row[i] = base + (gather ? (long)gather[x] : (long)x) * o.ld + chunk8[i];
        }
    }
    // FULL: the slice lies inside the contraction (k0 + BK <= n_cont), no clamping needed
    // AUX: cache policy bits of the load instruction (2: non-temporal)
    template <bool FULL, int AUX = 0>
    __device__ __forceinline__ void load(const Operand& o, int k0, uint16_t* tile) const {
        typedef __attribute__((address_space(3))) void* lds_p;
        typedef const __attribute__((address_space(1))) void* glb_p;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int k = FULL ? k0 : min(k0 + chunk8[i], o.n_cont - 8) - chunk8[i];
            __builtin_amdgcn_global_load_lds((glb_p)(row[i] + k), (lds_p)(tile + (wave * N + i) * 64 * 8), 16, 0, AUX);
        }
    }
    __device__ __forceinline__ void load(const Operand& o, int k0, uint16_t* tile, int, bool stream = false) const {
        if (stream) { if (k0 + BK <= o.n_cont) load<true, 2>(o, k0, tile); else load<false, 2>(o, k0, tile); }
        else { if (k0 + BK <= o.n_cont) load<true>(o, k0, tile); else load<false>(o, k0, tile); }
    }
    __device__ __forceinline__ void fix_tail(const Operand& o, int k0, uint16_t* tile, int tid) const {
        const int lane = tid & 63;
#pragma unroll
        for (int i = 0; i < N; ++i)
            if (k0 + chunk8[i] >= o.n_cont) {
                const u32x4 zero = {0u, 0u, 0u, 0u};
                *(u32x4*)(tile + ((wave * N + i) * 64 + lane) * 8) = zero;
            }
    }
};

template <int BK>
__device__ __forceinline__ bf16x8 frag_swizzled(const uint16_t* tile, int block_row0, int kk, int lane) {
    const int x = block_row0 + (lane & 31);
    const int c = (kk * 2 + (lane >> 5)) ^ dma_swizzle<BK>(x);
    return *(const bf16x8*)(tile + x * BK + c * 8);
}

// LDS budget of a kernel shape (shared by the kernel and its launcher).
template <int MODE, int TR, int TC, int WR, int WC, int WK, int BK, bool RTRANS, bool CTRANS, int PIPE>
struct Shape {
    static constexpr int MR = TR / (32 * WR), MC = TC / (32 * WC);
    static constexpr int WTC = MC * 32;                 // columns of a wavefront's tile
    static constexpr int SPITCH = WTC + 4;              // update epilogue: fp32 staging row, padded
    static constexpr bool DIRECT = PIPE == PIPE_DMA || PIPE == PIPE_RING;       // global -> LDS loads, unpadded swizzled tiles
    static constexpr int THREADS = 64 * (WR * WC * WK + (PIPE == PIPE_RING ? RING_LOADERS : 0));
    static constexpr int R_ELEMS = DIRECT ? TR * BK : RTRANS ? BK * tpitch(TR) : TR * dpitch(BK);
    static constexpr int C_ELEMS = DIRECT ? TC * BK : CTRANS ? BK * tpitch(TC) : TC * dpitch(BK);
    static constexpr int RING_BUFS = RING_BYTES / ((R_ELEMS + C_ELEMS) * 2);
    static constexpr int OPER_BYTES = (PIPE == PIPE_PLAIN ? 1 : PIPE == PIPE_RING ? RING_BUFS : 2) * (R_ELEMS + C_ELEMS) * 2;
    static constexpr int STAGE_BYTES = MODE == MODE_UPD ? 4 * 32 * SPITCH * 4 : 0;
    static constexpr int KRED_BYTES = WK > 1 ? WR * WC * MR * MC * 16 * 64 * 4 : 0;   // one k group's partial tiles
    static constexpr int SMEM1 = OPER_BYTES > STAGE_BYTES ? OPER_BYTES : STAGE_BYTES;
    static constexpr int SMEM_BYTES = SMEM1 > KRED_BYTES ? SMEM1 : KRED_BYTES;
};

// ---- the kernel ----------------------------------------------------------------
// TR x TC output tile; WR x WC x WK wavefronts: WR x WC of them tile the output, each owning MR x MC
// MFMA blocks of 32x32, and WK groups of those split every slice along k (their partial tiles are
// summed through LDS at the end, in fixed order).  BK = slice length.  One slice is always in
// flight in registers ahead of the one being multiplied; with PIPE_LDS2 the LDS tiles are double-buffered,
// so the next slice is written while the current one is read and a slice costs one barrier, not two.
// CONV_R / CONV_C: that operand is the implicit patch matrix of a convolution (Operand::cv_c).
template <int MODE, int TR, int TC, int WR, int WC, int WK, int BK, bool RTRANS, bool CTRANS, int PIPE, bool SHADOW_CACHED = false,
          bool GATHER_C = false, bool CONV_R = false, bool CONV_C = false>
__global__ void __launch_bounds__(64 * (WR * WC * WK + (PIPE == PIPE_RING ? RING_LOADERS : 0))) gemm_bf16_kernel(Args a) {
    static_assert(!CONV_R || (!RTRANS && PIPE != PIPE_DMA), "implicit R operand: k-contiguous, staged through registers");
    static_assert(!CONV_C || (CTRANS && !GATHER_C && MODE == MODE_UPD), "implicit C operand: the update's transposed operand");
    constexpr int NW = WR * WC * WK, NT = 64 * NW;
    constexpr int MR = TR / (32 * WR), MC = TC / (32 * WC);
    static_assert(MR >= 1 && MC >= 1, "tile too small for the wave grid");
    static_assert((BK / 16) % WK == 0, "slice must split evenly over the k groups");
    static_assert(MODE != MODE_UPD || (WK == 1 && NW == 4 && PIPE == PIPE_PLAIN), "the update epilogue assumes 4 wavefronts, no k split, one LDS buffer");
    constexpr bool DIRECT = PIPE == PIPE_DMA || PIPE == PIPE_RING;
    static_assert(PIPE != PIPE_RING || (WK == 1 && MODE != MODE_UPD), "ring pipeline: forward / backward-data without a k split");
    static_assert(NT % (TR / 8) == 0 && NT % (TC / 8) == 0, "loader column mapping");
    typedef Shape<MODE, TR, TC, WR, WC, WK, BK, RTRANS, CTRANS, PIPE> SH;
    constexpr int WTC = SH::WTC, SPITCH = SH::SPITCH, R_ELEMS = SH::R_ELEMS, C_ELEMS = SH::C_ELEMS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];     // SH::SMEM_BYTES, set at launch
    uint16_t* Rs = (uint16_t*)smem;                 // buffer b: Rs + b*(R_ELEMS + C_ELEMS), Cs likewise
    uint16_t* Cs = Rs + R_ELEMS;
    constexpr int BUF_ELEMS = R_ELEMS + C_ELEMS;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave / (WR * WC), wrc = wave % (WR * WC);
    const int wr = wrc / WC, wc = wrc % WC;
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2) in launch order, so
    // workgroup g runs on XCD g%8.  Give every XCD one contiguous range of the logical order
    // (learner, row tile, column tile): the tiles of a learner then share that learner's operands
    // through a single L2 instead of pulling them into all eight.
    const int logical = (int)(blockIdx.x & 7) * a.chunk + (int)(blockIdx.x >> 3);
    if (logical >= a.total_wg) return;
    const int learner = logical / (a.tiles_r * a.tiles_c);
    const int tile = logical - learner * (a.tiles_r * a.tiles_c);
    const int tile_r = tile / a.tiles_c, tile_c = tile - tile_r * a.tiles_c;
    const int r0 = tile_r * TR, c0 = tile_c * TC;

    const uint16_t* Rbase = a.R.base + (size_t)learner * a.R.lstride;
    const uint16_t* Cbase = a.C.base + (size_t)learner * a.C.lstride;
    int c_koff = 0;
    if constexpr (CONV_C) {                     // "learner" = (real learner, range of positions): the image stack is the real learner's
        Cbase = a.C.base + (size_t)(learner / a.cv_splits) * a.C.lstride;
        c_koff = (learner % a.cv_splits) * a.C.n_rows;
    }
    const int32_t* Rg = a.R.gather ? a.R.gather + (long)learner * a.R.gstride : nullptr;
    const int32_t* Cg = a.C.gather ? a.C.gather + (long)learner * a.C.gstride : nullptr;

    f32x16 acc[MR][MC];
#pragma unroll
    for (int i = 0; i < MR; ++i)
#pragma unroll
        for (int j = 0; j < MC; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    DirectLoader<TR, BK, NT> rdl; TransLoader<TR, BK, NT, false> rtl; ConvDirectLoader<TR, BK, NT> rcl;
    DirectLoader<TC, BK, NT> cdl; TransLoader<TC, BK, NT, GATHER_C> ctl; ConvTransLoader<TC, BK, NT> ccl;
    if constexpr (!DIRECT) {                    // (direct global->LDS pipelines set up their own loaders below)
        if constexpr (CONV_R) rcl.init(a.R, Rbase, r0, tid);
        else if (RTRANS) rtl.init(a.R, Rbase, Rg, r0, tid); else rdl.init(a.R, Rbase, Rg, r0, tid);
        if constexpr (CONV_C) ccl.init(a.C, Cbase, c_koff, c0, tid);
        else if (CTRANS) ctl.init(a.C, Cbase, Cg, c0, tid); else cdl.init(a.C, Cbase, Cg, c0, tid);
    }
    StageRegs<TR * BK / 8 / NT> rg;
    StageRegs<TC * BK / 8 / NT> cg;
    float bias_sum = 0.f;                       // update: column sum of dZ for row r0 + tid
    uint32_t touched = 0;                       // update of the first layer: see the prefetch below

    auto fetch = [&](int k0) {
        if constexpr (CONV_R) rcl.load(rg, a.R, k0);
        else if (RTRANS) rtl.load(rg, a.R, k0, tid); else rdl.load(rg, a.R, k0);
        if constexpr (CONV_C) ccl.load(cg, a.C, k0, tid);
        else if (CTRANS) ctl.load(cg, a.C, k0, tid); else cdl.load(cg, a.C, k0, MODE == MODE_FWD && a.c_stream);
    };
    auto stash = [&](int buf) {
        if constexpr (CONV_R) rcl.store(rg, Rs + buf * BUF_ELEMS, tid);
        else if (RTRANS) rtl.store(rg, Rs + buf * BUF_ELEMS, tid); else rdl.store(rg, Rs + buf * BUF_ELEMS, tid);
        if constexpr (CONV_C) ccl.store(cg, Cs + buf * BUF_ELEMS, tid);
        else if (CTRANS) ctl.store(cg, Cs + buf * BUF_ELEMS, tid); else cdl.store(cg, Cs + buf * BUF_ELEMS, tid);
    };
    // Fragments of k slab kq+1 are requested before the MFMAs of slab kq are issued (two register
    // sets, statically indexed), so that the matrix cores do not wait for an LDS round trip per slab.
    // Fragments of k slab kq+1 are requested before the MFMAs of slab kq are issued (two register
    // sets, statically indexed), so that the matrix cores do not wait for an LDS round trip per slab.
    auto multiply_tiles = [&](const uint16_t* R, const uint16_t* C) {
        constexpr int KQ = BK / 16 / WK;
        bf16x8 cf[2][MC], rf[2][MR];
        auto fetch_frags = [&](int set, int kq) {
            const int kk = wk * KQ + kq;
#pragma unroll
            for (int j = 0; j < MC; ++j)
                if constexpr (DIRECT) cf[set][j] = frag_swizzled<BK>(C, (wc * MC + j) * 32, kk, lane);
                else cf[set][j] = CTRANS ? frag_trans<TC>(C, (wc * MC + j) * 32, kk, lane)
                                         : frag_direct<BK>(C, (wc * MC + j) * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < MR; ++i)
                if constexpr (DIRECT) rf[set][i] = frag_swizzled<BK>(R, (wr * MR + i) * 32, kk, lane);
                else rf[set][i] = RTRANS ? frag_trans<TR>(R, (wr * MR + i) * 32, kk, lane)
                                         : frag_direct<BK>(R, (wr * MR + i) * 32, kk, lane);
        };
        fetch_frags(0, 0);
#pragma unroll
        for (int kq = 0; kq < KQ; ++kq) {
            if (kq + 1 < KQ) fetch_frags((kq + 1) & 1, kq + 1);
#pragma unroll
            for (int i = 0; i < MR; ++i)
#pragma unroll
                for (int j = 0; j < MC; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf[kq & 1][j], rf[kq & 1][i], acc[i][j], 0, 0, 0);
        }
        // Pin that order for the instruction scheduler (it would otherwise fold the two fragment sets
        // back into one and read each slab right before its MFMAs): LDS reads of slab 0, then for every
        // slab the reads of the next one followed by its own MFMAs.
        constexpr int DS_PER_SLAB = MC * ((!DIRECT && CTRANS) ? 2 : 1) + MR * ((!DIRECT && RTRANS) ? 2 : 1);
        __builtin_amdgcn_sched_group_barrier(0x100, DS_PER_SLAB, 0);
#pragma unroll
        for (int kq = 0; kq < KQ; ++kq) {
            if (kq + 1 < KQ) __builtin_amdgcn_sched_group_barrier(0x100, DS_PER_SLAB, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MR * MC, 0);
        }
    };
    auto multiply = [&](int buf) { multiply_tiles(Rs + buf * BUF_ELEMS, Cs + buf * BUF_ELEMS); };

    // Update epilogue: a lane owns eight consecutive columns of a row, 16 bytes of either plane.
    constexpr int L8_PER_ROW = WTC / 8;
    constexpr int ROWS_PER_IT = 64 / L8_PER_ROW;
    constexpr int ITS = 32 / ROWS_PER_IT;
    u32x4 mhi[MODE == MODE_UPD ? MR : 1][MODE == MODE_UPD ? ITS : 1];
    u32x4 mlo[MODE == MODE_UPD ? MR : 1][MODE == MODE_UPD ? ITS : 1];

    // What the epilogue reads from memory (bias of the lane's columns; ReLU mask of its outputs) is
    // requested here, ahead of the contraction, so that its latency is not paid after the last slice
    // -- for single-block wavefront tiles only: with more blocks the extra registers cost occupancy.
    // Only the wavefronts of k group 0 reach the epilogue.
    constexpr bool EARLY = MR * MC == 1;
    // bias of four columns: raw hi / lo words (requested early, joined only where they are used: joining
    // at once would make every request wait for its own answer)
    auto bias_raw = [&](int j, int q, u32x2& h, u32x2& l) {
        const uint16_t* bh = a.bias_hi + (size_t)learner * a.bias_lstride;
        const uint16_t* bl = a.bias_lo + (size_t)learner * a.bias_lstride;
        const int c = c0 + (wc * MC + j) * 32 + q * 8 + (lane >> 5) * 4;
        h = (u32x2){0u, 0u}; l = (u32x2){0u, 0u};
        if (!a.bias_hi) return;                   // product without a bias term
        if (c + 4 <= a.nC) {                      // four columns at once (the planes are 8-byte aligned there)
            h = *(const u32x2*)(bh + c); l = *(const u32x2*)(bl + c);
        } else {                                  // ragged end: column by column, zeros beyond the layer
            uint32_t hv[4] = {0u, 0u, 0u, 0u}, lv[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 4; ++e) if (c + e < a.nC) { hv[e] = bh[c + e]; lv[e] = bl[c + e]; }
            h = (u32x2){hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16)};
            l = (u32x2){lv[0] | (lv[1] << 16), lv[2] | (lv[3] << 16)};
        }
    };
    auto bias_join = [&](const u32x2& h, const u32x2& l) {
        uint32_t b0, b1, b2, b3;
        split_join2(h.x, l.x, b0, b1);
        split_join2(h.y, l.y, b2, b3);
        return (f32x4){__builtin_bit_cast(float, b0), __builtin_bit_cast(float, b1),
                       __builtin_bit_cast(float, b2), __builtin_bit_cast(float, b3)};
    };
    auto mask_of = [&](int i, int j, int q) {
        const int r = r0 + (wr * MR + i) * 32 + (lane & 31);
        const int c = c0 + (wc * MC + j) * 32 + q * 8 + (lane >> 5) * 4;
        u32x2 m = {0u, 0u};
        if (a.act_prev && r < a.nR && c < a.nC)
            m = *(const u32x2*)(a.act_prev + (size_t)learner * a.act_lstride + (size_t)r * a.ld_act + c);
        return m;
    };
    u32x2 ebh[4], ebl[4];
    u32x2 emask[4];
    if (EARLY && wk == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (MODE == MODE_FWD) bias_raw(0, q, ebh[q], ebl[q]);
            if (MODE == MODE_BWD) emask[q] = mask_of(0, 0, q);
        }
    }

    if constexpr (PIPE == PIPE_RING) {
        static_assert(!RTRANS && !CTRANS, "direct LDS loads: k-contiguous operands only");
        // Slice s lives in buffer s % NB and is requested NB - 1 slices ahead, both operands alike: the
        // memory pipeline of a compute unit hands loads back in the order they were issued, so the
        // activations (cache hits) cannot overtake the weights (which come from memory, once each) and
        // gain nothing from being requested later.  Barrier s (one per slice, all wavefronts): the
        // loaders arrive once slice s has landed, the multipliers once they are done with slice s-1;
        // after it the loaders refill the buffer of slice s-1.  The loaders' barrier carries no fence:
        // a fence would make them wait for everything they have requested.
        constexpr int NB = SH::RING_BUFS, D = NB - 1;
        constexpr int LN = (TR + TC) * BK / 8 / (64 * RING_LOADERS);     // loads per loader wavefront and slice
        static_assert(D >= 1 && D <= 5 && D * LN <= 63, "the slices in flight must fit the wavefront's load counter");
        const int slices = a.nK / BK;               // (whole slices: checked by the launcher)
        if (__builtin_amdgcn_readfirstlane(wave) >= NW) {
            DmaLoader<TR, BK, 64 * RING_LOADERS> rdma; DmaLoader<TC, BK, 64 * RING_LOADERS> cdma;
            rdma.init(a.R, Rbase, Rg, r0, tid - NT);
            cdma.init(a.C, Cbase, Cg, c0, tid - NT);
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (d < slices) {
                    rdma.template load<true>(a.R, d * BK, Rs + d * BUF_ELEMS);
                    if (a.c_stream) cdma.template load<true, 2>(a.C, d * BK, Cs + d * BUF_ELEMS);
                    else cdma.template load<true>(a.C, d * BK, Cs + d * BUF_ELEMS);
                }
            int fill = D;                           // buffer of slice s + D
            for (int s = 0; s < slices; ++s) {
                // slice s has landed when at most the younger ones are on their way
                switch (min(D - 1, slices - 1 - s)) {
                    case 4: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(D > 4 ? 4 * LN : 0) : "memory"); break;
                    case 3: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(D > 3 ? 3 * LN : 0) : "memory"); break;
                    case 2: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(D > 2 ? 2 * LN : 0) : "memory"); break;
                    case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(D > 1 ? LN : 0) : "memory"); break;
                    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                }
                asm volatile("s_barrier" ::: "memory");
                if (s + D < slices) {
                    rdma.template load<true>(a.R, (s + D) * BK, Rs + fill * BUF_ELEMS);
                    if (a.c_stream) cdma.template load<true, 2>(a.C, (s + D) * BK, Cs + fill * BUF_ELEMS);
                    else cdma.template load<true>(a.C, (s + D) * BK, Cs + fill * BUF_ELEMS);
                }
                fill = fill == NB - 1 ? 0 : fill + 1;
            }
            asm volatile("s_barrier" ::: "memory");
            return;
        }
        int buf = 0;
        for (int s = 0; s < slices; ++s) {
            __syncthreads();
            multiply(buf);
            buf = buf == NB - 1 ? 0 : buf + 1;
        }
        __syncthreads();                                // tiles are dead: the epilogue reuses their LDS
    } else if constexpr (PIPE == PIPE_DMA) {
        static_assert(!RTRANS && !CTRANS && MODE != MODE_UPD, "direct LDS loads: k-contiguous operands only");
        DmaLoader<TR, BK, NT> rdma; DmaLoader<TC, BK, NT> cdma;
        rdma.init(a.R, Rbase, Rg, r0, tid);
        cdma.init(a.C, Cbase, Cg, c0, tid);
        rdma.load(a.R, 0, Rs, tid);
        cdma.load(a.C, 0, Cs, tid, a.c_stream);
        int buf = 0;
        for (int k0 = 0; k0 < a.nK; k0 += BK, buf ^= 1) {
            __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): this wavefront's part of slice k0 is in LDS
            if (k0 + BK > a.R.n_cont || k0 + BK > a.C.n_cont) {      // ragged end of the contraction
                rdma.fix_tail(a.R, k0, Rs + buf * BUF_ELEMS, tid);
                cdma.fix_tail(a.C, k0, Cs + buf * BUF_ELEMS, tid);
            }
            __syncthreads();                            // everyone's part is; the other buffer is no longer read
            if (k0 + BK < a.nK) {                       // next slice lands while this one is multiplied
                rdma.load(a.R, k0 + BK, Rs + (buf ^ 1) * BUF_ELEMS, tid);
                cdma.load(a.C, k0 + BK, Cs + (buf ^ 1) * BUF_ELEMS, tid, a.c_stream);
            }
            multiply(buf);
        }
        __syncthreads();                                // tiles are dead: the k-group reduction reuses their LDS
    } else {
        // Update of the first layer: the rows that the next local step samples are scattered over the data
        // set, and its forward pass, with one slice of look-ahead, would pay the latency of such a read in
        // every slice.  This launch lasts long, so its workgroups touch those rows, one 128-byte line
        // per lane (the learner's rows are spread over the learner's workgroups, which run on the XCD
        // that will run its forward tiles).  One unpredicated load per lane, so that it can be
        // counted; its row index is looked up first of all, so that waiting for the index does not
        // mean waiting for the loads below; the value is only kept alive until the end of the kernel.
        // Without a next step, or without a gather, the line touched is one of this launch's own operand.
        const uint32_t* touch_at = nullptr;
        if (MODE == MODE_UPD) {
            const int lines_per_row = (a.C.n_cont * 2 + 127) / 128;
            const int lines = a.C.n_rows * lines_per_row;                 // of this learner
            const int wgs = a.tiles_r * a.tiles_c;
            const int per_wg = min((lines + wgs - 1) / wgs, NT);          // beyond NT lines the rest stays untouched
            const int line = min(tile * per_wg + min(tid, per_wg - 1), lines - 1);
            const int row = line / lines_per_row, ln = line - row * lines_per_row;
            long mrow = row;
            if constexpr (GATHER_C) mrow = ((a.next_gather ? a.next_gather : a.C.gather) + (long)learner * a.C.gstride)[row];
            touch_at = (const uint32_t*)(Cbase + mrow * a.C.ld + ln * 64);
            if constexpr (CONV_C) touch_at = (const uint32_t*)Cbase;     // nothing to prefetch: the images are this launch's own operand
        }
        fetch(0);
        if (MODE == MODE_UPD) {
            __builtin_amdgcn_sched_barrier(0);          // keep the operand loads the oldest
            // The master tile (both planes) is independent of the product: its loads go out right after
            // the first operand slice and are in flight during the contraction.  They are issued
            // without predicates (rows and columns beyond the layer are clamped; those lanes store
            // nothing later), so that the compiler can count them: the wait for the operand slice is
            // then "all but these", not "everything".
            // (with partial outputs nothing is stepped; the loads then go to learner 0's tile and are ignored,
            // so that the load sequence keeps its branch-free shape)
            const size_t mlearner = a.partial ? 0 : (size_t)learner;
            const uint16_t* hbase = a.ws + mlearner * a.ws_lstride;
            const uint16_t* lbase = a.wlo + mlearner * a.ws_lstride;
            const int c = min(c0 + wc * WTC + (lane % L8_PER_ROW) * 8, a.nC - 8);
#pragma unroll
            for (int i = 0; i < MR; ++i)
#pragma unroll
                for (int it = 0; it < ITS; ++it) {
                    const int r = min(r0 + (wr * MR + i) * 32 + it * ROWS_PER_IT + lane / L8_PER_ROW, a.nR - 1);
                    // hi was left in the memory-side cache by the previous writer when it fits there
                    // (otherwise it is streamed like lo, so as not to push anything else out)
                    mhi[i][it] = SHADOW_CACHED ? *(const u32x4*)(hbase + (size_t)r * a.nC + c)
                                               : __builtin_nontemporal_load((const u32x4*)(hbase + (size_t)r * a.nC + c));
                    mlo[i][it] = __builtin_nontemporal_load((const u32x4*)(lbase + (size_t)r * a.nC + c));
                }
            __builtin_amdgcn_sched_barrier(0);
            touched = *touch_at;
        }
        if (PIPE == PIPE_PLAIN) {
            auto slice = [&](int k0) {
                stash(0);
                __syncthreads();
                if (k0 + BK < a.nK) fetch(k0 + BK);     // next slice in flight during the MFMAs
                multiply(0);
                if (MODE == MODE_UPD && tile_c == 0 && tid < TR) {
                    // R tile of the update is dZ as [sample][unit]: column tid summed over the slice's samples
#pragma unroll 8
                    for (int k = 0; k < BK; ++k) bias_sum += bf16_to_f32(Rs[k * tpitch(TR) + tid]);
                }
                __syncthreads();
            };
            // The first slice stands outside the loop: there the compiler knows that the operand loads
            // are the oldest outstanding ones and waits only for them, not for the master tile.
            slice(0);
            for (int k0 = BK; k0 < a.nK; k0 += BK) slice(k0);
        } else {
            stash(0);
            __syncthreads();
            if (BK < a.nK) fetch(BK);
            int buf = 0;
            for (int k0 = 0; k0 < a.nK; k0 += BK, buf ^= 1) {
                if (k0 + BK < a.nK) {
                    stash(buf ^ 1);                     // slice k0+BK, written while slice k0 is read
                    if (k0 + 2 * BK < a.nK) fetch(k0 + 2 * BK);
                }
                multiply(buf);
                __syncthreads();
            }
        }
    }

    if (WK > 1) {
        // sum the k groups' partial tiles into group 0, group by group (fixed order), through one LDS patch
        float* red = (float*)smem;
#pragma unroll
        for (int g = 1; g < WK; ++g) {
            if (wk == g) {
#pragma unroll
                for (int i = 0; i < MR; ++i)
#pragma unroll
                    for (int j = 0; j < MC; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            red[((wrc * MR * MC + i * MC + j) * 16 + e) * 64 + lane] = acc[i][j][e];
            }
            __syncthreads();
            if (wk == 0) {
#pragma unroll
                for (int i = 0; i < MR; ++i)
#pragma unroll
                    for (int j = 0; j < MC; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            acc[i][j][e] += red[((wrc * MR * MC + i * MC + j) * 16 + e) * 64 + lane];
            }
            if (g + 1 < WK) __syncthreads();
        }
        if (wk != 0) return;
    }

    // ---- epilogue: lane owns, per block, row r = l%32 and columns 8q + 4(l/32) + 0..3, q = 0..3
    if (MODE != MODE_UPD) {
        // What the epilogue reads (bias of the lane's columns, ReLU masks of its outputs) is requested here in one
        // go, before any of it is used: one round trip to memory instead of one per block and column group.
        u32x2 pbh[MODE == MODE_FWD ? MC : 1][4], pbl[MODE == MODE_FWD ? MC : 1][4];
        u32x2 pmk[MODE == MODE_BWD ? MR : 1][MODE == MODE_BWD ? MC : 1][4];
        if (!EARLY) {
            if constexpr (MODE == MODE_FWD) {
#pragma unroll
                for (int j = 0; j < MC; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) bias_raw(j, q, pbh[j][q], pbl[j][q]);
            } else {
#pragma unroll
                for (int i = 0; i < MR; ++i)
#pragma unroll
                    for (int j = 0; j < MC; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) pmk[i][j][q] = mask_of(i, j, q);
            }
        }
        // bf16 outputs leave through a per-wavefront LDS patch (the operand tiles are dead by now): the accumulator
        // layout gives a lane 8 bytes in each of many rows, and stored like that every 128-byte line of the output
        // is written in sixteen pieces; out of the patch a lane stores 16 bytes and a wavefront whole row segments.
        constexpr bool STAGED = WK == 1;
        constexpr int OP = WTC + 8;                             // patch row: the wavefront's columns plus 16 bytes
        static_assert(!STAGED || NW * 32 * OP * 2 <= SH::SMEM_BYTES, "output patches fit the operand tiles' LDS");
        const bool bf16_out = MODE == MODE_FWD ? (a.epi == EPI_GRAM || a.relu != 0) : !(a.epi == EPI_RAW || a.epi == EPI_LOGITS);
        const bool staged = STAGED && bf16_out;
        uint16_t* opatch = (uint16_t*)smem + wave * 32 * OP;
        const int c_end = MODE == MODE_FWD ? a.ld_out : a.nC;  // first column that is not stored (a multiple of 8 for bf16 outputs)
#pragma unroll
        for (int i = 0; i < MR; ++i) {
            const int r = r0 + (wr * MR + i) * 32 + (lane & 31);
            const bool r_ok = r < a.nR;
#pragma unroll
            for (int j = 0; j < MC; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = c0 + (wc * MC + j) * 32 + q * 8 + (lane >> 5) * 4;
                    const bool ok = r_ok && c < c_end;
                    float v0 = acc[i][j][4 * q + 0], v1 = acc[i][j][4 * q + 1];
                    float v2 = acc[i][j][4 * q + 2], v3 = acc[i][j][4 * q + 3];
                    u32x2 o;
                    if (MODE == MODE_FWD) {
                        u32x2 bh2, bl2;
                        if (EARLY) { bh2 = ebh[q]; bl2 = ebl[q]; } else { bh2 = pbh[j][q]; bl2 = pbl[j][q]; }
                        const f32x4 bq = bias_join(bh2, bl2);
                        v0 += bq.x; v1 += bq.y; v2 += bq.z; v3 += bq.w;
                        if (a.epi == EPI_GRAM) {
                            o = (u32x2){pack2(a.alpha * v0, a.alpha * v1), pack2(a.alpha * v2, a.alpha * v3)};
                        } else if (a.relu) {
                            o = (u32x2){pack2(fmaxf(v0, 0.f), fmaxf(v1, 0.f)), pack2(fmaxf(v2, 0.f), fmaxf(v3, 0.f))};
                        } else {
                            if (ok) *(f32x4*)((float*)a.out + (size_t)learner * a.out_lstride + (size_t)r * a.ld_out + c) = (f32x4){v0, v1, v2, v3};
                            continue;
                        }
                    } else {
                        if (a.base && ok) {
                            const f32x4 bs = *(const f32x4*)(a.base + (size_t)learner * a.base_lstride + (size_t)r * a.ld_base + c);
                            v0 += bs.x; v1 += bs.y; v2 += bs.z; v3 += bs.w;
                        }
                        if (a.epi == EPI_RAW || a.epi == EPI_LOGITS) {
                            if (ok) *(f32x4*)((float*)a.out + (size_t)learner * a.out_lstride + (size_t)r * a.ld_out + c) = (f32x4){v0, v1, v2, v3};
                            continue;
                        }
                        if (a.epi == EPI_RELU) {
                            v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f);
                        } else {
                            const u32x2 m = EARLY ? emask[q] : pmk[i][j][q];
                            // stored activations are relu outputs (never negative): positive <=> non-zero magnitude
                            v0 = (m.x & 0x7FFFu) ? v0 : 0.f;
                            v1 = (m.x & 0x7FFF0000u) ? v1 : 0.f;
                            v2 = (m.y & 0x7FFFu) ? v2 : 0.f;
                            v3 = (m.y & 0x7FFF0000u) ? v3 : 0.f;
                        }
                        o = (u32x2){pack2(v0, v1), pack2(v2, v3)};
                    }
                    if (staged) *(u32x2*)(opatch + (lane & 31) * OP + j * 32 + q * 8 + (lane >> 5) * 4) = o;
                    else if (ok) *(u32x2*)((uint16_t*)a.out + (size_t)learner * a.out_lstride + (size_t)r * a.ld_out + c) = o;
                }
            }
            if (staged) {
                // (the patch is this wavefront's own, and a wavefront's LDS accesses complete in order)
                constexpr int CPRW = WTC / 8, RPP = 64 / CPRW;  // 16-byte chunks per patch row, rows per pass
                const int rblk = r0 + (wr * MR + i) * 32;
#pragma unroll
                for (int pass = 0; pass < 32 / RPP; ++pass) {
                    const int row = pass * RPP + lane / CPRW, ch = lane % CPRW;
                    const int rr = rblk + row, cc = c0 + wc * WTC + ch * 8;
                    const u32x4 v = *(const u32x4*)(opatch + row * OP + ch * 8);
                    if (rr < a.nR && cc < c_end)
                        *(u32x4*)((uint16_t*)a.out + (size_t)learner * a.out_lstride + (size_t)rr * a.ld_out + cc) = v;
                }
            }
        }
    } else {
        // Update: the master tile is read and written as whole row segments.  Each wavefront passes one
        // 32-row block of its accumulators through a private LDS patch so that a lane ends up with four
        // consecutive columns of a row and 64/(WTC/4) rows are covered per access, WTC*4 contiguous bytes each.
        float* stage = (float*)smem + wave * 32 * SPITCH;
        uint16_t* hbase = a.ws + (size_t)learner * a.ws_lstride;
        uint16_t* lbase = a.wlo + (size_t)learner * a.ws_lstride;
        const int rr = lane / L8_PER_ROW, cc = (lane % L8_PER_ROW) * 8;
        const int c = c0 + wc * WTC + cc;
#pragma unroll
        for (int i = 0; i < MR; ++i) {
            const int rblk = r0 + (wr * MR + i) * 32;
            if (i > 0) __syncthreads();                 // previous patch contents are dead
#pragma unroll
            for (int j = 0; j < MC; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v = {acc[i][j][4 * q + 0], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *(f32x4*)(stage + (lane & 31) * SPITCH + j * 32 + q * 8 + (lane >> 5) * 4) = v;
                }
            __syncthreads();
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                const int r = rblk + it * ROWS_PER_IT + rr;
                const float* gp = stage + (it * ROWS_PER_IT + rr) * SPITCH + cc;
                const f32x4 g0 = *(const f32x4*)gp, g1 = *(const f32x4*)(gp + 4);
                if (a.partial) {
                    if (r < a.nR && c < a.nC) {
                        float* pp = a.partial + ((size_t)learner * a.nR + r) * a.nC + c;
                        *(f32x4*)pp = g0;
                        *(f32x4*)(pp + 4) = g1;
                    }
                    continue;
                }
                if (r < a.nR && c < a.nC) {
                    float step[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
                    if (a.u) {                                  // heavy ball inside the learner
                        f32x4* up = (f32x4*)(a.u + (size_t)learner * a.w_lstride + (size_t)r * a.nC + c);
                        const f32x4 u0 = __builtin_nontemporal_load(up), u1 = __builtin_nontemporal_load(up + 1);
                        const float uo[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) step[e] = a.beta * uo[e] + step[e];
                        __builtin_nontemporal_store((f32x4){step[0], step[1], step[2], step[3]}, up);
                        __builtin_nontemporal_store((f32x4){step[4], step[5], step[6], step[7]}, up + 1);
                    }
                    u32x4 oh, ol;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint32_t b0, b1, h2, l2;
                        split_join2(mhi[i][it][q], mlo[i][it][q], b0, b1);
                        const float w0 = __builtin_bit_cast(float, b0) - a.lr * step[2 * q];
                        const float w1 = __builtin_bit_cast(float, b1) - a.lr * step[2 * q + 1];
                        split_pack2(__builtin_bit_cast(uint32_t, w0), __builtin_bit_cast(uint32_t, w1), h2, l2);
                        oh[q] = h2; ol[q] = l2;
                    }
                    // The hi plane is what the next forward pass reads.  When the hi planes of all learners
                    // fit there, an ordinary store leaves it in the memory-side cache; when they do not, it
                    // would only displace other lines.  The lo plane (and the velocity) is streamed once
                    // per step and always bypasses the cache.
                    if (SHADOW_CACHED) *(u32x4*)(hbase + (size_t)r * a.nC + c) = oh;
                    else __builtin_nontemporal_store(oh, (u32x4*)(hbase + (size_t)r * a.nC + c));
                    __builtin_nontemporal_store(ol, (u32x4*)(lbase + (size_t)r * a.nC + c));
                }
            }
        }
        if (a.partial) {
            if (tile_c == 0 && tid < TR && r0 + tid < a.nR) a.partial_bias[(size_t)learner * a.nR + r0 + tid] = bias_sum;
        } else if (!a.skip_bias && tile_c == 0 && tid < TR && r0 + tid < a.nR) {
            const size_t at = (size_t)learner * a.w_lstride + r0 + tid;
            if (a.ub) { bias_sum = a.beta * a.ub[at] + bias_sum; a.ub[at] = bias_sum; }
            const size_t sat = (size_t)learner * a.ws_lstride + r0 + tid;
            const float b = __builtin_bit_cast(float, split_join(a.bhi[sat], a.blo[sat])) - a.lr * bias_sum;
            a.bhi[sat] = (uint16_t)split_hi(__builtin_bit_cast(uint32_t, b));
            a.blo[sat] = (uint16_t)split_lo(__builtin_bit_cast(uint32_t, b));
        }
        asm volatile("" :: "v"(touched));               // the touched lines' loads are not dead code
    }
}

template <int MODE, int TR, int TC, int WR, int WC, int WK, int BK, bool RT, bool CT, int PIPE, bool SC = false, bool GC = false,
          bool CVR = false, bool CVC = false>
hipError_t launch(Args a, int P, hipStream_t st) {
    a.tiles_c = (a.nC + TC - 1) / TC;
    a.tiles_r = (a.nR + TR - 1) / TR;
    a.total_wg = a.tiles_c * a.tiles_r * P;
    a.chunk = (a.total_wg + 7) / 8;
    dim3 grid(8 * a.chunk);
    constexpr int SMEM = Shape<MODE, TR, TC, WR, WC, WK, BK, RT, CT, PIPE>::SMEM_BYTES;
    static_assert(SMEM <= 160 * 1024, "more LDS than a compute unit has");
    if (SMEM > 64 * 1024) {                     // beyond the default limit: raise it once for this kernel
        static hipError_t raised = hipFuncSetAttribute(
            (const void*)gemm_bf16_kernel<MODE, TR, TC, WR, WC, WK, BK, RT, CT, PIPE, SC, GC, CVR, CVC>,
            hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
        if (raised != hipSuccess) return raised;
    }
    if (PIPE == PIPE_RING && (a.nK % BK != 0 || a.nK > a.R.n_cont || a.nK > a.C.n_cont)) return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_bf16_kernel<MODE, TR, TC, WR, WC, WK, BK, RT, CT, PIPE, SC, GC, CVR, CVC>), grid,
                       dim3(Shape<MODE, TR, TC, WR, WC, WK, BK, RT, CT, PIPE>::THREADS), SMEM, st, a);
    return hipGetLastError();
}

int round8(int x) { return (x + 7) / 8 * 8; }

// Launch shapes: rows x columns of the output tile (_K2: eight wavefronts, two k groups, slices of 128).
enum { T128x128 = 0, T128x64 = 1, T64x128 = 2, T64x64_K2 = 3, T256x128 = 4 };

// Measured on MI355X over the workload shapes (batch 64..256, widths 1024..4096, 8..32 learners):
// with >= 512 tiles of 128x128 the launch fills the chip with the tile that reads LDS least per
// flop; smaller problems are LDS- and barrier-bound per workgroup, and the 64x64 tile with two k
// groups (most wavefronts per compute unit, half as many barriers per k) wins.
int pick_tile(int mode, int nR, int nC, int nK, int P) {
    const long tiles128 = (long)((nR + 127) / 128) * ((nC + 127) / 128) * P;
    // few output columns (convolution channels): a 64-column tile wastes least
    if (nC <= 64 && nR > 64 && tiles128 >= 512) return T128x64;
    if (mode == MODE_FWD) {
        if (nR % 256 == 0 && nK % 64 == 0 && nK >= 128 && (long)(nR / 256) * ((nC + 127) / 128) * P >= 192) return T256x128;
        if (nR <= 64) return (long)((nC + 127) / 128) * P >= 512 ? T64x128 : T64x64_K2;
        return tiles128 >= 512 ? T128x128 : T64x64_K2;
    }
    // backward-data, measured at the 4096-wide layers: 128x128 95 us against 119 us for 128x64 (batch 256),
    // 64x128 222 us against 249 us for 64x64 (batch 64)
    if (nR <= 64) return (long)((nC + 127) / 128) * P >= 512 ? T64x128 : T64x64_K2;
    if (tiles128 >= 512) return T128x128;
    return tiles128 >= 256 ? T128x64 : T64x64_K2;
}

template <int MODE, bool RT, bool CT>
hipError_t launch_tiled(const Args& a, int P, int tile, hipStream_t st) {
    switch (tile) {
        case T128x128:
            // forward: slices of 64 straight into LDS (rows of 128 bytes); measured 10 % faster than staging
            // through registers at the 4096-wide layers
            if constexpr (MODE == MODE_FWD) return launch<MODE, 128, 128, 2, 2, 1, 64, RT, CT, PIPE_DMA>(a, P, st);
            else return launch<MODE, 128, 128, 2, 2, 1, 64, RT, CT, PIPE_PLAIN>(a, P, st);
        case T256x128:
            if constexpr (MODE == MODE_FWD) return launch<MODE, 256, 128, 2, 2, 1, 64, RT, CT, PIPE_RING>(a, P, st);
            else return hipErrorInvalidValue;
        case T128x64:  return launch<MODE, 128, 64, 2, 2, 1, 64, RT, CT, PIPE_PLAIN>(a, P, st);
        case T64x128:  return launch<MODE, 64, 128, 2, 2, 1, 64, RT, CT, PIPE_PLAIN>(a, P, st);
        default:
            // forward: slices of 128 loaded straight into LDS (measured 26 against 30 us for layer 1 of the
            // CIFAR-MLP workload); backward-data (weights read through the transpose path): slices of 64,
            // double-buffered LDS filled from registers
            if constexpr (MODE == MODE_FWD) return launch<MODE, 64, 64, 2, 2, 2, 128, RT, CT, PIPE_DMA>(a, P, st);
            else return launch<MODE, 64, 64, 2, 2, 2, 64, RT, CT, PIPE_LDS2>(a, P, st);
    }
}

}  // namespace

hipError_t bf16_forward(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.in, c.gather ? 0 : c.in_stride, c.ld_in, c.gather, c.gather_stride, c.B, c.d_in};
    a.C = {c.ws, c.shared_w ? 0 : c.ws_stride, c.d_in, nullptr, 0, c.d_out, c.d_in};
    a.nR = c.B; a.nC = c.d_out; a.nK = c.d_in;
    a.bias_hi = c.bhi; a.bias_lo = c.blo; a.bias_lstride = c.ws_stride;
    a.out = c.out; a.out_lstride = c.out_stride; a.ld_out = c.ld_out; a.relu = c.relu;
    a.c_stream = !c.shadow_cached && !c.shared_w;
    return launch_tiled<MODE_FWD, false, false>(a, c.P, pick_tile(MODE_FWD, a.nR, a.nC, a.nK, c.P), st);
}

hipError_t bf16_backward_data(const LayerCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.dz, c.dz_stride, c.ld_dz, nullptr, 0, c.B, round8(c.d_out)};
    a.C = {c.ws, c.shared_w ? 0 : c.ws_stride, c.d_in, nullptr, 0, c.d_out, c.d_in};      // memory row = k: Cm(c, k) = W[k][c]
    a.nR = c.B; a.nC = c.d_in; a.nK = c.d_out;
    a.act_prev = (const uint16_t*)c.in; a.act_lstride = c.in_stride; a.ld_act = c.ld_in;
    a.out = c.dz_prev; a.out_lstride = c.dz_prev_stride; a.ld_out = c.ld_in;
    if (c.bwd_raw) { a.epi = EPI_RAW; a.act_prev = nullptr; }
    return launch_tiled<MODE_BWD, false, true>(a, c.P, pick_tile(MODE_BWD, a.nR, a.nC, a.nK, c.P), st);
}

hipError_t bf16_update(const LayerCall& c, hipStream_t st) {
    Args a = {};
    int rows = c.rows ? c.rows : c.B;
    int P = c.P;
    size_t r_stride = c.dz_stride, c_stride = c.gather ? 0 : c.in_stride;
    if (c.partial) {                               // ranges of rows as separate "learners" (rows are contiguous per learner)
        if (c.gather || c.splits < 1 || rows % c.splits != 0 || c.dz_stride != (size_t)rows * c.ld_dz ||
            c.in_stride != (size_t)rows * c.ld_in) return hipErrorInvalidValue;
        rows /= c.splits; P *= c.splits;
        r_stride = (size_t)rows * c.ld_dz; c_stride = (size_t)rows * c.ld_in;
        a.partial = c.partial; a.partial_bias = c.partial_bias;
    }
    a.R = {(const uint16_t*)c.dz, r_stride, c.ld_dz, nullptr, 0, rows, c.ld_dz};         // memory row = k: R(r, k) = dZ[k][r]
    a.C = {(const uint16_t*)c.in, c_stride, c.ld_in, c.gather, c.gather_stride, rows, c.d_in};
    a.nR = c.d_out; a.nC = c.d_in; a.nK = rows;
    a.skip_bias = c.skip_bias;
    a.ws = c.ws; a.wlo = c.wlo; a.ws_lstride = c.ws_stride; a.bhi = c.bhi; a.blo = c.blo; a.w_lstride = c.w_stride;
    a.lr = c.lr; a.u = c.u; a.ub = c.ub; a.beta = c.beta;
    a.next_gather = c.gather ? c.next_gather : nullptr;
    // Tile shapes from measured sweeps (whole rounds, same box): wavefront tiles of 32x64 in both regimes
    // (128-byte row segments per plane), as 128x64 where the bf16 planes stay in the memory-side
    // cache (CIFAR-MLP) and as 64x128 where they stream (the 4096-wide workloads with batches up to 128).
    if (c.shadow_cached) {
        if (c.gather) return launch<MODE_UPD, 128, 64, 4, 1, 1, 64, true, true, PIPE_PLAIN, true, true>(a, P, st);
        return launch<MODE_UPD, 128, 64, 4, 1, 1, 64, true, true, PIPE_PLAIN, true, false>(a, P, st);
    }
    if (rows > 128) {
        // Long contractions: per output tile the two operands (read out of the L2 cache, B rows each) weigh as
        // much as the master tile itself, and a compute unit can only pull so many bytes per clock; a
        // 128x128 tile reads a third less of them per weight (large: 15.0 -> 14.5 ms per round).
        if (c.gather) return launch<MODE_UPD, 128, 128, 2, 2, 1, 64, true, true, PIPE_PLAIN, false, true>(a, P, st);
        return launch<MODE_UPD, 128, 128, 2, 2, 1, 64, true, true, PIPE_PLAIN, false, false>(a, P, st);
    }
    if (c.gather) return launch<MODE_UPD, 64, 128, 2, 2, 1, 64, true, true, PIPE_PLAIN, false, true>(a, P, st);
    return launch<MODE_UPD, 64, 128, 2, 2, 1, 64, true, true, PIPE_PLAIN, false, false>(a, P, st);
}

// ---- 3x3 convolutions on the implicit patch matrix (no im2col): see ConvCall in kavg_internal.h ----
namespace {
bool conv_call_ok(const ConvCall& c) {
    return c.P >= 1 && c.B >= 1 && c.H >= 1 && c.W >= 1 && c.c_in >= 8 && c.c_in % 8 == 0 && c.c_out >= 8 && c.c_out % 8 == 0 &&
           c.c_in <= 4096 && c.c_out <= 4096 && (long)c.B * c.H * c.W < (1L << 30) && c.H * c.W < (1 << 14) * 4 && c.W < (1 << 14);
}
}  // namespace

hipError_t bf16_conv_forward(const ConvCall& c, hipStream_t st) {
    if (!conv_call_ok(c) || c.H * c.W >= (1 << 14)) return hipErrorInvalidValue;
    const int rows = c.B * c.H * c.W;
    Args a = {};
    a.R = {(const uint16_t*)c.in, (size_t)rows * c.c_in, c.c_in, nullptr, 0, rows, 9 * c.c_in};
    operand_conv(a.R, c.c_in, c.H, c.W, +1);
    a.C = {c.ws, c.ws_stride, 9 * c.c_in, nullptr, 0, c.c_out, 9 * c.c_in};
    a.nR = rows; a.nC = c.c_out; a.nK = 9 * c.c_in;
    a.bias_hi = c.bhi; a.bias_lo = c.blo; a.bias_lstride = c.ws_stride;
    a.out = c.out; a.out_lstride = (size_t)rows * c.c_out; a.ld_out = c.c_out; a.relu = 1;
    if (c.c_out <= 64) return launch<MODE_FWD, 128, 64, 2, 2, 1, 64, false, false, PIPE_PLAIN, false, false, true, false>(a, c.P, st);
    return launch<MODE_FWD, 128, 128, 2, 2, 1, 64, false, false, PIPE_PLAIN, false, false, true, false>(a, c.P, st);
}

// dZ_in[n,h,w,ci] = [act_in > 0] * sum_{tap,o} dZ[n, h-(kh-1), w-(kw-1), o] * Wrot[(tap,o)][ci]
hipError_t bf16_conv_backward_data(const ConvCall& c, hipStream_t st) {
    if (!conv_call_ok(c) || c.H * c.W >= (1 << 14)) return hipErrorInvalidValue;
    const int rows = c.B * c.H * c.W;
    Args a = {};
    a.R = {(const uint16_t*)c.dz, (size_t)rows * c.c_out, c.c_out, nullptr, 0, rows, 9 * c.c_out};
    operand_conv(a.R, c.c_out, c.H, c.W, -1);
    a.C = {c.wrot, c.wrot_stride, c.c_in, nullptr, 0, 9 * c.c_out, c.c_in};        // memory row = k = (tap, o)
    a.nR = rows; a.nC = c.c_in; a.nK = 9 * c.c_out;
    a.act_prev = (const uint16_t*)c.in; a.act_lstride = (size_t)rows * c.c_in; a.ld_act = c.c_in;
    a.out = c.dz_in; a.out_lstride = (size_t)rows * c.c_in; a.ld_out = c.c_in;
    if (c.c_in <= 64) return launch<MODE_BWD, 128, 64, 2, 2, 1, 64, false, true, PIPE_PLAIN, false, false, true, false>(a, c.P, st);
    return launch<MODE_BWD, 128, 128, 2, 2, 1, 64, false, true, PIPE_PLAIN, false, false, true, false>(a, c.P, st);
}

// fp32 partial weight gradients of `splits` ranges of positions per learner (conv_step_kernel adds them)
hipError_t bf16_conv_update_partial(const ConvCall& c, hipStream_t st) {
    const int rows = c.B * c.H * c.W;
    if (!conv_call_ok(c) || c.H * c.W >= (1 << 14) || c.splits < 1 || rows % c.splits != 0 || !c.partial || !c.partial_bias)
        return hipErrorInvalidValue;
    const int range = rows / c.splits;
    Args a = {};
    a.R = {(const uint16_t*)c.dz, (size_t)range * c.c_out, c.c_out, nullptr, 0, range, c.c_out};      // memory row = k: R(r, k) = dZ[k][r]
    a.C = {(const uint16_t*)c.in, (size_t)rows * c.c_in, c.c_in, nullptr, 0, range, 9 * c.c_in};
    operand_conv(a.C, c.c_in, c.H, c.W, +1);
    a.cv_splits = c.splits;
    a.nR = c.c_out; a.nC = 9 * c.c_in; a.nK = range;
    a.ws = c.ws; a.wlo = c.wlo; a.ws_lstride = c.ws_stride; a.bhi = (uint16_t*)c.bhi; a.blo = (uint16_t*)c.blo; a.w_lstride = c.ws_stride;
    a.partial = c.partial; a.partial_bias = c.partial_bias;
    return launch<MODE_UPD, 128, 64, 4, 1, 1, 64, true, true, PIPE_PLAIN, true, false, false, true>(a, c.P * c.splits, st);
}

hipError_t bf16_gram(const GramCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.R, c.R_gather ? 0 : c.R_stride, c.ldR, c.R_gather, c.R_gstride, c.nR, round8(c.nK)};
    a.C = {(const uint16_t*)c.C, c.C_gather ? 0 : c.C_stride, c.ldC, c.C_gather, c.C_gstride, c.nC, round8(c.nK)};
    a.nR = c.nR; a.nC = c.nC; a.nK = c.nK;
    a.out = c.out; a.out_lstride = c.out_stride; a.ld_out = c.ld_out; a.relu = 1;
    a.epi = EPI_GRAM; a.alpha = c.alpha;
    return launch_tiled<MODE_FWD, false, false>(a, c.P, pick_tile(MODE_FWD, a.nR, a.nC, a.nK, c.P), st);
}

hipError_t bf16_apply(const ApplyCall& c, hipStream_t st) {
    Args a = {};
    a.R = {(const uint16_t*)c.S, c.S_stride, c.ldS, nullptr, 0, c.nR, round8(c.nK)};
    a.C = {(const uint16_t*)c.M, c.M_stride, c.ldM, nullptr, 0, c.nK, c.nC_cont};      // memory row = k
    a.nR = c.nR; a.nC = c.nC; a.nK = c.nK;
    a.base = c.base; a.base_lstride = c.base_stride; a.ld_base = c.ld_base;
    a.out = c.out; a.out_lstride = c.out_stride; a.ld_out = c.ld_out;
    if (c.epi == KAVG_APPLY_MASK) {
        a.epi = EPI_STD; a.act_prev = (const uint16_t*)c.act; a.act_lstride = c.act_stride; a.ld_act = c.ld_act;
    } else {
        a.epi = c.epi == KAVG_APPLY_RELU ? EPI_RELU : EPI_LOGITS;
    }
    return launch_tiled<MODE_BWD, false, true>(a, c.P, pick_tile(MODE_BWD, a.nR, a.nC, a.nK, c.P), st);
}

namespace {
// one lane per (learner, unit): the column of dZ is summed over the step's rows in ascending order
__global__ void __launch_bounds__(256) bias_step_kernel(uint16_t* bhi, uint16_t* blo, size_t b_stride, const uint16_t* dz,
                                                        int ld_dz, size_t dz_stride, int rows, int d, float lr) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int learner = blockIdx.y;
    if (c >= d) return;
    const uint16_t* p = dz + (size_t)learner * dz_stride + c;
    float sum = 0.f;
#pragma unroll 8
    for (int r = 0; r < rows; ++r) sum += bf16_to_f32(p[(size_t)r * ld_dz]);
    const size_t at = (size_t)learner * b_stride + c;
    const float b = __builtin_bit_cast(float, split_join(bhi[at], blo[at])) - lr * sum;
    bhi[at] = (uint16_t)split_hi(__builtin_bit_cast(uint32_t, b));
    blo[at] = (uint16_t)split_lo(__builtin_bit_cast(uint32_t, b));
}
}  // namespace

hipError_t launch_bias_step(uint16_t* bhi, uint16_t* blo, size_t b_stride, const void* dz, int ld_dz,
                            size_t dz_stride, int P, int rows, int d, float lr, hipStream_t st) {
    hipLaunchKernelGGL(bias_step_kernel, dim3((d + 255) / 256, P), dim3(256), 0, st, bhi, blo, b_stride,
                       (const uint16_t*)dz, ld_dz, dz_stride, rows, d, lr);
    return hipGetLastError();
}

}  // namespace kavg
