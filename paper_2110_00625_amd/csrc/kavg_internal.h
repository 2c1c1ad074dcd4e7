// Internal launch interface between the C boundary (kavg_api.hip) and the
// kernel translation units.  Every launcher validates nothing: the boundary
// has already checked shapes; launchers only derive grids from them.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/kavg.h"

namespace kavg {

// ---- minibatch index stream (Algorithm 1: "randomly sample a mini-batch") ----
// idx[P][K][B], entry (j,k,s) = SplitMix64 draw with counter j*2^40 + (t0+k)*2^16 + s, mod N.
hipError_t launch_index_stream(int32_t* idx, int P, int K, int B, uint64_t seed,
                               uint32_t t0, uint32_t N, hipStream_t st);
// copy caller indices into idx, clamping into [0,N) and raising *flag on any entry outside
hipError_t launch_index_import(int32_t* idx, const int32_t* user, size_t count, uint32_t N,
                               int* flag, hipStream_t st);
// raise *flag if any label lies outside [0,C)
hipError_t launch_label_check(const int32_t* y, size_t N, int C, int* flag, hipStream_t st);

// ---- meta level (Algorithm 1: a, d, v, w~, restart of the learners) ----
// shadow_cached: write the shadows with ordinary stores (they fit in the memory-side cache) or streaming ones
hipError_t launch_meta_update(float* w_tilde, float* v, float* reps, size_t stride,
                              uint16_t* shadow, size_t sstride, int P, size_t n, float mu,
                              int shadow_cached, hipStream_t st);
// the same step on replicas stored as hi / lo planes (split.h), [P][stride] 16-bit each
hipError_t launch_meta_update_split(float* w_tilde, float* v, uint16_t* hi, uint16_t* lo, size_t stride,
                                    int P, size_t n, float mu, int hi_cached, hipStream_t st);
hipError_t launch_broadcast_split(const float* w_tilde, uint16_t* hi, uint16_t* lo, size_t stride,
                                  int P, size_t n, hipStream_t st);
// w^j <- w~ for all j (and shadows): the "set w^j = w~_n" of the first round
hipError_t launch_broadcast(const float* w_tilde, float* reps, size_t stride,
                            uint16_t* shadow, size_t sstride, int P, size_t n, hipStream_t st);

// ---- loss and its gradient ----
// logits [P][B][ldz] fp32; labels y[idx[j][m]]; dz: learner j's B rows of ldz at dz + j*dz_learner_stride
// (fp32 or bf16), pad columns zeroed; rowloss [P][B].  dZ = (softmax - onehot)/B.
hipError_t launch_softmax_ce(const float* logits, int ldz, int C, const int32_t* y,
                             const int32_t* idx, long idx_learner_stride, int B, int P,
                             void* dz, long dz_learner_stride, int dz_bf16, float* rowloss, hipStream_t st);
// losses[k][j] = mean_m rowloss[k][j][m]
hipError_t launch_loss_mean(const float* rowloss, float* losses, int KP, int B, hipStream_t st);

// ---- per-learner dense layers ----
struct LayerCall {
    int P, B;              // learners, rows per learner
    int d_in, d_out;       // layer shape: W [d_out][d_in]
    // parameters, fp32 mode: learner j's W at w + j*w_stride, bias at b + j*w_stride
    float* w;       size_t w_stride;      // weights of this layer (first learner); null in bf16 mode
    float* b;                               // bias of this layer (same stride); null in bf16 mode
    // parameters, bf16 mode: every fp32 master value is stored as two 16-bit planes (split.h):
    // ws = the bf16 values the products read, wlo = the remainders; same for the bias
    uint16_t* ws;   size_t ws_stride;     // hi plane of the weights (first learner), else null
    uint16_t* wlo;                          // lo plane of the weights (stride ws_stride)
    uint16_t* bhi;  uint16_t* blo;          // hi / lo planes of the bias (stride ws_stride)
    int shadow_cached;                    // updates access the bf16 (hi) plane with ordinary (1) or streaming (0) loads / stores
    // activations entering the layer: [P][B][ld_in]; or, with gather != null, rows X[gather[j][m]]
    const void* in; int ld_in; size_t in_stride;
    const int32_t* gather; long gather_stride;
    // update of the first layer only: rows the NEXT local step will gather (same layout as gather),
    // or null.  The kernel touches them so that the next forward pass finds them in cache.
    const int32_t* next_gather;
    // activations leaving the layer / logits: [P][B][ld_out]
    void* out; int ld_out; size_t out_stride;
    // gradient w.r.t. this layer's pre-activation: [P][B][ld_dz]
    const void* dz; int ld_dz; size_t dz_stride;
    // gradient w.r.t. the previous layer's pre-activation (output of backward-data): [P][B][ld_in]
    void* dz_prev; size_t dz_prev_stride;
    int relu;              // forward: apply ReLU (hidden layer) / keep fp32 logits (last layer)
    void* scratch;         // fp32 forward: partial tiles of a split contraction (see f32_forward_plan)
    float lr;
    // learner-level momentum: velocity of this layer's weights (learner 0; stride w_stride) and of its
    // bias, null when off.  u <- beta u + g, w <- w - lr u.
    float* u; float* ub; float beta;
    // deferred weight updates (bf16 mode):
    int shared_w;          // forward / backward-data: every learner's stored weights equal learner 0's (round start): read those
    int bwd_raw;           // backward-data: write the unmasked fp32 product to dz_prev instead of the masked bf16 one
    int rows;              // update: rows of dz / in to contract over (0: B) -- the steps since the last refresh
    int skip_bias;         // update: leave the bias alone (it is stepped after every local step)
    // update with fp32 partial outputs instead of a step on the master (long contractions split over
    // `splits` ranges of rows that run as separate workgroups): partial [P*splits][d_out][d_in],
    // partial_bias [P*splits][d_out]; B must be a multiple of splits
    float* partial; float* partial_bias; int splits;
};

// ---- deferred weight updates (Algorithm 1: every local step adds a rank-B term -lr dZ^T A to the
// learner's weights; between two refreshes of the stored replica the products use the stored
// weights plus those terms, W_k x = W_0 x - lr sum_i dZ_i^T (A_i x)) ----
// out[j][r][c] = bf16(alpha * sum_k R[j][r][k] * C[j][c][k]); R, C bf16 with k contiguous; either may be
// gathered rows of a shared matrix (stride 0, gather != null)
struct GramCall {
    int P, nR, nC, nK;
    const void* R; int ldR; size_t R_stride; const int32_t* R_gather; long R_gstride;
    const void* C; int ldC; size_t C_stride; const int32_t* C_gather; long C_gstride;
    void* out; int ld_out; size_t out_stride;
    float alpha;
};
// out[j][r][c] = epi(base[j][r][c] + sum_h S[j][r][h] * M[j][h][c]); S bf16 [nR][ldS], M bf16 [nK][ldM],
// base fp32.  epi: KAVG_APPLY_RELU -> bf16 relu; KAVG_APPLY_LOGITS -> fp32; KAVG_APPLY_MASK -> bf16,
// zero where act[j][r][c] <= 0.  nC_cont: readable columns of M (multiple of 8, >= nC).
enum { KAVG_APPLY_RELU = 0, KAVG_APPLY_LOGITS = 1, KAVG_APPLY_MASK = 2 };
struct ApplyCall {
    int P, nR, nC, nC_cont, nK;
    const void* S; int ldS; size_t S_stride;
    const void* M; int ldM; size_t M_stride;
    const float* base; int ld_base; size_t base_stride;
    int epi;
    const void* act; int ld_act; size_t act_stride;
    void* out; int ld_out; size_t out_stride;
};
hipError_t bf16_gram(const GramCall& c, hipStream_t st);
hipError_t bf16_apply(const ApplyCall& c, hipStream_t st);
// b[j][c] -= lr * sum_r dz[j][r][c] on bias planes (split.h); dz bf16 [P][rows][ld_dz]
hipError_t launch_bias_step(uint16_t* bhi, uint16_t* blo, size_t b_stride, const void* dz, int ld_dz,
                            size_t dz_stride, int P, int rows, int d, float lr, hipStream_t st);

// fp32 path
// splits of the forward contraction of a layer and the contraction range of each; shapes only
int f32_forward_plan(int P, int B, int d_in, int d_out, int* chunk_out);
hipError_t f32_forward(const LayerCall& c, hipStream_t st);
hipError_t f32_backward_data(const LayerCall& c, hipStream_t st);
hipError_t f32_update(const LayerCall& c, hipStream_t st);
// bf16 MFMA path
hipError_t bf16_forward(const LayerCall& c, hipStream_t st);
hipError_t bf16_backward_data(const LayerCall& c, hipStream_t st);
hipError_t bf16_update(const LayerCall& c, hipStream_t st);

// ---- classifier head for small class counts (last layer: forward + loss + data gradient, then update) ----
bool head_supported(int C);
// idx: this step's indices of learner 0, idx_lstride elements between learners
hipError_t head_forward_backward(const LayerCall& c, const int32_t* y, const int32_t* idx, long idx_lstride,
                                 float* rowloss, int bf16, hipStream_t st);
hipError_t head_update(const LayerCall& c, const int32_t* idx, long idx_lstride, int bf16, hipStream_t st);

// ---- convolutional layers (conv.hip): 3x3, stride 1, zero padding 1, channels-last bf16 images ----
// patches[j][(n,h,w)][(kh,kw,c)] from images in[j][n][h][w][c] (or, with gather, from rows gather[j*gstride+n] of a shared set)
hipError_t launch_im2col(const void* in, size_t in_lstride, const int32_t* gather, long gstride, void* patches,
                         int P, int B, int H, int W, int c, hipStream_t st);
// fp32 per-(position, tap, channel) data gradients folded back onto the image, masked by act > 0, bf16
hipError_t launch_col2im_mask(const float* draw, const void* act, void* dprev, int P, int B, int H, int W, int c,
                              hipStream_t st);
hipError_t launch_pool_forward(const void* act, void* pooled, int P, int B, int HW, int c, hipStream_t st);
hipError_t launch_pool_backward(const void* dpool, const void* act, void* dz, int P, int B, int HW, int c, hipStream_t st);
// master -= lr * (sum of the S fp32 partial gradients), weights [n_w] and bias [n_b] of one layer, planes of split.h
hipError_t launch_conv_step(uint16_t* whi, uint16_t* wlo, uint16_t* bhi, uint16_t* blo, size_t lstride, const float* partial,
                            const float* pbias, int P, int S, int n_w, int n_b, float lr, hipStream_t st);

// ---- 3x3 convolution (stride 1, zero padding 1) on channels-last images [P][B][H][W][c], the patch matrix formed
// inside the operand loaders of the MFMA kernel (no im2col buffer).  Weights [c_out][3][3][c_in] as two planes.
struct ConvCall {
    int P, B, H, W, c_in, c_out;
    uint16_t* ws; uint16_t* wlo; size_t ws_stride;     // hi / lo planes of the weights (first learner), learner stride
    const uint16_t* bhi; const uint16_t* blo;          // planes of the bias (same stride)
    const void* in;                                    // input images (bf16): forward and update operand, backward's ReLU mask
    void* out;                                         // forward: relu(conv + bias), bf16
    const void* dz;                                    // gradient w.r.t. this layer's pre-activation, bf16 images of c_out channels
    void* dz_in;                                       // backward: gradient w.r.t. the input layer's pre-activation (masked by in > 0)
    const uint16_t* wrot; size_t wrot_stride;          // backward: weights as [(tap, o)][c_in] (launch_rotate_weights), learner stride
    float* partial; float* partial_bias; int splits;   // update: fp32 partials [P*splits][c_out][9 c_in] / [P*splits][c_out]
};
hipError_t bf16_conv_forward(const ConvCall& c, hipStream_t st);
hipError_t bf16_conv_backward_data(const ConvCall& c, hipStream_t st);
hipError_t bf16_conv_update_partial(const ConvCall& c, hipStream_t st);
// wrot[j][(tap*c_out + o)*c_in + ci] = whi[j][(o*9 + tap)*c_in + ci]
hipError_t launch_rotate_weights(const uint16_t* whi, size_t w_lstride, uint16_t* wrot, size_t wrot_lstride, int P, int c_out,
                                 int c_in, hipStream_t st);

// ---- all K local steps of a small fp32 model in one launch (fused_small.hip) ----
struct FusedSmallCall {
    int P, K, B, d0, d1, C;            // learners, steps, rows; model d0 - d1 - C (one hidden layer)
    float* reps; size_t rep_stride;    // fp32 replicas; offsets of W_1, b_1, W_2, b_2 inside one
    size_t w1_off, b1_off, w2_off, b2_off;
    const float* X; const int32_t* y;  // data set [N][d0], labels
    int32_t* idx;                      // [P][K][B]: read (generate_idx = 0) or written (1: draws of the index stream)
    int generate_idx; uint64_t seed; uint32_t t0, N;
    uint64_t* partial;                 // scratch of fused_small_scratch_bytes: (value, tag) words, zero before the first launch
    uint32_t* hints;                   // ... followed by the hint words (partial + fused_small_partial_words)
    uint32_t tag0;                     // tags of this launch are tag0 + 1 .. tag0 + K; never reused on the same scratch
    int* err;                          // set to 1 when a reader ran out of polls
    float* losses;                     // [K][P] mean loss per step and learner
    float lr; unsigned spin_limit;
    int compute_units;                 // of the device (decides whether two workgroups share a column chunk)
};
int fused_small_chunks(int d0);
bool fused_small_shape_ok(int P, int K, int B, int d0, int d1, int C, int compute_units);
size_t fused_small_scratch_bytes(int P, int d0);
size_t fused_small_partial_words(int P, int d0);
hipError_t launch_fused_small(const FusedSmallCall& c, hipStream_t st);

// ---- device ceilings (measurement aid) ----
// one launch of the probe `kind` (KAVG_PROBE_*); *work_out = bytes moved or flops done by it
hipError_t launch_probe(int kind, void* a, void* b, size_t bytes, int iters, float* sink, hipStream_t st,
                        double* work_out);

}  // namespace kavg
