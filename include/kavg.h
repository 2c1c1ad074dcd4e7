/*
 * kavg.h -- C boundary of the M-AVG hot path (K-step averaging SGD with block
 * momentum) for one AMD MI355X (gfx950).
 *
 * The library runs Algorithm 1 of the paper (Section 2, "M-AVG Algorithm") on an
 * MLP with ReLU hidden layers and softmax cross-entropy, the instance of the
 * objective F(w) = (1/n) sum_i loss(y_i, f(x_i, w)) stated in Section 2:
 *
 *   every round n:   each of P learners starts from the global model w~_n and
 *                    takes K minibatch-SGD steps  w <- w - (lr/B) sum_s grad F(w; xi_s)
 *                    on its own replica                       (kavg_local_steps)
 *                    a = (1/P) sum_j w^j;  d = a - w~_n;  v <- mu v + d;
 *                    w~_{n+1} = w~_n + v;  every w^j <- w~_{n+1}   (kavg_meta_update)
 *
 * All P replicas live in device memory of one GPU; every step runs in HIP
 * kernels of this library.  There is no CPU fallback.
 *
 * Conventions
 *  - Every function returns an int status (KAVG_OK = 0).  Nothing throws,
 *    aborts or prints.  kavg_last_error() returns a text for the last failure
 *    on that context (owned by the context, valid until the next call on it).
 *  - "dev" pointers are device memory of the current HIP device, "host"
 *    pointers are ordinary host memory.  The library never allocates or frees
 *    device memory: the caller passes one workspace block and keeps it, the
 *    data set and any index array alive until kavg_destroy.
 *  - Work is enqueued on the HIP stream given to kavg_init (NULL = the default
 *    stream).  kavg_local_steps and kavg_meta_update return without waiting;
 *    the functions that copy to the host wait for the stream.
 *  - A context is not thread safe.
 *
 * Flat parameter layout (what "n floats" means everywhere): for l = 1..L the
 * weight matrix W_l row-major [d_l][d_{l-1}] (output-major), then the bias
 * b_l [d_l].  n = sum_l (d_l d_{l-1} + d_l).
 *
 * dtype
 *  KAVG_FP32: every tensor and every product in fp32.
 *  KAVG_BF16: operands of every matrix product are bf16: the data set (given
 *    as bf16), each replica's weights rounded to bf16 (nearest, ties away from
 *    zero), the stored hidden activations and the back-propagated dZ_l (nearest,
 *    ties to even).  Accumulation is fp32; logits, softmax, loss, biases, the
 *    learners' master parameters, the SGD update and the whole meta step are
 *    fp32.  A learner's fp32 parameters are stored as two 16-bit planes: the
 *    bf16 value the products read, and the low 16 bits of the fp32 pattern;
 *    together they are the exact fp32 value (kavg_replica joins them), so the
 *    products' operand is half of the master rather than a copy beside it.
 *    Requires d_0..d_{L-1} to be multiples of 8.
 */
#ifndef KAVG_H
#define KAVG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KAVG_OK      0
#define KAVG_EINVAL  1   /* bad argument                              */
#define KAVG_ENOMEM  2   /* workspace too small                       */
#define KAVG_EDEVICE 3   /* a HIP call failed                         */
#define KAVG_ESTATE  4   /* call order misuse (e.g. no data set yet)  */

#define KAVG_FP32 0
#define KAVG_BF16 1

typedef struct kavg_ctx kavg_ctx;

/* n for an MLP with n_layers weight matrices; dims has n_layers+1 entries
 * d_0..d_L.  Returns 0 on bad arguments. */
size_t kavg_num_params(int n_layers, const int* dims);

/* Bytes of device workspace kavg_init needs for this configuration (global
 * model, momentum buffer, P replicas (4 bytes per parameter in either mode), index stream, activations,
 * back-propagated gradients, losses).  Returns 0 on bad arguments. */
size_t kavg_workspace_bytes(int P, int K, int B, int n_layers, const int* dims, int dtype);

/* Create a context.  Hyper-parameters are those of Algorithm 1: P learners, K
 * local steps per round, per-learner minibatch B, step size lr >= 0 (gamma_n =
 * eta_n, fixed), block momentum mu in [0,1) (Theorem 1's range).
 * index_seed seeds the minibatch index stream (see kavg_set_indices).
 * workspace_dev: device block of at least kavg_workspace_bytes(...) bytes,
 * 256-byte aligned, BORROWED until kavg_destroy.  hip_stream: a hipStream_t,
 * BORROWED (NULL = default stream).
 * Errors: KAVG_EINVAL (P,K,B < 1, P or the step count beyond 2^24, B > 65536,
 * lr < 0, mu outside [0,1), n_layers < 1, a dim < 1, dims not multiples of 8
 * with KAVG_BF16, unknown dtype, null pointers, misaligned workspace),
 * KAVG_ENOMEM (workspace_bytes too small). */
int kavg_init(kavg_ctx** out, int P, int K, float lr, float mu,
              int n_layers, const int* dims, int B, int dtype, uint64_t index_seed,
              void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* The learner of Section 4's convolutional workloads (the paper trains CNNs on image sets): F is a
 * stack of n_conv 3x3 convolutions (stride 1, zero padding 1, each followed by ReLU) on H x W
 * channels-last images, the mean over the H*W positions, and then the MLP dims[0..n_layers] with
 * dims[0] == channels[n_conv]; everything else (Algorithm 1's local steps, averaging, block
 * momentum, index stream) is kavg_init's.  KAVG_BF16 arithmetic only.
 * channels[0..n_conv]: input channels, then each convolution's output channels, all multiples of 8
 * (pad the input images with zero channels).  The flat parameter vector holds, per convolution,
 * W [c_out][3][3][c_in] (row-major; tap (kh,kw) reads input pixel (h+kh-1, w+kw-1)) and then its bias
 * [c_out]; the MLP's layers follow in kavg_init's order.  kavg_set_data takes X [N][H][W][channels[0]]
 * bf16.  kavg_set_learner_momentum and kavg_set_refresh are refused on such a context.
 * kavg_num_params_conv / kavg_workspace_bytes_conv: length of the flat vector / bytes of workspace,
 * 0 for a configuration kavg_init_conv would refuse.
 * Errors: as kavg_init, plus KAVG_EINVAL for H or W outside [1,4096], n_conv outside [1,63], a
 * channel count that is not a multiple of 8 in [8,2048], B*H*W >= 2^30, dims[0] != channels[n_conv]. */
size_t kavg_num_params_conv(int H, int W, int n_conv, const int* channels, int n_layers, const int* dims);
size_t kavg_workspace_bytes_conv(int P, int K, int B, int H, int W, int n_conv, const int* channels,
                                 int n_layers, const int* dims);
int kavg_init_conv(kavg_ctx** out, int P, int K, float lr, float mu, int H, int W, int n_conv,
                   const int* channels, int n_layers, const int* dims, int B, uint64_t index_seed,
                   void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* kavg_init for callers that cannot allocate device memory (code running under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the context works in a block of
 * KAVG_STATIC_WORKSPACE_BYTES that lives inside the library's device image (one copy per GPU, held
 * until the process ends) instead of a caller workspace.  Neither this call nor any later call on
 * the context allocates or frees device memory.  Everything else is kavg_init: same arguments,
 * same kernels, same results; data set, index array and velocity block are still the caller's.
 * The block keeps whatever the previous context left in it; every piece a context reads is
 * written by it first (the range flag is cleared here, the rest by kavg_set_params / the kernels).
 * One context per device may use the block at a time: a second kavg_init_static on the same
 * device before kavg_destroy of the first returns KAVG_ESTATE (two contexts would race on it).
 * Errors: as kavg_init, plus KAVG_ENOMEM when kavg_workspace_bytes(...) exceeds
 * KAVG_STATIC_WORKSPACE_BYTES (checked before any device call), KAVG_EDEVICE when the block's
 * address cannot be obtained. */
#define KAVG_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
int kavg_init_static(kavg_ctx** out, int P, int K, float lr, float mu,
                     int n_layers, const int* dims, int B, int dtype, uint64_t index_seed,
                     void* hip_stream);

/* "initialize w~_1; v <- 0" of Algorithm 1, and "set w^j = w~_1": copies n
 * floats from w0_host into the global model, zeroes the momentum buffer,
 * writes every replica, resets round and step counters. */
int kavg_set_params(kavg_ctx* ctx, const float* w0_host);

/* Resume: global model w and momentum v (host, n floats each), round counter;
 * replicas are rebroadcast from w; the local step counter becomes round*K. */
int kavg_set_state(kavg_ctx* ctx, const float* w_host, const float* v_host, uint64_t round);

/* The data set {(x_i, y_i)}: X_dev row-major [N][d_0], fp32 for KAVG_FP32 and
 * bf16 (16-bit patterns) for KAVG_BF16; y_dev [N] class ids in [0, d_L).
 * BORROWED.  N in [1, 2^31). */
int kavg_set_data(kavg_ctx* ctx, const void* X_dev, const int32_t* y_dev, int64_t N);

/* Small fp32 models (KAVG_FP32, one hidden layer of at most 64 units, at most 16 classes, B <= 64,
 * d_0 a multiple of 4, P * ceil(d_0/64) no larger than the device's number of compute units, no
 * learner-level momentum) run all K local steps of Algorithm 1 in ONE launch that keeps the
 * learners' parameters on chip; workgroups of a learner wait for each other through counters in
 * the workspace, with a bounded number of polls (a wait that gives up makes the next call that
 * synchronises return KAVG_EDEVICE).  Same arithmetic as the launch-per-layer path up to the order
 * of fp32 sums.  kavg_fused: 1 when kavg_local_steps takes that path on this context.
 * kavg_set_fused(ctx, 0) switches it off (the steps then run as separate launches), 1 on again. */
int kavg_fused(const kavg_ctx* ctx);
int kavg_set_fused(kavg_ctx* ctx, int on);
/* Polls a workgroup of that launch spends on one wait for the others before it gives up (default 2^20, about a
 * second).  A wait that gives up never hangs the device: the launch runs to its end, the learners' replicas are
 * then not valid, and the next call that synchronises returns KAVG_EDEVICE once; install parameters again
 * (kavg_set_params / kavg_set_state) to go on.  Errors: KAVG_EINVAL for polls < 1. */
int kavg_set_wait_limit(kavg_ctx* ctx, unsigned polls);

/* Minibatch sampling ("randomly sample a mini-batch of size B", Algorithm 1).
 * idx_dev == NULL (default): learner j draws slot s of its t-th local step as
 *   SplitMix64 output number (c+1) of a generator seeded with index_seed,
 *   c = j*2^40 + t*2^16 + s, reduced mod N  -- i.i.d. uniform with replacement;
 *   t counts the learner's local steps since kavg_set_params.
 * idx_dev != NULL: int32 [P][K][B] device array used by every following
 *   kavg_local_steps call (BORROWED; every entry must lie in [0, N), which is
 *   checked on the device: offending entries are clamped into range and
 *   kavg_local_steps's next synchronising call reports KAVG_EINVAL). */
int kavg_set_indices(kavg_ctx* ctx, const int32_t* idx_dev);

/* K local minibatch-SGD steps on each of the P learners (inner loop of
 * Algorithm 1): sample, forward, softmax cross-entropy and its gradient,
 * backward, in-place update of the learner's replica.  Asynchronous.
 * Calling it twice without a meta update simply takes 2K local steps.
 * Errors: KAVG_ESTATE without parameters or data, KAVG_EDEVICE. */
int kavg_local_steps(kavg_ctx* ctx);

/* The meta level of Algorithm 1 in one fused pass: average the replicas, block
 * displacement d, block momentum v <- mu v + d, w~ <- w~ + v, and rebroadcast
 * w~ to every replica.  Asynchronous.  Increments the round. */
int kavg_meta_update(kavg_ctx* ctx);

/* Copy-outs (host pointers; each waits for the stream).  n must equal
 * kavg_num_params, else KAVG_EINVAL. */
int kavg_params(kavg_ctx* ctx, float* out_host, size_t n);            /* w~              */
int kavg_momentum(kavg_ctx* ctx, float* out_host, size_t n);          /* v               */
int kavg_replica(kavg_ctx* ctx, int j, float* out_host, size_t n);    /* w^j, 0 <= j < P */
/* [K][P] mean minibatch loss of every learner at every step of the last kavg_local_steps */
int kavg_losses(kavg_ctx* ctx, float* out_host);
/* [P][K][B] indices used by the last kavg_local_steps */
int kavg_indices(kavg_ctx* ctx, int32_t* out_host);

/* Learner-level momentum.  Section 2 notes that momentum "can also" be added at
 * the learner level (block momentum acts at the meta level); the form is not
 * given, so heavy ball is taken: every learner j keeps a velocity u^j and its
 * local step becomes  u <- beta u + g,  w <- w - lr u  (g = mean minibatch
 * gradient).  u^j persists across meta rounds (it is not reset when the learner
 * restarts from w~) and is zeroed by this call, kavg_set_params and
 * kavg_set_state.  velocity_dev: device block of kavg_velocity_bytes(ctx) bytes,
 * 256-byte aligned, BORROWED until kavg_destroy or until momentum is switched
 * off again with beta = 0.  Errors: KAVG_EINVAL (beta outside [0,1), beta > 0
 * without a buffer, misaligned), KAVG_ENOMEM (buffer too small). */
size_t kavg_velocity_bytes(const kavg_ctx* ctx);
int kavg_set_learner_momentum(kavg_ctx* ctx, float beta, void* velocity_dev, size_t bytes);
int kavg_velocity(kavg_ctx* ctx, int j, float* out_host, size_t n);   /* u^j; KAVG_ESTATE when off */

/* Deferred weight updates (KAVG_BF16).  The local step of Algorithm 1, w <- w - (lr/B) sum_s grad F(w; xi_s),
 * changes a layer's weights by the rank-B term -lr dZ^T A.  With a refresh period m > 1 the stored
 * replicas are brought up to date only every m local steps (and at the end of kavg_local_steps), by one
 * product over the m*B samples; between refreshes every product with the current weights is formed as
 * the product with the stored weights plus the pending terms, e.g. forward
 *     A W_k^T = A W_0^T - lr sum_{i<k} (A A_i^T) dZ_i ,
 * whose inner factors are only B x B per pending step.  The iterates are those of Algorithm 1 in exact
 * arithmetic; in bf16 the pending terms enter unrounded instead of through a re-rounded weight matrix,
 * and the inner factors are rounded to bf16.  A thin last layer (at most 16 classes) keeps being stepped
 * at once; biases always are.  m = 1 (default) is the plain path.  Pays when m*B is small against the
 * layer widths; needs the activations and dZ of m steps.
 * history_dev: device block of kavg_refresh_bytes(ctx, m) bytes, 256-byte aligned, BORROWED until
 * kavg_destroy or until m is set back to 1.  Waits for the stream.
 * Errors: KAVG_EINVAL (m outside [1, K], KAVG_FP32 context, null / misaligned block), KAVG_ENOMEM
 * (block too small), KAVG_ESTATE (learner-level momentum is on). */
size_t kavg_refresh_bytes(const kavg_ctx* ctx, int refresh);     /* 0 on bad arguments or refresh < 2 */
int kavg_set_refresh(kavg_ctx* ctx, int refresh, void* history_dev, size_t bytes);

/* Measurement aid for callers that report per-kernel time (not part of the
 * method): while a class's bit is set in class_mask, one launch in `every` of
 * that class (the first, the every+1-th, ...) is bracketed by a HIP event pair
 * on the context's stream; an event costs a few microseconds of stream time, so
 * a sparse sample keeps the timed region close to an unobserved one.
 * kavg_profile waits for the stream, clears the totals and installs the mask
 * (0 = off); kavg_profile_read waits for the stream and returns, per class, the
 * summed elapsed milliseconds and the number of bracketed launches since then
 * (arrays of KAVG_NCLASS entries, host).  KAVG_EINVAL: unknown class bit, every < 1. */
#define KAVG_CLASS_INDEX    0   /* minibatch index stream / import        */
#define KAVG_CLASS_FORWARD  1   /* per-layer forward products              */
#define KAVG_CLASS_LOSS     2   /* softmax cross-entropy + gradient, loss mean */
#define KAVG_CLASS_BACKWARD 3   /* per-layer data gradients                */
#define KAVG_CLASS_UPDATE   4   /* per-layer weight gradient + SGD update  */
#define KAVG_CLASS_META     5   /* fused meta step                         */
#define KAVG_CLASS_HEAD     6   /* last layer with <= 16 classes: forward + loss + data gradient, and its update */
#define KAVG_CLASS_CORRECTION 7  /* deferred updates: the low-rank terms of forward and backward products */
#define KAVG_NCLASS         8
int kavg_profile(kavg_ctx* ctx, unsigned class_mask, unsigned every);
int kavg_profile_read(kavg_ctx* ctx, double* ms_out, long long* launches_out);

/* Replay of the K local steps as one HIP graph (Algorithm 1, the inner loop
 * over k: the launches of a round differ from those of the next only in the
 * minibatch indices, which a kernel outside the graph writes first).  For
 * launch-bound shapes (small layers, few learners) this removes most of the
 * host's per-launch cost; results are bit-identical to the eager path, which
 * stays the default.  With on != 0, kavg_local_steps runs eagerly once more
 * (after kavg_init, kavg_set_data or kavg_set_learner_momentum), records the
 * sequence on its next call and replays it from then on; calls made while
 * kavg_profile has a non-zero mask run eagerly.  on == 0 waits for the stream
 * and drops the recording.  KAVG_ESTATE: the context works on the default
 * (null) stream, which cannot be captured.  While a call records, no other
 * thread-unsafe HIP call may be made on this thread's behalf on that stream. */
int kavg_graph(kavg_ctx* ctx, int on);

/* Measurement aid (not part of the method): one launch of a probe kernel on hip_stream, so that a
 * benchmark can state what this device reaches with the access pattern of the fused meta step of
 * Algorithm 1 (every lane owns a 16-byte piece of each of 16 interleaved rows, non-temporal):
 *   KAVG_PROBE_READ   reads `bytes` of a_dev;         KAVG_PROBE_WRITE  overwrites `bytes` of a_dev;
 *   KAVG_PROBE_COPY   reads a_dev, writes b_dev (equal parts, like the meta step);
 *   KAVG_PROBE_MFMA   `iters` x 4 independent v_mfma_f32_32x32x16_bf16 per wavefront, 8 workgroups
 *                     per compute unit, no memory traffic (buffers unused).
 * a_dev / b_dev: device blocks of at least `bytes` (16-byte aligned; rounded down to a multiple of
 * 256 bytes), sink_dev: one float of device memory (never written in practice).  *work_out (host)
 * receives the bytes moved (both directions counted) or the flops of the launch.  Asynchronous;
 * the caller times it.  Errors: KAVG_EINVAL (unknown kind, null / misaligned pointers, bytes < 256,
 * iters < 1), KAVG_EDEVICE. */
#define KAVG_PROBE_READ  0
#define KAVG_PROBE_WRITE 1
#define KAVG_PROBE_COPY  2
#define KAVG_PROBE_MFMA  3
int kavg_probe(int kind, void* a_dev, void* b_dev, size_t bytes, int iters, float* sink_dev,
               void* hip_stream, double* work_out);

uint64_t    kavg_round(const kavg_ctx* ctx);
const char* kavg_last_error(const kavg_ctx* ctx);   /* ctx == NULL: text of the last failed kavg_init */
int         kavg_destroy(kavg_ctx* ctx);            /* waits for the stream, frees the host context  */

/* The fused meta step (same kernel as kavg_meta_update) on caller-owned
 * arrays, for a flat parameter vector of any length n >= 1:
 *   w_tilde_dev [n], v_dev [n]: updated in place;
 *   replicas_dev: P replicas, replica j at replicas_dev + j*replica_stride
 *     (replica_stride >= n, in floats); read, then overwritten with w~_{n+1};
 *   shadow_dev: NULL, or bf16 copies (nearest, ties away from zero) written at
 *     shadow_dev + j*shadow_stride.
 * Pointers 16-byte aligned and strides multiples of 4 (8 for the shadow) take
 * the vector path; anything else takes a slower scalar path.  Asynchronous on
 * hip_stream.  Errors: KAVG_EINVAL (P < 1, n < 1, stride < n, mu outside
 * [0,1), null pointers), KAVG_EDEVICE. */
int kavg_meta_update_flat(float* w_tilde_dev, float* v_dev, float* replicas_dev,
                          size_t replica_stride, uint16_t* shadow_dev, size_t shadow_stride,
                          int P, size_t n, float mu, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KAVG_H */
