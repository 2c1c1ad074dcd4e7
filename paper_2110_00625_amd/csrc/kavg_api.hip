// C boundary of the M-AVG hot path: context, workspace carve-up, and the
// launch sequences of the learner loop and the meta step (Algorithm 1).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/kavg.h"
#include "kavg_internal.h"
#include "conv_wgrad.h"
#include "conv_direct.h"
#include "conv_first.h"
#include "split.h"

using namespace kavg;

namespace {

constexpr size_t ALIGN = 256;
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t n = 0, stride = 0;          // parameters per replica, padded replica stride (elements)
    int ldz = 0;                       // padded class count (logits / dZ_L leading dimension)
    size_t off_w = 0, off_v = 0, off_reps = 0, off_shadow = 0, off_idx = 0, off_flag = 0;
    size_t off_logits = 0, off_rowloss = 0, off_losses = 0, off_scratch = 0;
    std::vector<size_t> off_act, off_dz;   // per layer l = 1..L (index l-1); act of the last layer unused
    std::vector<size_t> w_off, b_off;      // parameter offsets inside a replica
    // convolution stack in front of the MLP (kavg_init_conv); empty for a plain MLP
    std::vector<size_t> cw_off, cb_off;    // parameter offsets of the convolutions (they come first in the flat vector)
    std::vector<size_t> off_patch, off_cact, off_cdz;   // per convolution: patch matrix, output images, their dZ
    std::vector<int> splits;               // ranges of positions its weight gradient is split over
    std::vector<int> splits_halo;          // the same for the all-taps weight-gradient kernel; 0: shape not covered
    size_t off_draw = 0, off_pool = 0, off_dpool = 0, off_partial = 0, off_pbias = 0;
    bool conv_implicit = false;            // convolutions 2.. form their patch matrices inside the MFMA kernel's loaders
    size_t off_wrot = 0;                   // ... and their data gradient reads the weights as [(tap, o)][c_in]
    // all K steps of a small fp32 model in one launch (fused_small.hip): scratch and wait counters; 0 = shape not eligible
    size_t off_fused = 0;
    size_t total = 0;
};

// H x W images, channels ch[0] (input) .. ch[M]; ch empty: plain MLP
struct ConvSpec { int H = 0, W = 0; std::vector<int> ch; };

bool conv_ok(const ConvSpec& cv, int L, const int* dims, int dtype, int B) {
    if (cv.ch.empty()) return true;
    if (dtype != KAVG_BF16 || cv.H < 1 || cv.W < 1 || cv.H > 4096 || cv.W > 4096 || cv.ch.size() < 2 || cv.ch.size() > 64) return false;
    for (int c : cv.ch) if (c < 8 || c % 8 != 0 || c > 2048) return false;
    if ((size_t)B * cv.H * cv.W >= ((size_t)1 << 30)) return false;
    return dims[0] == cv.ch.back();
}

bool shapes_ok(int P, int K, int B, int L, const int* dims, int dtype) {
    if (P < 1 || K < 1 || B < 1 || L < 1 || !dims) return false;
    if (P > (1 << 24) || K > (1 << 24) || B > (1 << 16)) return false;
    if (dtype != KAVG_FP32 && dtype != KAVG_BF16) return false;
    for (int l = 0; l <= L; ++l) {
        if (dims[l] < 1 || dims[l] > (1 << 24)) return false;
        if (dtype == KAVG_BF16 && l < L && dims[l] % 8 != 0) return false;
    }
    return true;
}

Layout make_layout(int P, int K, int B, int L, const int* dims, int dtype, const ConvSpec& cv = ConvSpec()) {
    Layout lo;
    const size_t esz = dtype == KAVG_BF16 ? 2 : 4;     // activation / dZ element size
    size_t o = 0;
    const int M = cv.ch.empty() ? 0 : (int)cv.ch.size() - 1;
    for (int t = 1; t <= M; ++t) {
        lo.cw_off.push_back(o);
        o += (size_t)cv.ch[t] * 9 * cv.ch[t - 1];
        lo.cb_off.push_back(o);
        o += cv.ch[t];
    }
    for (int l = 1; l <= L; ++l) {
        lo.w_off.push_back(o);
        o += (size_t)dims[l] * dims[l - 1];
        lo.b_off.push_back(o);
        o += dims[l];
    }
    lo.n = o;
    lo.stride = round_up(lo.n, 64);
    lo.ldz = (int)round_up((size_t)dims[L], 8);
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = round_up(p + bytes, ALIGN); return at; };
    lo.off_w = take(lo.stride * 4);
    lo.off_v = take(lo.stride * 4);
    // fp32 mode: P replicas of fp32.  bf16 mode: every replica as two 16-bit planes (split.h), the
    // lo planes where the fp32 replicas would be, the hi planes (the bf16 operands) after them.
    lo.off_reps = take((size_t)P * lo.stride * (dtype == KAVG_BF16 ? 2 : 4));
    lo.off_shadow = dtype == KAVG_BF16 ? take((size_t)P * lo.stride * 2) : 0;
    lo.off_idx = take((size_t)P * K * B * 4);
    lo.off_flag = take(ALIGN);
    for (int l = 1; l <= L; ++l) {
        const size_t ld = l == L ? (size_t)lo.ldz : (size_t)dims[l];
        lo.off_act.push_back(l < L ? take((size_t)P * B * ld * esz) : 0);
        lo.off_dz.push_back(take((size_t)P * B * ld * esz));
    }
    lo.off_logits = take((size_t)P * B * lo.ldz * 4);
    lo.off_rowloss = take((size_t)K * P * B * 4);
    lo.off_losses = take((size_t)K * P * 4);
    if (dtype == KAVG_FP32) {          // partial tiles of the split forward contractions
        size_t need = 0;
        for (int l = 1; l <= L; ++l) {
            const int splits = f32_forward_plan(P, B, dims[l - 1], dims[l], nullptr);
            const size_t ld = l == L ? (size_t)lo.ldz : (size_t)dims[l];
            if (splits > 1 && (size_t)splits * P * B * ld * 4 > need) need = (size_t)splits * P * B * ld * 4;
        }
        lo.off_scratch = need ? take(need) : 0;
        // (sized for a device of up to 256 compute units; the context decides with the real count)
        if (L == 2 && M == 0 && fused_small_shape_ok(P, K, B, dims[0], dims[1], dims[2], 256))
            lo.off_fused = take(fused_small_scratch_bytes(P, dims[0]));
    }
    if (M > 0) {
        const size_t rows = (size_t)B * cv.H * cv.W;
        size_t draw = 0, partial = 0, pbias = 0, wrot = 0;
        lo.conv_implicit = (size_t)cv.H * cv.W < ((size_t)1 << 14);     // range of the loaders' multiply-shift divisions
        for (int t = 1; t <= M; ++t) {
            const int S1 = (t == 1 && lo.conv_implicit) ? conv_first_splits(P, B, cv.H, cv.W, cv.ch[0], cv.ch[1]) : 0;
            // explicit patches: every convolution of very large images, and a first convolution (it gathers its images)
            // that the kernels of conv_first.hip do not cover
            const bool expl = (t == 1 && S1 == 0) || !lo.conv_implicit;
            lo.off_patch.push_back(expl ? take((size_t)P * rows * 9 * cv.ch[t - 1] * 2) : 0);
            lo.off_cact.push_back(take((size_t)P * rows * cv.ch[t] * 2));
            lo.off_cdz.push_back(take((size_t)P * rows * cv.ch[t] * 2));
            if (t > 1 && !lo.conv_implicit && (size_t)P * rows * 9 * cv.ch[t - 1] * 4 > draw) draw = (size_t)P * rows * 9 * cv.ch[t - 1] * 4;
            if (t > 1 && lo.conv_implicit && (size_t)P * 9 * cv.ch[t] * cv.ch[t - 1] * 2 > wrot) wrot = (size_t)P * 9 * cv.ch[t] * cv.ch[t - 1] * 2;
            // split the weight gradient's contraction until the launch has some hundreds of workgroups,
            // keeping at least 256 positions per range
            const size_t tiles = (size_t)((cv.ch[t] + 127) / 128) * ((9 * cv.ch[t - 1] + 127) / 128) * P;
            int S = 1;
            while (tiles * S < 512 && rows % (2 * (size_t)S) == 0 && rows / (2 * (size_t)S) >= 256) S *= 2;
            lo.splits.push_back(S);
            const int Sh = t == 1 ? S1 : lo.conv_implicit ? conv_wgrad_halo_splits(P, B, cv.H, cv.W, cv.ch[t - 1], cv.ch[t]) : 0;
            lo.splits_halo.push_back(Sh);
            if (Sh > S) S = Sh;                                          // (sizes the partial buffers below)
            const size_t nw = (size_t)cv.ch[t] * 9 * cv.ch[t - 1];
            if ((size_t)P * S * nw * 4 > partial) partial = (size_t)P * S * nw * 4;
            if ((size_t)P * S * cv.ch[t] * 4 > pbias) pbias = (size_t)P * S * cv.ch[t] * 4;
        }
        lo.off_draw = draw ? take(draw) : 0;
        lo.off_wrot = wrot ? take(wrot) : 0;
        lo.off_pool = take((size_t)P * B * cv.ch[M] * 2);
        lo.off_dpool = take((size_t)P * B * cv.ch[M] * 2);
        lo.off_partial = take(partial);
        lo.off_pbias = take(pbias);
    }
    lo.total = p;
    return lo;
}

char g_init_error[256] = "";

// ---- workspace inside the library, for callers that cannot allocate device memory ----
// One block per device (every GPU that loads the library holds its own copy until the process
// ends).  In host code the array's name is only a handle: its device address is looked up once per
// device with hipGetSymbolAddress and kept in g_static_ptr; everything below uses that pointer.
constexpr size_t STATIC_WS_BYTES = KAVG_STATIC_WORKSPACE_BYTES;
constexpr int MAX_DEVICES = 64;
void* g_static_ptr[MAX_DEVICES] = {};          // device address of `scratch` on device d (null: not looked up yet)
kavg_ctx* g_static_owner[MAX_DEVICES] = {};    // the context that currently works in it

}  // namespace

static __device__ __align__(256) unsigned char scratch[KAVG_STATIC_WORKSPACE_BYTES];

// No exception may cross the C boundary: host allocations inside the library (layout tables, event
// pools, staging vectors) are the only possible source.
#define KAVG_NOTHROW_BEGIN try {
#define KAVG_NOTHROW_END(ctx)                                                                   \
    } catch (const std::bad_alloc&) { return fail(ctx, KAVG_ENOMEM, "host allocation failed"); } \
    catch (...) { return fail(ctx, KAVG_ENOMEM, "unexpected host failure"); }

// carve-up of the history block of deferred weight updates (kavg_set_refresh)
struct HistoryLayout {
    std::vector<size_t> act, dz;        // per layer l = 1..L (index l-1): activations leaving / dZ of the layer, [P][m*B][ld]
    size_t z0 = 0, s = 0, total = 0;    // fp32 [P][B][maxld]; bf16 [P][B][ldS]
    int ldS = 0, maxld = 0;
};

struct kavg_ctx {
    int P, K, B, L, dtype;
    float lr, mu;
    uint64_t seed;
    std::vector<int> dims;
    Layout lo;
    char* ws;
    hipStream_t stream;
    const void* X;
    const int32_t* y;
    int64_t N;
    const int32_t* user_idx;
    uint32_t t0;          // local steps every learner has taken
    uint64_t round;
    bool have_params, have_steps;
    bool replicas_equal = false;   // every replica holds the global model (no local step since the last rebroadcast)
    float beta;           // learner-level momentum, 0 = off
    float* vel;           // [P][stride] velocities, caller memory, null = off
    char err[256];
    // measurement aid: HIP event pairs around the launches of selected kernel classes
    unsigned prof_mask;
    unsigned prof_every;                            // bracket one launch in prof_every of a class
    unsigned long long prof_seen[KAVG_NCLASS];      // launches of the class since kavg_profile
    std::vector<hipEvent_t> prof_ev[KAVG_NCLASS];   // start/stop alternate
    size_t prof_used[KAVG_NCLASS];
    double prof_ms[KAVG_NCLASS];
    long long prof_launches[KAVG_NCLASS];
    // replay of the K-step launch sequence as one HIP graph (kavg_graph)
    bool graph_on = false;
    bool warm = false;                  // the sequence has run eagerly once with the current pointers
    hipGraphExec_t gexec = nullptr;
    ConvSpec cv;                        // convolution stack in front of the MLP (empty: plain MLP)
    bool fused_ok = false;              // the shape and the device allow all K steps in one launch (fused_small.hip)
    bool fused_on = true;               // ... and the caller has not switched it off (kavg_set_fused)
    unsigned spin_limit = 1u << 20;     // polls a workgroup of that launch spends on one wait before it gives up
    int compute_units = 0;
    uint32_t fused_tag = 0;             // steps that launch has exchanged partials for so far (their tags on the scratch)
    // deferred weight updates (kavg_set_refresh): history block, its carve-up, refresh period
    int refresh = 1;
    char* hist = nullptr;
    HistoryLayout hl;
    int static_dev = -1;                // >= 0: the context works in the library's own workspace of that device

    float* w_tilde() const { return (float*)(ws + lo.off_w); }
    float* v() const { return (float*)(ws + lo.off_v); }
    float* reps() const { return dtype == KAVG_BF16 ? nullptr : (float*)(ws + lo.off_reps); }            // fp32 mode
    uint16_t* lo_planes() const { return dtype == KAVG_BF16 ? (uint16_t*)(ws + lo.off_reps) : nullptr; }    // bf16 mode
    uint16_t* hi_planes() const { return dtype == KAVG_BF16 ? (uint16_t*)(ws + lo.off_shadow) : nullptr; }
    int32_t* idx() const { return (int32_t*)(ws + lo.off_idx); }
    int* flag() const { return (int*)(ws + lo.off_flag); }
    float* logits() const { return (float*)(ws + lo.off_logits); }
    float* rowloss() const { return (float*)(ws + lo.off_rowloss); }
    float* losses() const { return (float*)(ws + lo.off_losses); }
};

namespace {

void drop_graph(kavg_ctx* c);

int fail(kavg_ctx* c, int code, const char* fmt, ...) {
    char* dst = c ? c->err : g_init_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return code;
}

#define KAVG_HIP(ctx, call)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) return fail(ctx, KAVG_EDEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// wait for the stream, then report (and clear) the device-side range flag
int sync_and_check(kavg_ctx* c) {
    int flag[2] = {0, 0};                   // [0] range error, [1] a wait between workgroups gave up
    KAVG_HIP(c, hipMemcpyAsync(flag, c->flag(), sizeof(flag), hipMemcpyDeviceToHost, c->stream));
    KAVG_HIP(c, hipStreamSynchronize(c->stream));
    if (flag[0] || flag[1]) {
        KAVG_HIP(c, hipMemsetAsync(c->flag(), 0, sizeof(flag), c->stream));
        KAVG_HIP(c, hipStreamSynchronize(c->stream));
        if (flag[1])
            return fail(c, KAVG_EDEVICE, "a wait between the workgroups of the fused local steps ran out of polls; "
                        "the replicas are not valid (kavg_set_fused(ctx, 0) runs the steps as separate launches)");
        return fail(c, KAVG_EINVAL, "an index or label outside its range was found on the device");
    }
    return KAVG_OK;
}

int install_global(kavg_ctx* c, const float* w_host, const float* v_host) {
    KAVG_HIP(c, hipMemcpyAsync(c->w_tilde(), w_host, c->lo.n * 4, hipMemcpyHostToDevice, c->stream));
    if (v_host)
        KAVG_HIP(c, hipMemcpyAsync(c->v(), v_host, c->lo.n * 4, hipMemcpyHostToDevice, c->stream));
    else
        KAVG_HIP(c, hipMemsetAsync(c->v(), 0, c->lo.stride * 4, c->stream));
    if (c->dtype == KAVG_BF16)
        KAVG_HIP(c, launch_broadcast_split(c->w_tilde(), c->hi_planes(), c->lo_planes(), c->lo.stride, c->P,
                                           c->lo.n, c->stream));
    else
        KAVG_HIP(c, launch_broadcast(c->w_tilde(), c->reps(), c->lo.stride, nullptr, c->lo.stride, c->P,
                                     c->lo.n, c->stream));
    if (c->vel) KAVG_HIP(c, hipMemsetAsync(c->vel, 0, (size_t)c->P * c->lo.stride * 4, c->stream));
    KAVG_HIP(c, hipStreamSynchronize(c->stream));   // host buffers may be reused by the caller
    c->have_params = true;
    c->have_steps = false;
    c->replicas_equal = true;
    return KAVG_OK;
}

// Brackets one launch with an event pair when its class is being profiled.
struct Bracket {
    kavg_ctx* c; int cls; bool on; hipEvent_t stop;
    Bracket(kavg_ctx* ctx, int k) : c(ctx), cls(k), on(false), stop(nullptr) {
        if (!(c->prof_mask & (1u << cls))) return;
        if ((c->prof_seen[cls]++ % c->prof_every) != 0) return;
        std::vector<hipEvent_t>& pool = c->prof_ev[cls];
        while (pool.size() < c->prof_used[cls] + 2) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            pool.push_back(e);
        }
        hipEvent_t start = pool[c->prof_used[cls]];
        stop = pool[c->prof_used[cls] + 1];
        if (hipEventRecord(start, c->stream) != hipSuccess) return;
        c->prof_used[cls] += 2;
        on = true;
    }
    ~Bracket() { if (on) (void)hipEventRecord(stop, c->stream); }
};

// The bf16 (hi) planes of all learners are re-read by every forward pass.  If together they fit well
// inside the memory-side cache of the chip (256 MB), the kernels that write them use ordinary
// stores and the next reader finds them there; larger sets are written with streaming stores,
// which measured faster than letting them churn the cache.
int shadows_stay_cached(int P, size_t elems_per_learner) {
    return (size_t)P * elems_per_learner * 2 <= ((size_t)192 << 20) ? 1 : 0;
}

LayerCall layer_call(const kavg_ctx* c, int l /*1..L*/, int k) {
    const Layout& lo = c->lo;
    const size_t esz = c->dtype == KAVG_BF16 ? 2 : 4;
    const int L = c->L;
    LayerCall q = {};
    q.P = c->P; q.B = c->B;
    q.d_in = c->dims[l - 1]; q.d_out = c->dims[l];
    q.w_stride = lo.stride; q.ws_stride = lo.stride;
    if (c->dtype == KAVG_BF16) {
        q.ws = c->hi_planes() + lo.w_off[l - 1];  q.wlo = c->lo_planes() + lo.w_off[l - 1];
        q.bhi = c->hi_planes() + lo.b_off[l - 1]; q.blo = c->lo_planes() + lo.b_off[l - 1];
    } else {
        q.w = c->reps() + lo.w_off[l - 1];
        q.b = c->reps() + lo.b_off[l - 1];
    }
    q.shadow_cached = shadows_stay_cached(c->P, lo.stride);
    if (l == 1 && !c->cv.ch.empty()) {       // behind a convolution stack: the mean over the positions
        q.in = c->ws + lo.off_pool; q.ld_in = c->dims[0]; q.in_stride = (size_t)c->B * q.ld_in;
        q.dz_prev = c->ws + lo.off_dpool; q.dz_prev_stride = q.in_stride;
    } else if (l == 1) {
        q.in = c->X; q.ld_in = c->dims[0]; q.in_stride = 0;
        q.gather = c->idx() + (size_t)k * c->B; q.gather_stride = (long)c->K * c->B;
        q.next_gather = k + 1 < c->K ? q.gather + c->B : nullptr;
    } else {
        q.in = c->ws + lo.off_act[l - 2]; q.ld_in = c->dims[l - 1]; q.in_stride = (size_t)c->B * q.ld_in;
        q.dz_prev = c->ws + lo.off_dz[l - 2]; q.dz_prev_stride = (size_t)c->B * q.ld_in;
    }
    if (l < L) {
        q.out = c->ws + lo.off_act[l - 1]; q.ld_out = c->dims[l]; q.relu = 1;
    } else {
        q.out = c->logits(); q.ld_out = lo.ldz; q.relu = 0;
    }
    q.out_stride = (size_t)c->B * q.ld_out;
    q.dz = c->ws + lo.off_dz[l - 1]; q.ld_dz = l == L ? lo.ldz : c->dims[l];
    q.dz_stride = (size_t)c->B * q.ld_dz;
    q.lr = c->lr;
    q.beta = c->beta;
    q.u = c->vel ? c->vel + lo.w_off[l - 1] : nullptr;
    q.ub = c->vel ? c->vel + lo.b_off[l - 1] : nullptr;
    q.scratch = c->lo.off_scratch ? c->ws + c->lo.off_scratch : nullptr;
    (void)esz;
    return q;
}

}  // namespace

extern "C" {

size_t kavg_num_params(int n_layers, const int* dims) {
    if (n_layers < 1 || !dims) return 0;
    size_t n = 0;
    for (int l = 1; l <= n_layers; ++l) {
        if (dims[l] < 1 || dims[l - 1] < 1) return 0;
        n += (size_t)dims[l] * dims[l - 1] + dims[l];
    }
    return n;
}

size_t kavg_workspace_bytes(int P, int K, int B, int n_layers, const int* dims, int dtype) {
    if (!shapes_ok(P, K, B, n_layers, dims, dtype)) return 0;
    try { return make_layout(P, K, B, n_layers, dims, dtype).total; } catch (...) { return 0; }
}

}  // extern "C"

namespace {

bool conv_spec(ConvSpec* cv, int H, int W, int n_conv, const int* channels) {
    if (n_conv < 1 || n_conv > 63 || !channels) return false;
    cv->H = H; cv->W = W;
    cv->ch.assign(channels, channels + n_conv + 1);
    return true;
}

int init_common(kavg_ctx** out, int P, int K, float lr, float mu, int n_layers, const int* dims, int B,
                int dtype, uint64_t index_seed, void* workspace_dev, size_t workspace_bytes,
                void* hip_stream, const ConvSpec& cv) {
    if (!out) return fail(nullptr, KAVG_EINVAL, "out is null");
    *out = nullptr;
    kavg_ctx* c = nullptr;
    try {
    if (!shapes_ok(P, K, B, n_layers, dims, dtype))
        return fail(nullptr, KAVG_EINVAL, "bad shape: need P,K,B >= 1 (P,K <= 2^24, B <= 65536), "
                    "dims >= 1 and, for bf16, d_0..d_{L-1} multiples of 8");
    if (!conv_ok(cv, n_layers, dims, dtype, B))
        return fail(nullptr, KAVG_EINVAL, "bad convolution stack: need bf16, H,W in [1,4096], channel counts that are "
                    "multiples of 8 in [8,2048], B*H*W < 2^30 and d_0 equal to the last channel count");
    if (!(lr >= 0.f) || !std::isfinite(lr)) return fail(nullptr, KAVG_EINVAL, "lr must be finite and >= 0");
    if (!(mu >= 0.f && mu < 1.f)) return fail(nullptr, KAVG_EINVAL, "mu must lie in [0,1)");
    if (!workspace_dev || ((uintptr_t)workspace_dev % ALIGN) != 0)
        return fail(nullptr, KAVG_EINVAL, "workspace must be a non-null, 256-byte aligned device pointer");
    Layout lo = make_layout(P, K, B, n_layers, dims, dtype, cv);
    if (workspace_bytes < lo.total)
        return fail(nullptr, KAVG_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, lo.total);
    c = new (std::nothrow) kavg_ctx();
    if (!c) return fail(nullptr, KAVG_ENOMEM, "host allocation failed");
    c->cv = cv;
    c->P = P; c->K = K; c->B = B; c->L = n_layers; c->dtype = dtype;
    c->lr = lr; c->mu = mu; c->seed = index_seed;
    c->dims.assign(dims, dims + n_layers + 1);
    c->lo = lo;
    c->ws = (char*)workspace_dev;
    c->stream = (hipStream_t)hip_stream;
    c->X = nullptr; c->y = nullptr; c->N = 0; c->user_idx = nullptr;
    c->t0 = 0; c->round = 0; c->have_params = false; c->have_steps = false;
    c->beta = 0.f; c->vel = nullptr;
    c->err[0] = 0;
    c->prof_mask = 0;
    c->prof_every = 1;
    for (int k = 0; k < KAVG_NCLASS; ++k) { c->prof_used[k] = 0; c->prof_ms[k] = 0.0; c->prof_launches[k] = 0; c->prof_seen[k] = 0; }
    hipError_t e = hipMemsetAsync(c->flag(), 0, ALIGN, c->stream);
    if (e == hipSuccess && lo.off_fused) {
        int dev = 0, cus = 0;
        e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        c->compute_units = cus;
        c->fused_ok = e == hipSuccess && fused_small_shape_ok(P, K, B, dims[0], dims[1], dims[2], cus);
        if (e == hipSuccess) e = hipMemsetAsync(c->ws + lo.off_fused, 0, fused_small_scratch_bytes(P, dims[0]), c->stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        fail(nullptr, KAVG_EDEVICE, "clearing the workspace flag failed: %s", hipGetErrorString(e));
        delete c;
        return KAVG_EDEVICE;
    }
    *out = c;
    return KAVG_OK;
    } catch (...) {
        delete c;
        return fail(nullptr, KAVG_ENOMEM, "host allocation failed");
    }
}

}  // namespace

extern "C" {

int kavg_init(kavg_ctx** out, int P, int K, float lr, float mu, int n_layers, const int* dims, int B,
              int dtype, uint64_t index_seed, void* workspace_dev, size_t workspace_bytes,
              void* hip_stream) {
    return init_common(out, P, K, lr, mu, n_layers, dims, B, dtype, index_seed, workspace_dev, workspace_bytes,
                       hip_stream, ConvSpec());
}

size_t kavg_num_params_conv(int H, int W, int n_conv, const int* channels, int n_layers, const int* dims) {
    (void)H; (void)W;
    if (n_conv < 1 || !channels) return 0;
    size_t n = kavg_num_params(n_layers, dims);
    if (n == 0) return 0;
    for (int t = 1; t <= n_conv; ++t) {
        if (channels[t] < 1 || channels[t - 1] < 1) return 0;
        n += (size_t)channels[t] * 9 * channels[t - 1] + channels[t];
    }
    return n;
}

size_t kavg_workspace_bytes_conv(int P, int K, int B, int H, int W, int n_conv, const int* channels, int n_layers,
                                 const int* dims) {
    try {
        ConvSpec cv;
        if (!conv_spec(&cv, H, W, n_conv, channels)) return 0;
        if (!shapes_ok(P, K, B, n_layers, dims, KAVG_BF16) || !conv_ok(cv, n_layers, dims, KAVG_BF16, B)) return 0;
        return make_layout(P, K, B, n_layers, dims, KAVG_BF16, cv).total;
    } catch (...) { return 0; }
}

int kavg_init_conv(kavg_ctx** out, int P, int K, float lr, float mu, int H, int W, int n_conv, const int* channels,
                   int n_layers, const int* dims, int B, uint64_t index_seed, void* workspace_dev,
                   size_t workspace_bytes, void* hip_stream) {
    try {
        ConvSpec cv;
        if (!conv_spec(&cv, H, W, n_conv, channels)) {
            if (out) *out = nullptr;
            return fail(nullptr, KAVG_EINVAL, "need 1..63 convolutions and their channel counts");
        }
        return init_common(out, P, K, lr, mu, n_layers, dims, B, KAVG_BF16, index_seed, workspace_dev, workspace_bytes,
                           hip_stream, cv);
    } catch (...) {
        if (out) *out = nullptr;
        return fail(nullptr, KAVG_ENOMEM, "host allocation failed");
    }
}

int kavg_init_static(kavg_ctx** out, int P, int K, float lr, float mu, int n_layers, const int* dims, int B,
                     int dtype, uint64_t index_seed, void* hip_stream) {
    if (!out) return fail(nullptr, KAVG_EINVAL, "out is null");
    *out = nullptr;
    const size_t need = kavg_workspace_bytes(P, K, B, n_layers, dims, dtype);
    if (need == 0)
        return fail(nullptr, KAVG_EINVAL, "bad shape: need P,K,B >= 1 (P,K <= 2^24, B <= 65536), "
                    "dims >= 1 and, for bf16, d_0..d_{L-1} multiples of 8");
    if (need > STATIC_WS_BYTES)
        return fail(nullptr, KAVG_ENOMEM, "this configuration needs %zu bytes of workspace, the library's own block "
                    "holds %zu: use kavg_init with a caller workspace", need, STATIC_WS_BYTES);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(nullptr, KAVG_EDEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(nullptr, KAVG_EINVAL, "device ordinal %d not supported", dev);
    if (!g_static_ptr[dev]) {               // once per device, with that device current
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(nullptr, KAVG_EDEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_static_ptr[dev] = ptr;
    }
    if (g_static_owner[dev])
        return fail(nullptr, KAVG_ESTATE, "the library's workspace on device %d is in use by another context", dev);
    const int rc = kavg_init(out, P, K, lr, mu, n_layers, dims, B, dtype, index_seed, g_static_ptr[dev],
                             STATIC_WS_BYTES, hip_stream);
    if (rc != KAVG_OK) return rc;
    (*out)->static_dev = dev;
    g_static_owner[dev] = *out;
    return KAVG_OK;
}

int kavg_set_params(kavg_ctx* c, const float* w0_host) {
    if (!c) return KAVG_EINVAL;
    if (!w0_host) return fail(c, KAVG_EINVAL, "w0_host is null");
    c->t0 = 0;
    c->round = 0;
    return install_global(c, w0_host, nullptr);
}

int kavg_set_state(kavg_ctx* c, const float* w_host, const float* v_host, uint64_t round) {
    if (!c) return KAVG_EINVAL;
    if (!w_host || !v_host) return fail(c, KAVG_EINVAL, "null state pointer");
    if (round > ((uint64_t)1 << 24) / (uint64_t)c->K) return fail(c, KAVG_EINVAL, "round*K exceeds 2^24 local steps");
    c->round = round;
    c->t0 = (uint32_t)(round * (uint64_t)c->K);
    return install_global(c, w_host, v_host);
}

int kavg_set_data(kavg_ctx* c, const void* X_dev, const int32_t* y_dev, int64_t N) {
    if (!c) return KAVG_EINVAL;
    if (!X_dev || !y_dev) return fail(c, KAVG_EINVAL, "null data pointer");
    if (N < 1 || N >= ((int64_t)1 << 31)) return fail(c, KAVG_EINVAL, "N must lie in [1, 2^31)");
    if (((uintptr_t)X_dev & 15) != 0) return fail(c, KAVG_EINVAL, "X_dev must be 16-byte aligned");
    KAVG_HIP(c, launch_label_check(y_dev, (size_t)N, c->dims[c->L], c->flag(), c->stream));
    int rc = sync_and_check(c);
    if (rc != KAVG_OK) return rc == KAVG_EINVAL ? fail(c, KAVG_EINVAL, "a label lies outside [0, d_L)") : rc;
    c->X = X_dev; c->y = y_dev; c->N = N;
    drop_graph(c);
    return KAVG_OK;
}

int kavg_fused(const kavg_ctx* c) { return c && c->fused_ok && c->fused_on && !c->vel ? 1 : 0; }

int kavg_set_fused(kavg_ctx* c, int on) {
    if (!c) return KAVG_EINVAL;
    KAVG_HIP(c, hipStreamSynchronize(c->stream));
    c->fused_on = on != 0;
    drop_graph(c);
    return KAVG_OK;
}

int kavg_set_wait_limit(kavg_ctx* c, unsigned polls) {
    if (!c) return KAVG_EINVAL;
    if (polls < 1) return fail(c, KAVG_EINVAL, "the wait limit must be at least one poll");
    c->spin_limit = polls;
    return KAVG_OK;
}

int kavg_set_indices(kavg_ctx* c, const int32_t* idx_dev) {
    if (!c) return KAVG_EINVAL;
    c->user_idx = idx_dev;
    return KAVG_OK;
}

namespace {

// The K local steps of every learner after the indices are in place, and the per-step loss means.
// All arguments are fixed between calls (workspace pointers, data pointers, shapes), which is what
// lets kavg_local_steps replay this sequence as a graph.
int issue_steps_deferred(kavg_ctx* c);
int issue_steps_conv(kavg_ctx* c);

bool fused_now(const kavg_ctx* c) { return c->fused_ok && c->fused_on && !c->vel; }

// Small fp32 model: indices, all K steps and the per-step losses in one launch (fused_small.hip).  The launch
// carries the step counter (index stream, tags), so it is issued directly, never replayed from a graph.
int issue_steps_fused(kavg_ctx* c) {
    hipStream_t st = c->stream;
    if (c->fused_tag + (uint32_t)c->K + 1u < c->fused_tag) {    // the tags would wrap: start over on a clean scratch
        KAVG_HIP(c, hipMemsetAsync(c->ws + c->lo.off_fused, 0, fused_small_scratch_bytes(c->P, c->dims[0]), st));
        c->fused_tag = 0;
    }
    FusedSmallCall q{};
    q.P = c->P; q.K = c->K; q.B = c->B; q.d0 = c->dims[0]; q.d1 = c->dims[1]; q.C = c->dims[2];
    q.reps = c->reps(); q.rep_stride = c->lo.stride;
    q.w1_off = c->lo.w_off[0]; q.b1_off = c->lo.b_off[0]; q.w2_off = c->lo.w_off[1]; q.b2_off = c->lo.b_off[1];
    q.X = (const float*)c->X; q.y = c->y; q.idx = c->idx();
    q.generate_idx = c->user_idx ? 0 : 1; q.seed = c->seed; q.t0 = c->t0; q.N = (uint32_t)c->N;
    q.partial = (uint64_t*)(c->ws + c->lo.off_fused);
    q.hints = (uint32_t*)(q.partial + fused_small_partial_words(c->P, c->dims[0]));
    q.tag0 = c->fused_tag;
    q.err = c->flag() + 1;
    q.losses = c->losses();
    q.lr = c->lr; q.spin_limit = c->spin_limit;
    q.compute_units = c->compute_units;
    Bracket br(c, KAVG_CLASS_FORWARD);
    KAVG_HIP(c, launch_fused_small(q, st));
    c->fused_tag += (uint32_t)c->K;
    return KAVG_OK;
}

int issue_steps(kavg_ctx* c) {
    if (!c->cv.ch.empty()) return issue_steps_conv(c);
    if (c->refresh > 1) return issue_steps_deferred(c);
    hipStream_t st = c->stream;
    const bool bf = c->dtype == KAVG_BF16;
    const int L = c->L;

    // With few classes the last layer runs as two dedicated kernels (forward + loss + data gradient,
    // then its update) instead of four generic launches.
    const bool head = head_supported(c->dims[L]);
    for (int k = 0; k < c->K; ++k) {
        const int32_t* idx_k = c->idx() + (size_t)k * c->B;
        const long idx_ls = (long)c->K * c->B;
        float* rowloss_k = c->rowloss() + (size_t)k * c->P * c->B;
        for (int l = 1; l <= (head ? L - 1 : L); ++l) {      // forward
            LayerCall q = layer_call(c, l, k);
            Bracket br(c, KAVG_CLASS_FORWARD);
            KAVG_HIP(c, bf ? bf16_forward(q, st) : f32_forward(q, st));
        }
        if (head) {
            LayerCall q = layer_call(c, L, k);
            Bracket br(c, KAVG_CLASS_HEAD);
            KAVG_HIP(c, head_forward_backward(q, c->y, idx_k, idx_ls, rowloss_k, bf ? 1 : 0, st));
        } else {
            Bracket br(c, KAVG_CLASS_LOSS);
            KAVG_HIP(c, launch_softmax_ce(c->logits(), c->lo.ldz, c->dims[L], c->y, idx_k, idx_ls, c->B, c->P,
                                          c->ws + c->lo.off_dz[L - 1], (long)c->B * c->lo.ldz, bf ? 1 : 0, rowloss_k, st));
        }
        for (int l = L; l >= 1; --l) {                       // backward; W_l is read before it is updated
            LayerCall q = layer_call(c, l, k);
            if (head && l == L) {
                Bracket br(c, KAVG_CLASS_HEAD);
                KAVG_HIP(c, head_update(q, idx_k, idx_ls, bf ? 1 : 0, st));
                continue;
            }
            if (l > 1) {
                Bracket br(c, KAVG_CLASS_BACKWARD);
                KAVG_HIP(c, bf ? bf16_backward_data(q, st) : f32_backward_data(q, st));
            }
            Bracket br(c, KAVG_CLASS_UPDATE);
            KAVG_HIP(c, bf ? bf16_update(q, st) : f32_update(q, st));
        }
    }
    {
        Bracket br(c, KAVG_CLASS_LOSS);
        KAVG_HIP(c, launch_loss_mean(c->rowloss(), c->losses(), c->K * c->P, c->B, st));
    }
    return KAVG_OK;
}

// ---- deferred weight updates ----------------------------------------------------------------
// Algorithm 1's local step adds -lr dZ_k^T A_k to the learner's weights.  With a refresh period m > 1
// the stored replica is only brought up to date every m steps (one product over m*B samples instead
// of m read-modify-write passes over the master); in between, a product with the current weights
// W_k = W_0 - lr sum_{i<k} dZ_i^T A_i is formed as the product with the stored W_0 plus
//     forward:        - lr (A  H^T) G        H = [A_0; ..; A_{k-1}] inputs of the layer, G = [dZ_0; ..] its dZ
//     backward-data:  - lr (dZ G^T) H
// where the inner factors are B x kB matrices.  Activations and dZ of the steps since the last refresh
// are kept (the per-step buffers become slots of [P][m*B][d] histories); biases are stepped at once.
extern "C++" HistoryLayout history_layout(const kavg_ctx* c, int m) {
    HistoryLayout h;
    const int L = c->L;
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = round_up(p + bytes, ALIGN); return at; };
    h.act.assign(L, 0);
    h.dz.assign(L, 0);
    h.maxld = c->lo.ldz;
    for (int l = 1; l <= L; ++l) {
        const size_t ld = l == L ? (size_t)c->lo.ldz : (size_t)c->dims[l];
        if ((int)ld > h.maxld) h.maxld = (int)ld;
        if (l < L) h.act[l - 1] = take((size_t)c->P * m * c->B * ld * 2);
        h.dz[l - 1] = take((size_t)c->P * m * c->B * ld * 2);
    }
    // the fp32 buffer also receives raw backward products, as wide as the widest layer input it flows into
    for (int l = 1; l < L; ++l) if (c->dims[l] > h.maxld) h.maxld = c->dims[l];
    h.ldS = (int)round_up((size_t)m * c->B, 8);
    h.z0 = take((size_t)c->P * c->B * h.maxld * 4);
    h.s = take((size_t)c->P * c->B * h.ldS * 2);
    h.total = p;
    return h;
}

// The K local steps of a network whose MLP sits behind a stack of 3x3 convolutions (the CNN workloads
// of Section 4).  Per step a convolution is three products on B*H*W rows (forward, data gradient, weight
// gradient), and the mean over the positions joins the convolutions and the MLP.  Which kernels run them is
// decided per layer from its shape: the tile kernels for images 32 pixels wide (conv_first.hip,
// conv_direct.hip, conv_wgrad.hip), else the generic MFMA kernel on the implicit patch matrix, else (first
// layer, or images of 2^14 positions and more) the same kernel on a patch matrix that is written out.
int issue_steps_conv(kavg_ctx* c) {
    hipStream_t st = c->stream;
    const Layout& lo = c->lo;
    const ConvSpec& cv = c->cv;
    const int L = c->L, M = (int)cv.ch.size() - 1, P = c->P, B = c->B, H = cv.H, W = cv.W;
    const int rows = B * H * W;
    const bool head = head_supported(c->dims[L]);
    auto conv_call = [&](int t) {
        LayerCall q{};
        const int cin = 9 * cv.ch[t - 1], cout = cv.ch[t];
        q.P = P; q.B = rows; q.rows = rows; q.d_in = cin; q.d_out = cout;
        q.w_stride = lo.stride; q.ws_stride = lo.stride;
        q.ws = c->hi_planes() + lo.cw_off[t - 1];
        q.wlo = c->lo_planes() + lo.cw_off[t - 1];
        q.bhi = c->hi_planes() + lo.cb_off[t - 1];
        q.blo = c->lo_planes() + lo.cb_off[t - 1];
        q.shadow_cached = shadows_stay_cached(P, lo.stride);
        q.in = c->ws + lo.off_patch[t - 1]; q.ld_in = cin; q.in_stride = (size_t)rows * cin;
        q.out = c->ws + lo.off_cact[t - 1]; q.ld_out = cout; q.out_stride = (size_t)rows * cout;
        q.relu = 1;
        q.dz = c->ws + lo.off_cdz[t - 1]; q.ld_dz = cout; q.dz_stride = (size_t)rows * cout;
        q.lr = c->lr;
        return q;
    };
    auto implicit_call = [&](int t) {                               // convolution t >= 2 on the images of convolution t-1
        ConvCall v{};
        v.P = P; v.B = B; v.H = H; v.W = W; v.c_in = cv.ch[t - 1]; v.c_out = cv.ch[t];
        v.ws = c->hi_planes() + lo.cw_off[t - 1]; v.wlo = c->lo_planes() + lo.cw_off[t - 1]; v.ws_stride = lo.stride;
        v.bhi = c->hi_planes() + lo.cb_off[t - 1]; v.blo = c->lo_planes() + lo.cb_off[t - 1];
        v.in = c->ws + lo.off_cact[t - 2]; v.out = c->ws + lo.off_cact[t - 1];
        v.dz = c->ws + lo.off_cdz[t - 1]; v.dz_in = c->ws + lo.off_cdz[t - 2];
        v.wrot = (const uint16_t*)(c->ws + lo.off_wrot); v.wrot_stride = (size_t)9 * v.c_out * v.c_in;
        v.partial = (float*)(c->ws + lo.off_partial); v.partial_bias = (float*)(c->ws + lo.off_pbias);
        v.splits = lo.splits[t - 1];
        return v;
    };
    const bool first_direct = lo.conv_implicit && lo.splits_halo[0] > 0;   // the first convolution straight from the gathered images
    auto first_call = [&]() {
        ConvCall v{};
        v.P = P; v.B = B; v.H = H; v.W = W; v.c_in = cv.ch[0]; v.c_out = cv.ch[1];
        v.ws = c->hi_planes() + lo.cw_off[0]; v.wlo = c->lo_planes() + lo.cw_off[0]; v.ws_stride = lo.stride;
        v.bhi = c->hi_planes() + lo.cb_off[0]; v.blo = c->lo_planes() + lo.cb_off[0];
        v.out = c->ws + lo.off_cact[0]; v.dz = c->ws + lo.off_cdz[0];
        v.partial = (float*)(c->ws + lo.off_partial); v.partial_bias = (float*)(c->ws + lo.off_pbias);
        v.splits = lo.splits_halo[0];
        return v;
    };
    for (int k = 0; k < c->K; ++k) {
        const int32_t* idx_k = c->idx() + (size_t)k * B;
        const long idx_ls = (long)c->K * B;
        float* rowloss_k = c->rowloss() + (size_t)k * P * B;
        for (int t = 1; t <= M; ++t) {                              // convolutions, forward
            Bracket br(c, KAVG_CLASS_FORWARD);
            if (t == 1 && first_direct) {
                KAVG_HIP(c, conv_first_forward(first_call(), c->X, idx_k, idx_ls, st));
                continue;
            }
            if (t > 1 && lo.conv_implicit) {
                if (conv_direct_ok(H, W, cv.ch[t - 1], cv.ch[t], false)) KAVG_HIP(c, conv_direct_forward(implicit_call(t), st));
                else KAVG_HIP(c, bf16_conv_forward(implicit_call(t), st));
                continue;
            }
            if (t == 1)
                KAVG_HIP(c, launch_im2col(c->X, 0, idx_k, idx_ls, c->ws + lo.off_patch[0], P, B, H, W, cv.ch[0], st));
            else
                KAVG_HIP(c, launch_im2col(c->ws + lo.off_cact[t - 2], (size_t)rows * cv.ch[t - 1], nullptr, 0,
                                          c->ws + lo.off_patch[t - 1], P, B, H, W, cv.ch[t - 1], st));
            KAVG_HIP(c, bf16_forward(conv_call(t), st));
        }
        {
            Bracket br(c, KAVG_CLASS_FORWARD);
            KAVG_HIP(c, launch_pool_forward(c->ws + lo.off_cact[M - 1], c->ws + lo.off_pool, P, B, H * W, cv.ch[M], st));
        }
        for (int l = 1; l <= (head ? L - 1 : L); ++l) {             // MLP, forward
            Bracket br(c, KAVG_CLASS_FORWARD);
            KAVG_HIP(c, bf16_forward(layer_call(c, l, k), st));
        }
        if (head) {
            Bracket br(c, KAVG_CLASS_HEAD);
            KAVG_HIP(c, head_forward_backward(layer_call(c, L, k), c->y, idx_k, idx_ls, rowloss_k, 1, st));
        } else {
            Bracket br(c, KAVG_CLASS_LOSS);
            KAVG_HIP(c, launch_softmax_ce(c->logits(), lo.ldz, c->dims[L], c->y, idx_k, idx_ls, B, P,
                                          c->ws + lo.off_dz[L - 1], (long)B * lo.ldz, 1, rowloss_k, st));
        }
        for (int l = L; l >= 1; --l) {                              // MLP, backward; layer 1 hands dL/d(pooled) on
            LayerCall q = layer_call(c, l, k);
            if (head && l == L) {
                Bracket br(c, KAVG_CLASS_HEAD);
                KAVG_HIP(c, head_update(q, idx_k, idx_ls, 1, st));
                continue;
            }
            {
                Bracket br(c, KAVG_CLASS_BACKWARD);
                KAVG_HIP(c, bf16_backward_data(q, st));
            }
            Bracket br(c, KAVG_CLASS_UPDATE);
            KAVG_HIP(c, bf16_update(q, st));
        }
        // The gradient of the mean over the positions: written out for the generic kernels; the tile kernels of
        // the last convolution form it while loading (both of them must be in use, or the buffer is needed).
        const bool pool_fused = M > 1 && lo.conv_implicit && lo.splits_halo[M - 1] > 0 &&
                                B / lo.splits_halo[M - 1] <= conv_wgrad_halo_pool_images() &&
                                conv_direct_ok(H, W, cv.ch[M - 1], cv.ch[M], true);
        const void* dpool_M = c->ws + lo.off_dpool;
        if (!pool_fused) {
            Bracket br(c, KAVG_CLASS_BACKWARD);
            KAVG_HIP(c, launch_pool_backward(c->ws + lo.off_dpool, c->ws + lo.off_cact[M - 1], c->ws + lo.off_cdz[M - 1],
                                             P, B, H * W, cv.ch[M], st));
        }
        for (int t = M; t >= 1; --t) {                              // convolutions, backward
            if (t > 1 && lo.conv_implicit) {
                ConvCall v = implicit_call(t);
                {
                    Bracket br(c, KAVG_CLASS_BACKWARD);
                    if (conv_direct_ok(H, W, v.c_in, v.c_out, true)) {
                        KAVG_HIP(c, conv_direct_backward_data(v, (pool_fused && t == M) ? dpool_M : nullptr, st));
                    } else {
                        KAVG_HIP(c, launch_rotate_weights(v.ws, lo.stride, (uint16_t*)(c->ws + lo.off_wrot), v.wrot_stride, P,
                                                          v.c_out, v.c_in, st));
                        KAVG_HIP(c, bf16_conv_backward_data(v, st));
                    }
                }
                Bracket br(c, KAVG_CLASS_UPDATE);
                if (lo.splits_halo[t - 1] > 0) {
                    v.splits = lo.splits_halo[t - 1];
                    KAVG_HIP(c, conv_wgrad_halo(v, (pool_fused && t == M) ? dpool_M : nullptr, st));
                } else {
                    KAVG_HIP(c, bf16_conv_update_partial(v, st));
                }
                KAVG_HIP(c, launch_conv_step(v.ws, v.wlo, (uint16_t*)v.bhi, (uint16_t*)v.blo, lo.stride, v.partial, v.partial_bias,
                                             P, v.splits, v.c_out * 9 * v.c_in, v.c_out, c->lr, st));
                continue;
            }
            if (t == 1 && first_direct) {
                Bracket br(c, KAVG_CLASS_UPDATE);
                ConvCall v = first_call();
                KAVG_HIP(c, conv_first_wgrad(v, c->X, idx_k, idx_ls, st));
                KAVG_HIP(c, launch_conv_step(v.ws, v.wlo, (uint16_t*)v.bhi, (uint16_t*)v.blo, lo.stride, v.partial, v.partial_bias,
                                             P, v.splits, v.c_out * 9 * v.c_in, v.c_out, c->lr, st));
                continue;
            }
            LayerCall q = conv_call(t);
            if (t > 1) {
                Bracket br(c, KAVG_CLASS_BACKWARD);
                LayerCall r = q;
                r.bwd_raw = 1;
                r.dz_prev = c->ws + lo.off_draw; r.dz_prev_stride = (size_t)rows * q.d_in;
                KAVG_HIP(c, bf16_backward_data(r, st));
                KAVG_HIP(c, launch_col2im_mask((const float*)(c->ws + lo.off_draw), c->ws + lo.off_cact[t - 2],
                                               c->ws + lo.off_cdz[t - 2], P, B, H, W, cv.ch[t - 1], st));
            }
            Bracket br(c, KAVG_CLASS_UPDATE);
            q.partial = (float*)(c->ws + lo.off_partial);
            q.partial_bias = (float*)(c->ws + lo.off_pbias);
            q.splits = lo.splits[t - 1];
            KAVG_HIP(c, bf16_update(q, st));
            KAVG_HIP(c, launch_conv_step((uint16_t*)q.ws, (uint16_t*)q.wlo, (uint16_t*)q.bhi, (uint16_t*)q.blo, lo.stride,
                                         q.partial, q.partial_bias, P, q.splits, q.d_out * q.d_in, q.d_out, c->lr, st));
        }
    }
    {
        Bracket br(c, KAVG_CLASS_LOSS);
        KAVG_HIP(c, launch_loss_mean(c->rowloss(), c->losses(), c->K * P, B, st));
    }
    return KAVG_OK;
}

int issue_steps_deferred(kavg_ctx* c) {
    hipStream_t st = c->stream;
    const int L = c->L, P = c->P, B = c->B, K = c->K, m = c->refresh;
    const Layout& lo = c->lo;
    const bool head = head_supported(c->dims[L]);
    const int Lw = head ? L - 1 : L;                  // layers whose weights are kept deferred
    auto ld_of = [&](int l) { return l == L ? lo.ldz : c->dims[l]; };
    auto actH = [&](int l, int slot) { return c->hist + c->hl.act[l - 1] + (size_t)slot * B * c->dims[l] * 2; };
    auto dzH = [&](int l, int slot) { return c->hist + c->hl.dz[l - 1] + (size_t)slot * B * ld_of(l) * 2; };
    float* z0 = (float*)(c->hist + c->hl.z0);
    uint16_t* S = (uint16_t*)(c->hist + c->hl.s);
    const size_t z0_stride = (size_t)B * c->hl.maxld, S_stride = (size_t)B * c->hl.ldS;
    const long idx_ls = (long)K * B;

    // the launch description of layer l at step k, operands in their history slots
    auto call = [&](int l, int k, int slot) {
        LayerCall q = {};
        q.P = P; q.B = B; q.d_in = c->dims[l - 1]; q.d_out = c->dims[l];
        q.w_stride = lo.stride; q.ws_stride = lo.stride;
        q.ws = c->hi_planes() + lo.w_off[l - 1];  q.wlo = c->lo_planes() + lo.w_off[l - 1];
        q.bhi = c->hi_planes() + lo.b_off[l - 1]; q.blo = c->lo_planes() + lo.b_off[l - 1];
        q.shadow_cached = shadows_stay_cached(P, lo.stride);
        if (l == 1) {
            q.in = c->X; q.ld_in = c->dims[0]; q.in_stride = 0;
            q.gather = c->idx() + (size_t)k * B; q.gather_stride = idx_ls;
        } else {
            q.in = actH(l - 1, slot); q.ld_in = c->dims[l - 1]; q.in_stride = (size_t)m * B * q.ld_in;
            q.dz_prev = dzH(l - 1, slot); q.dz_prev_stride = (size_t)m * B * q.ld_in;
        }
        if (l < L) { q.out = actH(l, slot); q.ld_out = c->dims[l]; q.out_stride = (size_t)m * B * q.ld_out; q.relu = 1; }
        else { q.out = c->logits(); q.ld_out = lo.ldz; q.out_stride = (size_t)B * lo.ldz; q.relu = 0; }
        q.dz = dzH(l, slot); q.ld_dz = ld_of(l); q.dz_stride = (size_t)m * B * q.ld_dz;
        q.lr = c->lr;
        // until the first refresh of a round every stored replica still holds the global model: all
        // learners then read learner 0's copy, which the caches serve, instead of P copies from memory
        q.shared_w = (c->replicas_equal && k < m) ? 1 : 0;
        return q;
    };

    for (int k = 0; k < K; ++k) {
        const int slot = k % m, cnt = slot;           // cnt steps' updates are pending
        const int32_t* idx_k = c->idx() + (size_t)k * B;
        const int32_t* idx_hist = c->idx() + (size_t)(k - cnt) * B;      // rows of the pending steps, cnt*B per learner
        float* rowloss_k = c->rowloss() + (size_t)k * P * B;
        for (int l = 1; l <= Lw; ++l) {                                  // forward
            LayerCall q = call(l, k, slot);
            if (cnt == 0) {
                Bracket br(c, KAVG_CLASS_FORWARD);
                KAVG_HIP(c, bf16_forward(q, st));
                continue;
            }
            const int ld = ld_of(l);
            {
                Bracket br(c, KAVG_CLASS_FORWARD);
                LayerCall q0 = q;                                        // stored weights, bias included, fp32
                q0.out = z0; q0.ld_out = ld; q0.out_stride = z0_stride; q0.relu = 0;
                KAVG_HIP(c, bf16_forward(q0, st));
            }
            Bracket br(c, KAVG_CLASS_CORRECTION);
            GramCall g = {};
            g.P = P; g.nR = B; g.nC = cnt * B; g.nK = q.d_in;
            g.R = q.in; g.ldR = q.ld_in; g.R_stride = q.in_stride; g.R_gather = q.gather; g.R_gstride = idx_ls;
            g.ldC = q.ld_in;
            if (l == 1) { g.C = c->X; g.C_stride = 0; g.C_gather = idx_hist; g.C_gstride = idx_ls; }
            else { g.C = actH(l - 1, 0); g.C_stride = q.in_stride; }
            g.out = S; g.ld_out = c->hl.ldS; g.out_stride = S_stride; g.alpha = -c->lr;
            KAVG_HIP(c, bf16_gram(g, st));
            ApplyCall ap = {};
            ap.P = P; ap.nR = B; ap.nC = ld; ap.nC_cont = ld; ap.nK = cnt * B;
            ap.S = S; ap.ldS = c->hl.ldS; ap.S_stride = S_stride;
            ap.M = dzH(l, 0); ap.ldM = ld; ap.M_stride = (size_t)m * B * ld;
            ap.base = z0; ap.ld_base = ld; ap.base_stride = z0_stride;
            ap.epi = l < L ? KAVG_APPLY_RELU : KAVG_APPLY_LOGITS;
            ap.out = q.out; ap.ld_out = q.ld_out; ap.out_stride = q.out_stride;
            KAVG_HIP(c, bf16_apply(ap, st));
        }
        if (head) {
            LayerCall q = call(L, k, slot);
            Bracket br(c, KAVG_CLASS_HEAD);
            KAVG_HIP(c, head_forward_backward(q, c->y, idx_k, idx_ls, rowloss_k, 1, st));
        } else {
            Bracket br(c, KAVG_CLASS_LOSS);
            KAVG_HIP(c, launch_softmax_ce(c->logits(), lo.ldz, c->dims[L], c->y, idx_k, idx_ls, B, P, dzH(L, slot),
                                          (long)m * B * lo.ldz, 1, rowloss_k, st));
        }
        for (int l = L; l >= 1; --l) {                                   // backward
            LayerCall q = call(l, k, slot);
            if (head && l == L) {
                Bracket br(c, KAVG_CLASS_HEAD);
                KAVG_HIP(c, head_update(q, idx_k, idx_ls, 1, st));       // the thin last layer is stepped at once
                continue;
            }
            if (l > 1) {
                if (cnt == 0) {
                    Bracket br(c, KAVG_CLASS_BACKWARD);
                    KAVG_HIP(c, bf16_backward_data(q, st));
                } else {
                    {
                        Bracket br(c, KAVG_CLASS_BACKWARD);
                        LayerCall q0 = q;
                        q0.bwd_raw = 1; q0.dz_prev = z0; q0.dz_prev_stride = z0_stride;
                        KAVG_HIP(c, bf16_backward_data(q0, st));
                    }
                    Bracket br(c, KAVG_CLASS_CORRECTION);
                    GramCall g = {};
                    g.P = P; g.nR = B; g.nC = cnt * B; g.nK = q.ld_dz;
                    g.R = q.dz; g.ldR = q.ld_dz; g.R_stride = q.dz_stride;
                    g.C = dzH(l, 0); g.ldC = q.ld_dz; g.C_stride = q.dz_stride;
                    g.out = S; g.ld_out = c->hl.ldS; g.out_stride = S_stride; g.alpha = -c->lr;
                    KAVG_HIP(c, bf16_gram(g, st));
                    ApplyCall ap = {};
                    ap.P = P; ap.nR = B; ap.nC = q.ld_in; ap.nC_cont = q.ld_in; ap.nK = cnt * B;
                    ap.S = S; ap.ldS = c->hl.ldS; ap.S_stride = S_stride;
                    ap.M = actH(l - 1, 0); ap.ldM = q.ld_in; ap.M_stride = q.in_stride;
                    ap.base = z0; ap.ld_base = q.ld_in; ap.base_stride = z0_stride;
                    ap.epi = KAVG_APPLY_MASK; ap.act = q.in; ap.ld_act = q.ld_in; ap.act_stride = q.in_stride;
                    ap.out = q.dz_prev; ap.ld_out = q.ld_in; ap.out_stride = q.dz_prev_stride;
                    KAVG_HIP(c, bf16_apply(ap, st));
                }
            }
            Bracket br(c, KAVG_CLASS_UPDATE);
            KAVG_HIP(c, launch_bias_step(q.bhi, q.blo, lo.stride, q.dz, q.ld_dz, q.dz_stride, P, B, q.d_out, c->lr, st));
        }
        if (slot == m - 1 || k == K - 1) {                               // bring the stored replicas up to date
            for (int l = 1; l <= Lw; ++l) {
                LayerCall q = call(l, k, 0);
                q.rows = (slot + 1) * B; q.skip_bias = 1;
                if (l == 1) q.gather = idx_hist;
                Bracket br(c, KAVG_CLASS_UPDATE);
                KAVG_HIP(c, bf16_update(q, st));
            }
        }
    }
    {
        Bracket br(c, KAVG_CLASS_LOSS);
        KAVG_HIP(c, launch_loss_mean(c->rowloss(), c->losses(), K * P, B, st));
    }
    return KAVG_OK;
}

// forget the recorded sequence: its arguments (data, velocity buffer) are about to change
void drop_graph(kavg_ctx* c) {
    if (c->gexec) {
        (void)hipStreamSynchronize(c->stream);           // it may still be running
        (void)hipGraphExecDestroy(c->gexec);
        c->gexec = nullptr;
    }
    c->warm = false;
}

}  // namespace

int kavg_local_steps(kavg_ctx* c) {
    if (!c) return KAVG_EINVAL;
    if (!c->have_params) return fail(c, KAVG_ESTATE, "no parameters: call kavg_set_params first");
    if (!c->X) return fail(c, KAVG_ESTATE, "no data set: call kavg_set_data first");
    if ((uint64_t)c->t0 + (uint64_t)c->K > ((uint64_t)1 << 24))
        return fail(c, KAVG_ESTATE, "local step counter would exceed 2^24");
    hipStream_t st = c->stream;
    KAVG_NOTHROW_BEGIN
    const bool fused = fused_now(c);
    {
        Bracket br(c, KAVG_CLASS_INDEX);
        if (c->user_idx)
            KAVG_HIP(c, launch_index_import(c->idx(), c->user_idx, (size_t)c->P * c->K * c->B, (uint32_t)c->N,
                                            c->flag(), st));
        else if (!fused)                        // (the fused launch draws its own indices)
            KAVG_HIP(c, launch_index_stream(c->idx(), c->P, c->K, c->B, c->seed, c->t0, (uint32_t)c->N, st));
    }
    if (fused) {
        const int rc = issue_steps_fused(c);
        if (rc != KAVG_OK) return rc;
        c->t0 += (uint32_t)c->K;
        c->have_steps = true;
        c->replicas_equal = false;
        return KAVG_OK;
    }

    // Everything after the indices has the same arguments in every round, so it can be replayed.
    if (c->graph_on && c->warm && c->prof_mask == 0) {
        if (!c->gexec) {
            hipGraph_t g = nullptr;
            KAVG_HIP(c, hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
            const int rc = issue_steps(c);
            const hipError_t e = hipStreamEndCapture(st, &g);      // always ends the capture
            if (rc != KAVG_OK) { if (g) (void)hipGraphDestroy(g); return rc; }
            KAVG_HIP(c, e);
            const hipError_t ei = hipGraphInstantiate(&c->gexec, g, nullptr, nullptr, 0);
            (void)hipGraphDestroy(g);
            if (ei != hipSuccess) { c->gexec = nullptr; KAVG_HIP(c, ei); }
        }
        KAVG_HIP(c, hipGraphLaunch(c->gexec, st));
    } else {
        const int rc = issue_steps(c);
        if (rc != KAVG_OK) return rc;
        c->warm = true;
    }
    c->t0 += (uint32_t)c->K;
    c->have_steps = true;
    c->replicas_equal = false;
    return KAVG_OK;
    KAVG_NOTHROW_END(c)
}

int kavg_meta_update(kavg_ctx* c) {
    if (!c) return KAVG_EINVAL;
    if (!c->have_params) return fail(c, KAVG_ESTATE, "no parameters: call kavg_set_params first");
    KAVG_NOTHROW_BEGIN
    {
        Bracket br(c, KAVG_CLASS_META);
        if (c->dtype == KAVG_BF16)
            KAVG_HIP(c, launch_meta_update_split(c->w_tilde(), c->v(), c->hi_planes(), c->lo_planes(), c->lo.stride,
                                                 c->P, c->lo.n, c->mu, shadows_stay_cached(c->P, c->lo.stride),
                                                 c->stream));
        else
            KAVG_HIP(c, launch_meta_update(c->w_tilde(), c->v(), c->reps(), c->lo.stride, nullptr, c->lo.stride,
                                           c->P, c->lo.n, c->mu, 0, c->stream));
    }
    c->round += 1;
    c->replicas_equal = true;
    return KAVG_OK;
    KAVG_NOTHROW_END(c)
}

static int copy_out(kavg_ctx* c, const void* src, void* dst_host, size_t bytes) {
    KAVG_HIP(c, hipMemcpyAsync(dst_host, src, bytes, hipMemcpyDeviceToHost, c->stream));
    return sync_and_check(c);
}

int kavg_params(kavg_ctx* c, float* out_host, size_t n) {
    if (!c) return KAVG_EINVAL;
    if (!out_host || n != c->lo.n) return fail(c, KAVG_EINVAL, "need a buffer of exactly %zu floats", c->lo.n);
    if (!c->have_params) return fail(c, KAVG_ESTATE, "no parameters yet");
    return copy_out(c, c->w_tilde(), out_host, n * 4);
}

int kavg_momentum(kavg_ctx* c, float* out_host, size_t n) {
    if (!c) return KAVG_EINVAL;
    if (!out_host || n != c->lo.n) return fail(c, KAVG_EINVAL, "need a buffer of exactly %zu floats", c->lo.n);
    if (!c->have_params) return fail(c, KAVG_ESTATE, "no parameters yet");
    return copy_out(c, c->v(), out_host, n * 4);
}

int kavg_replica(kavg_ctx* c, int j, float* out_host, size_t n) {
    if (!c) return KAVG_EINVAL;
    if (!out_host || n != c->lo.n) return fail(c, KAVG_EINVAL, "need a buffer of exactly %zu floats", c->lo.n);
    if (j < 0 || j >= c->P) return fail(c, KAVG_EINVAL, "learner %d outside [0,%d)", j, c->P);
    if (!c->have_params) return fail(c, KAVG_ESTATE, "no parameters yet");
    if (c->dtype != KAVG_BF16) return copy_out(c, c->reps() + (size_t)j * c->lo.stride, out_host, n * 4);
    // bf16 mode: fetch the learner's two planes and join them into fp32 values on the host
    KAVG_NOTHROW_BEGIN
    std::vector<uint16_t> hi(n), lo(n);
    int rc = copy_out(c, c->hi_planes() + (size_t)j * c->lo.stride, hi.data(), n * 2);
    if (rc == KAVG_OK) rc = copy_out(c, c->lo_planes() + (size_t)j * c->lo.stride, lo.data(), n * 2);
    if (rc != KAVG_OK) return rc;
    for (size_t e = 0; e < n; ++e) {
        const uint32_t bits = split_join(hi[e], lo[e]);
        memcpy(out_host + e, &bits, 4);
    }
    return KAVG_OK;
    KAVG_NOTHROW_END(c)
}

int kavg_losses(kavg_ctx* c, float* out_host) {
    if (!c) return KAVG_EINVAL;
    if (!out_host) return fail(c, KAVG_EINVAL, "out_host is null");
    if (!c->have_steps) return fail(c, KAVG_ESTATE, "no local steps taken yet");
    return copy_out(c, c->losses(), out_host, (size_t)c->K * c->P * 4);
}

int kavg_indices(kavg_ctx* c, int32_t* out_host) {
    if (!c) return KAVG_EINVAL;
    if (!out_host) return fail(c, KAVG_EINVAL, "out_host is null");
    if (!c->have_steps) return fail(c, KAVG_ESTATE, "no local steps taken yet");
    return copy_out(c, c->idx(), out_host, (size_t)c->P * c->K * c->B * 4);
}

static int prof_drain(kavg_ctx* c) {
    KAVG_HIP(c, hipStreamSynchronize(c->stream));
    for (int k = 0; k < KAVG_NCLASS; ++k) {
        for (size_t i = 0; i + 1 < c->prof_used[k]; i += 2) {
            float ms = 0.f;
            KAVG_HIP(c, hipEventElapsedTime(&ms, c->prof_ev[k][i], c->prof_ev[k][i + 1]));
            c->prof_ms[k] += ms;
            c->prof_launches[k] += 1;
        }
        c->prof_used[k] = 0;
    }
    return KAVG_OK;
}

int kavg_profile(kavg_ctx* c, unsigned class_mask, unsigned every) {
    if (!c) return KAVG_EINVAL;
    if (class_mask >> KAVG_NCLASS) return fail(c, KAVG_EINVAL, "unknown kernel class in mask");
    if (every < 1) return fail(c, KAVG_EINVAL, "every must be >= 1");
    int rc = prof_drain(c);
    if (rc != KAVG_OK) return rc;
    for (int k = 0; k < KAVG_NCLASS; ++k) { c->prof_ms[k] = 0.0; c->prof_launches[k] = 0; c->prof_seen[k] = 0; }
    c->prof_mask = class_mask;
    c->prof_every = every;
    return KAVG_OK;
}

int kavg_profile_read(kavg_ctx* c, double* ms_out, long long* launches_out) {
    if (!c) return KAVG_EINVAL;
    if (!ms_out || !launches_out) return fail(c, KAVG_EINVAL, "null output");
    int rc = prof_drain(c);
    if (rc != KAVG_OK) return rc;
    for (int k = 0; k < KAVG_NCLASS; ++k) { ms_out[k] = c->prof_ms[k]; launches_out[k] = c->prof_launches[k]; }
    return KAVG_OK;
}

int kavg_graph(kavg_ctx* c, int on) {
    if (!c) return KAVG_EINVAL;
    if (on && c->stream == nullptr)
        return fail(c, KAVG_ESTATE, "graph replay needs a stream of its own: the default stream cannot be captured");
    if (!on) {
        KAVG_HIP(c, hipStreamSynchronize(c->stream));
        if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
    }
    c->graph_on = on != 0;
    return KAVG_OK;
}

size_t kavg_velocity_bytes(const kavg_ctx* c) { return c ? (size_t)c->P * c->lo.stride * 4 : 0; }

int kavg_set_learner_momentum(kavg_ctx* c, float beta, void* velocity_dev, size_t bytes) {
    if (!c) return KAVG_EINVAL;
    if (!(beta >= 0.f && beta < 1.f)) return fail(c, KAVG_EINVAL, "beta must lie in [0,1)");
    if (beta == 0.f || !velocity_dev) {
        if (beta != 0.f) return fail(c, KAVG_EINVAL, "beta > 0 needs a velocity buffer");
        KAVG_HIP(c, hipStreamSynchronize(c->stream));
        c->beta = 0.f; c->vel = nullptr;
        drop_graph(c);
        return KAVG_OK;
    }
    if (c->refresh > 1) return fail(c, KAVG_ESTATE, "deferred updates and learner-level momentum exclude each other");
    if (!c->cv.ch.empty()) return fail(c, KAVG_EINVAL, "learner-level momentum is not built for convolutional contexts");
    if (((uintptr_t)velocity_dev % ALIGN) != 0) return fail(c, KAVG_EINVAL, "velocity buffer must be 256-byte aligned");
    if (bytes < kavg_velocity_bytes(c)) return fail(c, KAVG_ENOMEM, "velocity buffer has %zu bytes, %zu needed", bytes, kavg_velocity_bytes(c));
    KAVG_HIP(c, hipMemsetAsync(velocity_dev, 0, kavg_velocity_bytes(c), c->stream));
    c->beta = beta; c->vel = (float*)velocity_dev;
    drop_graph(c);
    return KAVG_OK;
}

int kavg_velocity(kavg_ctx* c, int j, float* out_host, size_t n) {
    if (!c) return KAVG_EINVAL;
    if (!out_host || n != c->lo.n) return fail(c, KAVG_EINVAL, "need a buffer of exactly %zu floats", c->lo.n);
    if (j < 0 || j >= c->P) return fail(c, KAVG_EINVAL, "learner %d outside [0,%d)", j, c->P);
    if (!c->vel) return fail(c, KAVG_ESTATE, "learner-level momentum is off");
    KAVG_HIP(c, hipMemcpyAsync(out_host, c->vel + (size_t)j * c->lo.stride, n * 4, hipMemcpyDeviceToHost, c->stream));
    return sync_and_check(c);
}

size_t kavg_refresh_bytes(const kavg_ctx* c, int refresh) {
    if (!c || refresh < 2 || refresh > c->K || c->dtype != KAVG_BF16) return 0;
    try { return history_layout(c, refresh).total; } catch (...) { return 0; }
}

int kavg_set_refresh(kavg_ctx* c, int refresh, void* history_dev, size_t bytes) {
    if (!c) return KAVG_EINVAL;
    KAVG_NOTHROW_BEGIN
    if (refresh < 1 || refresh > c->K) return fail(c, KAVG_EINVAL, "refresh period must lie in [1, K]");
    KAVG_HIP(c, hipStreamSynchronize(c->stream));
    if (refresh == 1) {
        c->refresh = 1; c->hist = nullptr;
        drop_graph(c);
        return KAVG_OK;
    }
    if (c->dtype != KAVG_BF16) return fail(c, KAVG_EINVAL, "deferred updates are built for KAVG_BF16 only");
    if (!c->cv.ch.empty()) return fail(c, KAVG_EINVAL, "deferred updates are not built for convolutional contexts");
    if (c->vel) return fail(c, KAVG_ESTATE, "deferred updates and learner-level momentum exclude each other");
    if (!history_dev || ((uintptr_t)history_dev % ALIGN) != 0)
        return fail(c, KAVG_EINVAL, "history block must be a non-null, 256-byte aligned device pointer");
    HistoryLayout h = history_layout(c, refresh);
    if (bytes < h.total) return fail(c, KAVG_ENOMEM, "history block has %zu bytes, %zu needed", bytes, h.total);
    c->hl = h; c->refresh = refresh; c->hist = (char*)history_dev;
    drop_graph(c);
    return KAVG_OK;
    KAVG_NOTHROW_END(c)
}

uint64_t kavg_round(const kavg_ctx* c) { return c ? c->round : 0; }

const char* kavg_last_error(const kavg_ctx* c) { return c ? c->err : g_init_error; }

int kavg_destroy(kavg_ctx* c) {
    if (!c) return KAVG_EINVAL;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (c->static_dev >= 0 && g_static_owner[c->static_dev] == c) g_static_owner[c->static_dev] = nullptr;
    if (c->gexec) (void)hipGraphExecDestroy(c->gexec);
    for (int k = 0; k < KAVG_NCLASS; ++k)
        for (hipEvent_t ev : c->prof_ev[k]) (void)hipEventDestroy(ev);
    delete c;
    return e == hipSuccess ? KAVG_OK : KAVG_EDEVICE;
}

int kavg_meta_update_flat(float* w_tilde_dev, float* v_dev, float* replicas_dev, size_t replica_stride,
                          uint16_t* shadow_dev, size_t shadow_stride, int P, size_t n, float mu,
                          void* hip_stream) {
    if (!w_tilde_dev || !v_dev || !replicas_dev) return KAVG_EINVAL;
    if (P < 1 || n < 1 || replica_stride < n || !(mu >= 0.f && mu < 1.f)) return KAVG_EINVAL;
    if (shadow_dev && shadow_stride < n) return KAVG_EINVAL;
    hipError_t e = launch_meta_update(w_tilde_dev, v_dev, replicas_dev, replica_stride, shadow_dev,
                                      shadow_stride, P, n, mu, shadows_stay_cached(P, n), (hipStream_t)hip_stream);
    return e == hipSuccess ? KAVG_OK : KAVG_EDEVICE;
}

int kavg_probe(int kind, void* a_dev, void* b_dev, size_t bytes, int iters, float* sink_dev, void* hip_stream,
               double* work_out) {
    if (kind < KAVG_PROBE_READ || kind > KAVG_PROBE_MFMA || !sink_dev || !work_out) return KAVG_EINVAL;
    if (kind == KAVG_PROBE_MFMA) {
        if (iters < 1) return KAVG_EINVAL;
    } else {
        if (!a_dev || ((uintptr_t)a_dev & 15) || bytes < 256) return KAVG_EINVAL;
        if (kind == KAVG_PROBE_COPY && (!b_dev || ((uintptr_t)b_dev & 15))) return KAVG_EINVAL;
    }
    const hipError_t e = launch_probe(kind, a_dev, b_dev, bytes, iters, sink_dev, (hipStream_t)hip_stream, work_out);
    return e == hipSuccess ? KAVG_OK : KAVG_EDEVICE;
}

}  // extern "C"
