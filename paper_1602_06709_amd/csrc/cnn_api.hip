// C-ABI entry points: argument validation, kernel selection, error reporting.
#include <mutex>
#include <new>
#include <stdio.h>
#include <string.h>

#include "common.h"

namespace cnn {

int hip_check(cnn_ctx* ctx, hipError_t e, const char* what) {
    if (e == hipSuccess) return CNN_OK;
    if (ctx) snprintf(ctx->err, sizeof(ctx->err), "%s: %s", what, hipGetErrorString(e));
    return CNN_EHIP;
}
int launch_check(cnn_ctx* ctx, const char* what) { return hip_check(ctx, hipGetLastError(), what); }

int lds_attr_once(cnn_ctx* ctx, std::atomic<unsigned long long>& done, const void* fn, int bytes, const char* what) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_check(ctx, e, "hipGetDevice");
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return CNN_OK;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return hip_check(ctx, e, what);
    done.fetch_or(bit, std::memory_order_release);
    return CNN_OK;
}

ProfScope::ProfScope(cnn_ctx* c, const char* name, double flops) : ctx(c), ent(nullptr) {
    if (!c || !c->profile || c->prof_used >= 16384) return;
    if (c->prof_used == c->prof.size()) {
        ProfEntry e{name, flops, nullptr, nullptr};
        if (hipEventCreate(&e.e0) != hipSuccess) return;
        if (hipEventCreate(&e.e1) != hipSuccess) { (void)hipEventDestroy(e.e0); return; }
        c->prof.push_back(e);
    }
    ent = &c->prof[c->prof_used++];
    ent->name = name;
    ent->flops = flops;
    (void)hipEventRecord(ent->e0, c->stream);
}
ProfScope::~ProfScope() {
    if (ent) (void)hipEventRecord(ent->e1, ctx->stream);
}

}  // namespace cnn

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Fills the shape and checks the paper's layer parameters (Section 2.1: minibatch, ifm, ofm, out_h, out_w,
// k_h, k_w, stride).  Tensors are indexed with 32-bit element offsets inside the kernels.
int make_shape(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, ConvShape* s) {
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride < 1 || pad < 0) return CNN_EINVAL;
    const int P = cnn::out_dim(H, R, stride, pad), Q = cnn::out_dim(W, S, stride, pad);
    if (P <= 0 || Q <= 0) return CNN_EINVAL;
    const double lim = 2147483647.0;
    if ((double)N * C * H * W > lim || (double)N * K * P * Q > lim || (double)K * C * R * S > lim) return CNN_EUNSUPPORTED;
    *s = ConvShape{N, C, H, W, K, R, S, stride, pad, P, Q};
    return CNN_OK;
}

}  // namespace

// ---- The allocation-free variant of cnn_conv_bwd_weight: its partial sums live in a device array that is part of
// the library's code object instead of a caller's workspace.  `scratch` is a host-side stand-in for the array, not
// a device address: host code only ever uses the per-device pointer hipGetSymbolAddress returns for it.
static __device__ __align__(256) unsigned char scratch[CNN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // each device holds its own copy of the array at its own address

// The current device's copy of `scratch`; looked up once per device, with that device current.
int static_scratch(cnn_ctx* ctx, void** out) {
    int dev = -1;
    int st = cnn::hip_check(ctx, hipGetDevice(&dev), "hipGetDevice");
    if (st != CNN_OK) return st;
    if (dev < 0 || dev >= kMaxDevices) return CNN_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        st = cnn::hip_check(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (st != CNN_OK) return st;
        if (!p) return CNN_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CNN_OK;
}
}  // namespace

extern "C" {

int cnn_create(cnn_ctx** out, void* hip_stream) {
    if (!out) return CNN_EINVAL;
    cnn_ctx* c = new (std::nothrow) cnn_ctx;
    if (!c) return CNN_EINVAL;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->force_direct = 0;
    c->profile = 0;
    c->prof_used = 0;
    c->err[0] = 0;
    *out = c;
    return CNN_OK;
}
int cnn_destroy(cnn_ctx* ctx) {
    if (!ctx) return CNN_EINVAL;
    for (ProfEntry& e : ctx->prof) {
        (void)hipEventDestroy(e.e0);
        (void)hipEventDestroy(e.e1);
    }
    delete ctx;
    return CNN_OK;
}
int cnn_set_stream(cnn_ctx* ctx, void* hip_stream) {
    if (!ctx) return CNN_EINVAL;
    ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
    return CNN_OK;
}
int cnn_set_workspace(cnn_ctx* ctx, void* dev_ptr, size_t bytes) {
    if (!ctx || (bytes && !dev_ptr) || !aligned16(dev_ptr)) return CNN_EINVAL;
    ctx->ws = dev_ptr;
    ctx->ws_bytes = dev_ptr ? bytes : 0;
    return CNN_OK;
}
int cnn_set_option(cnn_ctx* ctx, int option, int value) {
    if (!ctx) return CNN_EINVAL;
    if (option == CNN_OPT_FORCE_DIRECT) { ctx->force_direct = value != 0; return CNN_OK; }
    if (option == CNN_OPT_PROFILE) { ctx->profile = value != 0; return CNN_OK; }
    return CNN_EINVAL;
}
const char* cnn_strerror(int status) {
    switch (status) {
        case CNN_OK: return "ok";
        case CNN_EINVAL: return "invalid argument";
        case CNN_EUNSUPPORTED: return "unsupported shape";
        case CNN_EWORKSPACE: return "workspace too small";
        case CNN_EHIP: return "HIP error";
        default: return "unknown status";
    }
}
const char* cnn_last_error(const cnn_ctx* ctx) { return ctx ? ctx->err : ""; }

int cnn_profile_count(const cnn_ctx* ctx) { return ctx ? (int)ctx->prof_used : CNN_EINVAL; }
int cnn_profile_get(cnn_ctx* ctx, int index, const char** kernel_name, double* flops, float* ms) {
    if (!ctx || index < 0 || (size_t)index >= ctx->prof_used) return CNN_EINVAL;
    ProfEntry& e = ctx->prof[index];
    int st = cnn::hip_check(ctx, hipEventSynchronize(e.e1), "hipEventSynchronize(profile)");
    if (st != CNN_OK) return st;
    float t = 0.f;
    st = cnn::hip_check(ctx, hipEventElapsedTime(&t, e.e0, e.e1), "hipEventElapsedTime(profile)");
    if (st != CNN_OK) return st;
    if (kernel_name) *kernel_name = e.name;
    if (flops) *flops = e.flops;
    if (ms) *ms = t;
    return CNN_OK;
}
int cnn_profile_reset(cnn_ctx* ctx) {
    if (!ctx) return CNN_EINVAL;
    ctx->prof_used = 0;
    return CNN_OK;
}

size_t cnn_workspace_bytes(int op, int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (op == CNN_OP_BLOCK_SEARCH) return cnn::block_search_ws();
    ConvShape s;
    if (make_shape(N, C, H, W, K, R, S, stride, pad, &s) != CNN_OK) return 0;
    switch (op) {
        case CNN_OP_CONV_BWD_WEIGHT_UNPOOL: return cnn::smallc_unpool_serves(s) ? cnn::smallc_conv_bwd_weight_ws(s) : 0;
        case CNN_OP_CONV_FWD: return cnn::mfma_conv_fwd_ws(s);
        case CNN_OP_CONV_FWD_RELU_POOL: return cnn::c3_pool_serves(s) ? 0 : cnn::mfma_conv_fwd_pool_ws(s);
        case CNN_OP_CONV_BWD_DATA: return cnn::mfma_conv_bwd_data_ws(s);
        case CNN_OP_CONV_BWD_WEIGHT: {
            // the kernels are tried in this order; one that does not serve the shape reports 0
            const size_t a = cnn::mfma_conv_bwd_weight_ws(s);
            if (a) return a;
            const size_t b = cnn::smallc_conv_bwd_weight_ws(s);
            return b ? b : cnn::igemm_conv_bwd_weight_ws(s);
        }
        case CNN_OP_FC_FWD: return cnn::mfma_gemm_ws(N, K, C);
        case CNN_OP_FC_BWD: {
            const size_t a = cnn::mfma_gemm_ws(N, C, K), b = cnn::mfma_gemm_ws(K, C, N);
            return a > b ? a : b;
        }
        default: return 0;
    }
}

static int conv_fwd_impl(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                         const float* x, const float* w, float* y, int relu) {
    if (!ctx || !x || !w || !y || !aligned16(x) || !aligned16(w) || !aligned16(y)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (!ctx->force_direct) {
        if (s.stride > 1 && s.C >= 16) {
            st = cnn::igemm_conv_fwd(ctx, s, x, w, y, relu);
            if (st != CNN_EUNSUPPORTED) return st;
        }
        st = cnn::mfma_conv_fwd(ctx, s, x, w, y, relu);
        if (st != CNN_EUNSUPPORTED) return st;
        st = cnn::c3_strided_conv_fwd(ctx, s, x, w, y, relu);
        if (st != CNN_EUNSUPPORTED) return st;
        st = cnn::igemm_conv_fwd(ctx, s, x, w, y, relu);
        if (st != CNN_EUNSUPPORTED) return st;
    }
    return cnn::direct_conv_fwd(ctx, s, x, w, y, relu);
}
int cnn_conv_fwd(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                 const float* x, const float* w, float* y) {
    return conv_fwd_impl(ctx, N, C, H, W, K, R, S, stride, pad, x, w, y, 0);
}
int cnn_conv_fwd_relu(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float* x, const float* w, float* a) {
    return conv_fwd_impl(ctx, N, C, H, W, K, R, S, stride, pad, x, w, a, 1);
}

int cnn_conv_fwd_relu_pool(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const float* x, const float* w, float* a, uint8_t* arg) {
    if (!ctx || !x || !w || !a || !arg || !aligned16(x) || !aligned16(w) || !aligned16(a)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if ((s.P | s.Q) & 1) return CNN_EINVAL;
    if (ctx->force_direct) return CNN_EUNSUPPORTED;
    st = cnn::c3_pool_conv_fwd(ctx, s, x, w, a, arg);
    if (st != CNN_EUNSUPPORTED) return st;
    return cnn::mfma_conv_fwd_pool(ctx, s, x, w, a, arg);
}

static int conv_bwd_data_impl(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                              const float* dy, const float* w, const float* act, float* dx) {
    if (!ctx || !dy || !w || !dx || !aligned16(dy) || !aligned16(w) || !aligned16(dx)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (!ctx->force_direct) {
        st = cnn::mfma_conv_bwd_data(ctx, s, dy, w, dx, act);
        if (st != CNN_EUNSUPPORTED) return st;
        st = cnn::igemm_conv_bwd_data(ctx, s, dy, w, dx, act);
        if (st != CNN_EUNSUPPORTED) return st;
    }
    return cnn::direct_conv_bwd_data(ctx, s, dy, w, dx, act);
}
int cnn_conv_bwd_data(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float* dy, const float* w, float* dx) {
    return conv_bwd_data_impl(ctx, N, C, H, W, K, R, S, stride, pad, dy, w, nullptr, dx);
}
int cnn_conv_bwd_data_relu(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const float* dy, const float* w, const float* x_act, float* dz) {
    if (!x_act || !aligned16(x_act)) return CNN_EINVAL;
    return conv_bwd_data_impl(ctx, N, C, H, W, K, R, S, stride, pad, dy, w, x_act, dz);
}

int cnn_conv_bwd_data_unpool_relu(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                  const float* dy, const float* w, const uint8_t* arg, const float* a_pool, float* dz) {
    if (!ctx || !dy || !w || !arg || !a_pool || !dz || !aligned16(dy) || !aligned16(w) || !aligned16(a_pool) ||
        !aligned16(dz))
        return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct) return CNN_EUNSUPPORTED;
    return cnn::mfma_conv_bwd_data(ctx, s, dy, w, dz, a_pool, arg);
}

int cnn_conv_bwd_weight(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                        const float* x, const float* dy, float* dw) {
    if (!ctx || !x || !dy || !dw || !aligned16(x) || !aligned16(dy) || !aligned16(dw)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (!ctx->force_direct) {
        st = cnn::mfma_conv_bwd_weight(ctx, s, x, dy, sink_dw(dw));
        if (st != CNN_EUNSUPPORTED) return st;
        st = cnn::smallc_conv_bwd_weight(ctx, s, x, dy, sink_dw(dw));
        if (st != CNN_EUNSUPPORTED) return st;
        st = cnn::igemm_conv_bwd_weight(ctx, s, x, dy, sink_dw(dw));
        if (st != CNN_EUNSUPPORTED) return st;
    }
    return cnn::direct_conv_bwd_weight(ctx, s, x, dy, dw);
}

int cnn_conv_bwd_weight_static(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dy, float* dw) {
    if (!ctx || !x || !dy || !dw || !aligned16(x) || !aligned16(dy) || !aligned16(dw)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (cnn_workspace_bytes(CNN_OP_CONV_BWD_WEIGHT, N, C, H, W, K, R, S, stride, pad) > (size_t)CNN_STATIC_SCRATCH_BYTES) {
        snprintf(ctx->err, sizeof(ctx->err), "cnn_conv_bwd_weight_static: the layer needs more than the %d bytes of "
                 "built-in scratch; use cnn_conv_bwd_weight with a workspace", CNN_STATIC_SCRATCH_BYTES);
        return CNN_EWORKSPACE;
    }
    void* ptr = nullptr;
    st = static_scratch(ctx, &ptr);
    if (st != CNN_OK) return st;
    // Same kernels as cnn_conv_bwd_weight, with the built-in array as their workspace.  Per-kernel profiling
    // creates event objects, so it is off for this call.
    void* const ws = ctx->ws;
    const size_t ws_bytes = ctx->ws_bytes;
    const int profile = ctx->profile;
    ctx->ws = ptr;
    ctx->ws_bytes = CNN_STATIC_SCRATCH_BYTES;
    ctx->profile = 0;
    st = cnn_conv_bwd_weight(ctx, N, C, H, W, K, R, S, stride, pad, x, dy, dw);
    ctx->ws = ws;
    ctx->ws_bytes = ws_bytes;
    ctx->profile = profile;
    return st;
}

// The second stage of the weight gradient (the sum over the minibatch splits, Section 3.1) hands each finished
// element to the SGD step of Section 3.4 instead of storing it.
int cnn_conv_bwd_weight_sgd(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            const float* x, const float* dy, float* w, float* v, float lr, float momentum) {
    if (!ctx || !x || !dy || !w || !aligned16(x) || !aligned16(dy) || !aligned16(w) || (v && !aligned16(v)))
        return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct) return CNN_EUNSUPPORTED;
    const GradSink sink{nullptr, w, v, lr, momentum};
    st = cnn::mfma_conv_bwd_weight(ctx, s, x, dy, sink);
    if (st != CNN_EUNSUPPORTED) return st;
    st = cnn::smallc_conv_bwd_weight(ctx, s, x, dy, sink);
    if (st != CNN_EUNSUPPORTED) return st;
    return cnn::igemm_conv_bwd_weight(ctx, s, x, dy, sink);
}

// ---- Section 2.3's transpose-weights kept resident: made once, handed to backpropagation, refreshed by the update
int cnn_conv_transpose_weights(cnn_ctx* ctx, int K, int C, int R, int S, const float* w, float* wT) {
    if (!ctx || !w || !wT || K <= 0 || C <= 0 || R <= 0 || S <= 0 || !aligned16(w) || !aligned16(wT)) return CNN_EINVAL;
    if ((double)K * C * R * S > 2147483647.0) return CNN_EUNSUPPORTED;
    return cnn::mfma_conv_transpose_weights(ctx, K, C, R * S, w, wT);
}

int cnn_conv_bwd_data_wt(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                         const float* dy, const float* wT, const float* x_act, const uint8_t* arg, float* dz) {
    if (!ctx || !dy || !wT || !dz || !aligned16(dy) || !aligned16(wT) || !aligned16(dz) || (x_act && !aligned16(x_act)) ||
        (arg && !x_act))
        return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct) return CNN_EUNSUPPORTED;
    return cnn::mfma_conv_bwd_data_wt(ctx, s, dy, wT, dz, x_act, arg);
}

int cnn_conv_bwd_weight_sgd_wt(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dy, float* w, float* v, float* wT, float lr, float momentum) {
    if (!ctx || !x || !dy || !w || !wT || !aligned16(x) || !aligned16(dy) || !aligned16(w) || !aligned16(wT) ||
        (v && !aligned16(v)))
        return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct) return CNN_EUNSUPPORTED;
    if (cnn::mfma_conv_bwd_weight_keeps_wt(s))      // the reduction writes every updated weight to both copies
        return cnn::mfma_conv_bwd_weight(ctx, s, x, dy, sink_sgd(w, v, lr, momentum, wT, s.K, s.C));
    st = cnn_conv_bwd_weight_sgd(ctx, N, C, H, W, K, R, S, stride, pad, x, dy, w, v, lr, momentum);
    if (st != CNN_OK) return st;
    return cnn::mfma_conv_transpose_weights(ctx, s.K, s.C, s.R * s.S, w, wT);
}

int cnn_conv_tile_info(int op, int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int32_t* tile,
                       double* bf) {
    if (!tile || !bf) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (op != CNN_OP_CONV_FWD && op != CNN_OP_CONV_FWD_RELU_POOL && op != CNN_OP_CONV_BWD_DATA) return CNN_EINVAL;
    if (!cnn::mfma_conv_tile_info(s, op, tile)) return CNN_EUNSUPPORTED;
    // backpropagation is the same kernel with the roles of the feature maps swapped and stride 1
    const int ifm = op == CNN_OP_CONV_BWD_DATA ? K : C;
    const int out_rows = op == CNN_OP_CONV_BWD_DATA ? H : s.P;
    // a tile of whole images counts as that many images (each with its own halo rows); one that ends inside an
    // image is counted like a single taller image
    const int images = tile[1] % out_rows == 0 ? tile[1] / out_rows : 1;
    *bf = cnn_bf_block_traversal(ifm, R, S, op == CNN_OP_CONV_BWD_DATA ? 1 : stride, images, tile[0], tile[1] / images,
                                 tile[2]);
    return CNN_OK;
}

static int bwd_weight_unpool_impl(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                  const float* x, const float* dpool, const uint8_t* arg, const GradSink& sink) {
    if (!ctx || !x || !dpool || !arg || !aligned16(x) || !aligned16(dpool)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, C, H, W, K, R, S, stride, pad, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct) return CNN_EUNSUPPORTED;
    return cnn::smallc_conv_bwd_weight_unpool(ctx, s, x, dpool, arg, sink);
}
int cnn_conv_bwd_weight_unpool(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dpool, const uint8_t* arg, float* dw) {
    if (!dw || !aligned16(dw)) return CNN_EINVAL;
    return bwd_weight_unpool_impl(ctx, N, C, H, W, K, R, S, stride, pad, x, dpool, arg, sink_dw(dw));
}
int cnn_conv_bwd_weight_unpool_sgd(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                   const float* x, const float* dpool, const uint8_t* arg, float* w, float* v, float lr,
                                   float momentum) {
    if (!w || !aligned16(w) || (v && !aligned16(v))) return CNN_EINVAL;
    return bwd_weight_unpool_impl(ctx, N, C, H, W, K, R, S, stride, pad, x, dpool, arg, GradSink{nullptr, w, v, lr, momentum});
}

// Fully-connected layers: the conv loop nest with k_h = k_w = out_h = out_w = 1 (Section 2.1), i.e. GEMMs.
int cnn_fc_fwd(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, float* y) {
    if (!ctx || !x || !w || !y || !aligned16(x) || !aligned16(w) || !aligned16(y)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, I, 1, 1, O, 1, 1, 1, 0, &s);
    if (st != CNN_OK) return st;
    if (!ctx->force_direct) {
        st = cnn::mfma_gemm(ctx, N, O, I, x, 0, w, 0, y);   // y[n][o] = sum_i x[n][i] w[o][i]
        if (st != CNN_EUNSUPPORTED) return st;
    }
    return cnn::direct_conv_fwd(ctx, s, x, w, y, 0);
}

int cnn_fc_bwd(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, const float* dy, float* dx,
               float* dw) {
    if (!ctx || !dy || !aligned16(dy)) return CNN_EINVAL;
    if (dx && (!w || !aligned16(w) || !aligned16(dx))) return CNN_EINVAL;
    if (dw && (!x || !aligned16(x) || !aligned16(dw))) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, I, 1, 1, O, 1, 1, 1, 0, &s);
    if (st != CNN_OK) return st;
    if (dw) {   // weight gradient first, as the paper orders it (Section 3.1)
        st = CNN_EUNSUPPORTED;
        if (!ctx->force_direct) st = cnn::mfma_gemm(ctx, O, I, N, dy, 1, x, 1, dw);   // dw[o][i] = sum_n dy[n][o] x[n][i]
        if (st == CNN_EUNSUPPORTED) st = cnn::direct_conv_bwd_weight(ctx, s, x, dy, dw);
        if (st != CNN_OK) return st;
    }
    if (dx) {
        st = CNN_EUNSUPPORTED;
        if (!ctx->force_direct) st = cnn::mfma_gemm(ctx, N, I, O, dy, 0, w, 1, dx);   // dx[n][i] = sum_o dy[n][o] w[o][i]
        if (st == CNN_EUNSUPPORTED) st = cnn::direct_conv_bwd_data(ctx, s, dy, w, dx, nullptr);
        if (st != CNN_OK) return st;
    }
    return CNN_OK;
}

int cnn_fc_bwd_sgd(cnn_ctx* ctx, int N, int I, int O, const float* x, float* w, const float* dy, float* dx, float* v,
                   float lr, float momentum) {
    return cnn_fc_bwd_sgd_act(ctx, N, I, O, x, w, dy, dx, v, lr, momentum, CNN_ACT_NONE);
}

// ---- fully-connected layers with the neighbouring activation folded into the GEMM's store
static bool act_ok(int act) { return act == CNN_ACT_NONE || act == CNN_ACT_RELU || act == CNN_ACT_SIGMOID; }

int cnn_fc_fwd_act(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, float* a, int act) {
    if (!act_ok(act)) return CNN_EINVAL;
    if (act == CNN_ACT_NONE) return cnn_fc_fwd(ctx, N, I, O, x, w, a);
    if (!ctx || !x || !w || !a || !aligned16(x) || !aligned16(w) || !aligned16(a)) return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, I, 1, 1, O, 1, 1, 1, 0, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct || !cnn::mfma_gemm_serves(N, O, I, 0, 0)) return CNN_EUNSUPPORTED;
    const GradSink sink = sink_act(a, act == CNN_ACT_RELU ? ACT_RELU : ACT_SIGMOID, nullptr);
    return cnn::mfma_gemm(ctx, N, O, I, x, 0, w, 0, nullptr, &sink);
}

int cnn_fc_bwd_act(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, const float* dy, float* dz,
                   float* dw, int act_in) {
    if (!act_ok(act_in)) return CNN_EINVAL;
    if (act_in == CNN_ACT_NONE || !dz) return cnn_fc_bwd(ctx, N, I, O, x, w, dy, dz, dw);
    if (!ctx || !dy || !x || !w || !aligned16(dy) || !aligned16(x) || !aligned16(w) || !aligned16(dz) ||
        (dw && !aligned16(dw)))
        return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, I, 1, 1, O, 1, 1, 1, 0, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct || !cnn::mfma_gemm_serves(N, I, O, 0, 1)) return CNN_EUNSUPPORTED;
    if (dw) {
        st = cnn_fc_bwd(ctx, N, I, O, x, w, dy, nullptr, dw);
        if (st != CNN_OK) return st;
    }
    const GradSink sink = sink_act(dz, act_in == CNN_ACT_RELU ? ACT_RELU_BWD : ACT_SIGMOID_BWD, x);
    return cnn::mfma_gemm(ctx, N, I, O, dy, 0, w, 1, nullptr, &sink);
}

int cnn_fc_bwd_sgd_act(cnn_ctx* ctx, int N, int I, int O, const float* x, float* w, const float* dy, float* dz, float* v,
                       float lr, float momentum, int act_in) {
    if (!act_ok(act_in)) return CNN_EINVAL;
    if (!ctx || !dy || !x || !w || !aligned16(dy) || !aligned16(x) || !aligned16(w) || (v && !aligned16(v)) ||
        (dz && !aligned16(dz)))
        return CNN_EINVAL;
    ConvShape s;
    int st = make_shape(N, I, 1, 1, O, 1, 1, 1, 0, &s);
    if (st != CNN_OK) return st;
    if (ctx->force_direct || !cnn::mfma_gemm_serves(O, I, N, 1, 1)) return CNN_EUNSUPPORTED;
    const bool fold = dz && act_in != CNN_ACT_NONE;
    if (fold && !cnn::mfma_gemm_serves(N, I, O, 0, 1)) return CNN_EUNSUPPORTED;
    if (dz) {   // backpropagation reads the weights of this iteration: before they are updated
        if (fold) {
            const GradSink dsink = sink_act(dz, act_in == CNN_ACT_RELU ? ACT_RELU_BWD : ACT_SIGMOID_BWD, x);
            st = cnn::mfma_gemm(ctx, N, I, O, dy, 0, w, 1, nullptr, &dsink);
        } else {
            st = cnn::mfma_gemm(ctx, N, I, O, dy, 0, w, 1, dz);
            if (st == CNN_EUNSUPPORTED) st = cnn::direct_conv_bwd_data(ctx, s, dy, w, dz, nullptr);
        }
        if (st != CNN_OK) return st;
    }
    const GradSink sink{nullptr, w, v, lr, momentum};
    return cnn::mfma_gemm(ctx, O, I, N, dy, 1, x, 1, nullptr, &sink);
}

}  // extern "C"
