// Internal declarations shared by the translation units of libcnn (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/cnn.h"

#include <atomic>
#include <stdarg.h>
#include <stdio.h>
#include <string>
#include <vector>

// ---- device-side vocabulary shared by the matrix-core kernels
typedef float f32x16 __attribute__((ext_vector_type(16)));     // accumulator of one v_mfma_f32_32x32x2_f32
typedef __attribute__((address_space(3))) float lds_float;      // LDS pointers are 32-bit: one VGPR each
constexpr int kOutOfRange = (int)0x80000000;   // buffer-load byte offset beyond any descriptor used here -> reads 0
constexpr int kRsrcWord3 = 0x00020000;         // raw buffer descriptor of 32-bit elements

// printf into a std::string.  Each kernel instantiation builds its profile name once in a function-local static
// (initialised thread-safely by the language), so two contexts on two threads never write one buffer.
inline std::string strf(const char* fmt, ...) {
    char buf[160];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    return std::string(buf);
}

struct ProfEntry {
    const char* name;
    double flops;
    hipEvent_t e0, e1;
};

struct cnn_ctx {
    hipStream_t stream;
    void* ws;
    size_t ws_bytes;
    int force_direct;
    int profile;
    std::vector<ProfEntry> prof;      // entries [0, prof_used) are live; the rest is a pool of created events
    size_t prof_used;
    char err[256];
};

struct ConvShape {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
};

// Where the last stage of a weight gradient puts each element g (flat index i of the [K][C][R][S] / [O][I] tensor):
// into dw[i], or, when w is set, straight into the SGD step of Section 3.4 without dw ever reaching memory:
//   v[i] <- mu * v[i] + g (when v is set);  w[i] <- w[i] - lr * v[i]   (v == nullptr: w[i] <- w[i] - lr * g)
// The arithmetic is the one k_sgd applies to a stored gradient, so both routes give the same bits.
// An activation folded into the store of a plain output (act == ACT_NONE otherwise).  The expressions are the ones
// the element-wise kernels use, so the folded and the separate route give the same bits.
//   ACT_RELU / ACT_SIGMOID: the forward activation of the stored value;
//   ACT_RELU_BWD / ACT_SIGMOID_BWD: the stored value is a gradient behind an activation whose OUTPUT is aux (same
//   index): it is multiplied by the activation's derivative (ReLU: 1 where aux > 0; sigmoid: aux * (1 - aux)).
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_SIGMOID = 2, ACT_RELU_BWD = 3, ACT_SIGMOID_BWD = 4 };
__device__ __forceinline__ float act_apply(int act, float c, float aux) {
    switch (act) {
        case ACT_RELU: return c > 0.f ? c : 0.f;
        case ACT_SIGMOID: return 1.0f / (1.0f + expf(-c));
        case ACT_RELU_BWD: return aux > 0.f ? c : 0.f;
        case ACT_SIGMOID_BWD: return c * aux * (1.0f - aux);
        default: return c;
    }
}

struct GradSink {
    float* dw;
    float* w;
    float* v;
    float lr, mu;
    int act;             // only with w == nullptr
    const float* aux;
    // only with w != nullptr, convolution weights [K][C][RS]: the mirrored transpose-weights kept beside them
    // (wT[c][k][RS-1-t] = w[k][c][t], what backpropagation reads) receive every updated weight as well
    float* wT;
    int wt_K, wt_C;
};
inline GradSink sink_dw(float* dw) { return GradSink{dw, nullptr, nullptr, 0.f, 0.f, ACT_NONE, nullptr, nullptr, 0, 0}; }
inline GradSink sink_act(float* out, int act, const float* aux) { return GradSink{out, nullptr, nullptr, 0.f, 0.f, act, aux, nullptr, 0, 0}; }
inline GradSink sink_sgd(float* w, float* v, float lr, float mu, float* wT = nullptr, int K = 0, int C = 0) {
    return GradSink{nullptr, w, v, lr, mu, ACT_NONE, nullptr, wT, K, C};
}

__device__ __forceinline__ void sink_store(const GradSink& k, size_t i, float g) {
    if (k.w) {
        float vel = g;
        if (k.v) {
            vel = fmaf(k.mu, k.v[i], g);
            k.v[i] = vel;
        }
        k.w[i] = fmaf(-k.lr, vel, k.w[i]);
    } else if (k.act != ACT_NONE) {
        k.dw[i] = act_apply(k.act, g, k.act >= ACT_RELU_BWD ? k.aux[i] : 0.f);
    } else {
        k.dw[i] = g;
    }
}

namespace cnn {

inline int out_dim(int in, int k, int stride, int pad) {
    const int span = in + 2 * pad - k;
    return span < 0 ? 0 : span / stride + 1;
}

// Brackets the kernel launches made during its lifetime with a pair of events when profiling is on.
struct ProfScope {
    cnn_ctx* ctx;
    ProfEntry* ent;
    ProfScope(cnn_ctx* c, const char* name, double flops);
    ~ProfScope();
};

inline double conv_flops(const ConvShape& s) {   // Section 3.1: 2 * MB * ifm * ofm * k_w * k_h * out_w * out_h per pass
    return 2.0 * s.N * s.C * s.K * s.R * s.S * s.P * s.Q;
}

int hip_check(cnn_ctx* ctx, hipError_t e, const char* what);   // records text, returns CNN_OK / CNN_EHIP
// A kernel's limit on dynamic LDS is an attribute of the (kernel, device) pair: sets it to `bytes` the first time the
// kernel is launched on the current device (`done`: one bit per device, one object per kernel).
int lds_attr_once(cnn_ctx* ctx, std::atomic<unsigned long long>& done, const void* fn, int bytes, const char* what);
constexpr int kMaxLdsBytes = 160 * 1024;      // LDS of a gfx950 compute unit
int launch_check(cnn_ctx* ctx, const char* what);              // hipGetLastError after a launch

// ---- plain one-thread-per-output kernels: any shape, slow; the fallback of every contraction
int direct_conv_fwd(cnn_ctx*, const ConvShape&, const float* x, const float* w, float* y, int relu);
int direct_conv_bwd_data(cnn_ctx*, const ConvShape&, const float* dy, const float* w, float* dx, const float* act);
int direct_conv_bwd_weight(cnn_ctx*, const ConvShape&, const float* x, const float* dy, float* dw);

// ---- MFMA paths; each returns CNN_EUNSUPPORTED (without launching) for shapes it does not cover
int mfma_conv_fwd(cnn_ctx*, const ConvShape&, const float* x, const float* w, float* y, int relu);
int mfma_conv_bwd_data(cnn_ctx*, const ConvShape&, const float* dy, const float* w, float* dx, const float* act,
                       const unsigned char* arg = nullptr);
// the same with the mirrored transpose-weights handed in (wT[c][k][R-1-r][S-1-s] = w[k][c][r][s]) instead of made per call
int mfma_conv_bwd_data_wt(cnn_ctx*, const ConvShape&, const float* dy, const float* wT, float* dx, const float* act,
                          const unsigned char* arg);
int mfma_conv_transpose_weights(cnn_ctx*, int K, int C, int RS, const float* w, float* wT);
// does the weight-gradient kernel that serves the shape refresh sink.wT itself?
bool mfma_conv_bwd_weight_keeps_wt(const ConvShape&);
int mfma_conv_bwd_weight(cnn_ctx*, const ConvShape&, const float* x, const float* dy, const GradSink& sink);
size_t mfma_conv_bwd_weight_ws(const ConvShape&);
size_t mfma_conv_bwd_data_ws(const ConvShape&);
size_t mfma_conv_fwd_ws(const ConvShape&);
size_t mfma_conv_fwd_pool_ws(const ConvShape&);
int mfma_conv_fwd_pool(cnn_ctx*, const ConvShape&, const float* x, const float* w, float* a, unsigned char* arg);
bool mfma_conv_tile_info(const ConvShape&, int op, int32_t tile[8]);
size_t block_search_ws();
// 3x3 first layer (3 input feature maps, 224 columns, 64 features) with ReLU + 2x2 max-pool in the epilogue
int c3_pool_conv_fwd(cnn_ctx*, const ConvShape&, const float* x, const float* w, float* a, unsigned char* arg);
bool c3_pool_serves(const ConvShape&);
// strided first layer (3 input feature maps, 11x11 / 4)
int c3_strided_conv_fwd(cnn_ctx*, const ConvShape&, const float* x, const float* w, float* y, int relu);
// few input feature maps (first layers), any kernel size / stride
int smallc_conv_bwd_weight(cnn_ctx*, const ConvShape&, const float* x, const float* dy, const GradSink& sink);
size_t smallc_conv_bwd_weight_ws(const ConvShape&);
// ... with the gradient given behind a 2x2 max-pool (pooled size + window positions)
int smallc_conv_bwd_weight_unpool(cnn_ctx*, const ConvShape&, const float* x, const float* dpool, const unsigned char* arg,
                                  const GradSink& sink);
bool smallc_unpool_serves(const ConvShape&);

// implicit GEMM with a gathered operand: any kernel size, stride and padding (everything the kernels above leave)
int igemm_conv_fwd(cnn_ctx*, const ConvShape&, const float* x, const float* w, float* y, int relu);
int igemm_conv_bwd_data(cnn_ctx*, const ConvShape&, const float* dy, const float* w, float* dx, const float* act);
int igemm_conv_bwd_weight(cnn_ctx*, const ConvShape&, const float* x, const float* dy, const GradSink& sink);
size_t igemm_conv_bwd_weight_ws(const ConvShape&);

// C[M][Nn] = op(A) * op(B); row-major operands.
//   a_kmajor == 0: A is [M][Kd] (contraction index contiguous);  != 0: A is [Kd][M]
//   b_kmajor == 0: B is [Nn][Kd] (contraction index contiguous); != 0: B is [Kd][Nn]
// sink (optional): C is a weight gradient that goes into the SGD step instead of memory (C itself may then be null)
int mfma_gemm(cnn_ctx*, int M, int Nn, int Kd, const float* A, int a_kmajor, const float* B, int b_kmajor, float* C,
              const GradSink* sink = nullptr);
bool mfma_gemm_serves(int M, int Nn, int Kd, int a_kmajor, int b_kmajor);
size_t mfma_gemm_ws(int M, int Nn, int Kd);

}  // namespace cnn
