// Plain kernels: one thread per output element, the definition written out.  They cover every
// shape the ABI admits and are the fallback when no tiled kernel applies (Section 2.1 statements).
#include "common.h"

namespace {

__global__ void k_direct_conv_fwd(ConvShape s, int relu, const float* __restrict__ x, const float* __restrict__ w,
                                  float* __restrict__ y) {
    const size_t total = (size_t)s.N * s.K * s.P * s.Q;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        size_t f = i;
        const int q = f % s.Q; f /= s.Q;
        const int p = f % s.P; f /= s.P;
        const int k = f % s.K; f /= s.K;
        const int n = (int)f;
        float acc = 0.f;
        for (int c = 0; c < s.C; ++c)
            for (int r = 0; r < s.R; ++r) {
                const int h = p * s.stride + r - s.pad;
                if (h < 0 || h >= s.H) continue;
                for (int t = 0; t < s.S; ++t) {
                    const int ww = q * s.stride + t - s.pad;
                    if (ww < 0 || ww >= s.W) continue;
                    acc = fmaf(x[(((size_t)n * s.C + c) * s.H + h) * s.W + ww],
                               w[(((size_t)k * s.C + c) * s.R + r) * s.S + t], acc);
                }
            }
        y[i] = (relu && acc < 0.f) ? 0.f : acc;
    }
}

__global__ void k_direct_conv_bwd_data(ConvShape s, const float* __restrict__ dy, const float* __restrict__ w,
                                       const float* __restrict__ act, float* __restrict__ dx) {
    const size_t total = (size_t)s.N * s.C * s.H * s.W;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        size_t f = i;
        const int ww = f % s.W; f /= s.W;
        const int h = f % s.H; f /= s.H;
        const int c = f % s.C; f /= s.C;
        const int n = (int)f;
        float acc = 0.f;
        for (int k = 0; k < s.K; ++k)
            for (int r = 0; r < s.R; ++r) {
                const int hn = h + s.pad - r;
                if (hn < 0 || hn % s.stride) continue;
                const int p = hn / s.stride;
                if (p >= s.P) continue;
                for (int t = 0; t < s.S; ++t) {
                    const int wn = ww + s.pad - t;
                    if (wn < 0 || wn % s.stride) continue;
                    const int q = wn / s.stride;
                    if (q >= s.Q) continue;
                    acc = fmaf(dy[(((size_t)n * s.K + k) * s.P + p) * s.Q + q],
                               w[(((size_t)k * s.C + c) * s.R + r) * s.S + t], acc);
                }
            }
        dx[i] = (act && !(act[i] > 0.f)) ? 0.f : acc;
    }
}

// One workgroup per weight-gradient element; threads stride over (n,p,q); tree reduction in LDS.
__global__ void __launch_bounds__(256) k_direct_conv_bwd_weight(ConvShape s, const float* __restrict__ x,
                                                                const float* __restrict__ dy,
                                                                float* __restrict__ dw) {
    __shared__ float red[256];
    size_t f = blockIdx.x;
    const int t = f % s.S; f /= s.S;
    const int r = f % s.R; f /= s.R;
    const int c = f % s.C; f /= s.C;
    const int k = (int)f;
    const size_t npq = (size_t)s.N * s.P * s.Q;
    float acc = 0.f;
    for (size_t j = threadIdx.x; j < npq; j += blockDim.x) {
        size_t g = j;
        const int q = g % s.Q; g /= s.Q;
        const int p = g % s.P; g /= s.P;
        const int n = (int)g;
        const int h = p * s.stride + r - s.pad, ww = q * s.stride + t - s.pad;
        if (h < 0 || h >= s.H || ww < 0 || ww >= s.W) continue;
        acc = fmaf(x[(((size_t)n * s.C + c) * s.H + h) * s.W + ww], dy[(((size_t)n * s.K + k) * s.P + p) * s.Q + q], acc);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) dw[blockIdx.x] = red[0];
}

inline unsigned grid_for(size_t total, int block) {
    size_t g = (total + block - 1) / block;
    const size_t cap = 256u * 32u;
    return (unsigned)(g < cap ? (g ? g : 1) : cap);
}

}  // namespace

namespace cnn {

int direct_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* y, int relu) {
    const size_t total = (size_t)s.N * s.K * s.P * s.Q;
    ProfScope ps(ctx, "k_direct_conv_fwd", conv_flops(s));
    hipLaunchKernelGGL(k_direct_conv_fwd, dim3(grid_for(total, 256)), dim3(256), 0, ctx->stream, s, relu, x, w, y);
    return launch_check(ctx, "direct_conv_fwd");
}
int direct_conv_bwd_data(cnn_ctx* ctx, const ConvShape& s, const float* dy, const float* w, float* dx, const float* act) {
    const size_t total = (size_t)s.N * s.C * s.H * s.W;
    ProfScope ps(ctx, "k_direct_conv_bwd_data", conv_flops(s));
    hipLaunchKernelGGL(k_direct_conv_bwd_data, dim3(grid_for(total, 256)), dim3(256), 0, ctx->stream, s, dy, w, act, dx);
    return launch_check(ctx, "direct_conv_bwd_data");
}
int direct_conv_bwd_weight(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, float* dw) {
    const size_t total = (size_t)s.K * s.C * s.R * s.S;
    ProfScope ps(ctx, "k_direct_conv_bwd_weight", conv_flops(s));
    hipLaunchKernelGGL(k_direct_conv_bwd_weight, dim3((unsigned)total), dim3(256), 0, ctx->stream, s, x, dy, dw);
    return launch_check(ctx, "direct_conv_bwd_weight");
}

}  // namespace cnn
