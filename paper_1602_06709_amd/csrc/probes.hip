// Measurement aids: what this GPU sustains on the two resources the training kernels are bound by, measured with
// kernels of the library itself so that a benchmark can quote its kernels against a ceiling anyone can reproduce.
//   cnn_probe_mfma:    back-to-back v_mfma_f32_32x32x2_f32 on registers only (no memory, no LDS)
//   cnn_probe_stream:  read-only / write-only / copy streams over large arrays
#include "common.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaGroups = 512;        // two workgroups of four waves per compute unit: every SIMD holds two waves
constexpr int kMfmaChains = 8;          // independent accumulators per wave: the 16-pass MFMA never waits on itself

__global__ void __launch_bounds__(256) k_probe_mfma(int iters, float seed, float* __restrict__ sink) {
    f32x16 acc[kMfmaChains];
#pragma unroll
    for (int j = 0; j < kMfmaChains; ++j)
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    // dense operands of ordinary magnitude (the rate depends a little on the operand values: zeros run faster)
    const float a = seed + 1e-3f * (float)(threadIdx.x % 61), b = 1.0f - 7e-4f * (float)(threadIdx.x % 53);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < kMfmaChains; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kMfmaChains; ++j)
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// The stream kernels take the launch shape of the SGD update: few resident workgroups per compute unit (the launch
// reserves LDS it never uses), workgroups in address order, non-temporal accesses, so that the chip works on a few
// MB of the arrays at any moment.  Floats in flight per thread (U) and workgroups per compute unit are the best
// measured per direction: read 2 x 2, write 1 x 1, copy 2 x 2.
constexpr int kStreamBlock = 512;
constexpr int kNonTemporal = 2;
template <int MODE> struct StreamCfg;
template <> struct StreamCfg<CNN_STREAM_READ> { static constexpr int U = 2, LDS = 64 * 1024; };
template <> struct StreamCfg<CNN_STREAM_WRITE> { static constexpr int U = 1, LDS = 96 * 1024; };
template <> struct StreamCfg<CNN_STREAM_COPY> { static constexpr int U = 2, LDS = 64 * 1024; };

template <int MODE>
__global__ void __launch_bounds__(kStreamBlock) k_probe_stream(size_t n4, const float* __restrict__ src, float* __restrict__ dst) {
    constexpr int U = StreamCfg<MODE>::U;
    const size_t base = (size_t)blockIdx.x * kStreamBlock * U;
    const size_t left = (n4 - base) * sizeof(v4f);
    const int bytes = left > (size_t)kStreamBlock * U * sizeof(v4f) ? kStreamBlock * U * (int)sizeof(v4f) : (int)left;
    v4f t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) t[u] = v4f{1.f, 2.f, 3.f, 4.f};
    if (MODE != CNN_STREAM_WRITE) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(src) + 4 * base, 0, bytes, kRsrcWord3);
#pragma unroll
        for (int u = 0; u < U; ++u)
            t[u] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(
                                               rs, (u * kStreamBlock + (int)threadIdx.x) * (int)sizeof(v4f), 0, kNonTemporal));
    }
    if (MODE == CNN_STREAM_READ) {
        // keeps the loads alive without a store: the condition holds for no input
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float s = t[u].x + t[u].y + t[u].z + t[u].w;
            if (s != s && t[u].x == 12345.678f) dst[0] = s;
        }
    } else {
        const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(dst + 4 * base, 0, bytes, kRsrcWord3);
#pragma unroll
        for (int u = 0; u < U; ++u)
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, t[u]), rd,
                                                   (u * kStreamBlock + (int)threadIdx.x) * (int)sizeof(v4f), 0, kNonTemporal);
    }
}

template <int MODE>
int launch_stream(cnn_ctx* ctx, const char* name, size_t n4, const float* src, float* dst) {
    const size_t groups = (n4 + (size_t)kStreamBlock * StreamCfg<MODE>::U - 1) / ((size_t)kStreamBlock * StreamCfg<MODE>::U);
    if (groups > 0x7fffffffu) return CNN_EUNSUPPORTED;
    static std::atomic<unsigned long long> attr_done{0};     // one bit per device: the attribute is the device's
    {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_probe_stream<MODE>), StreamCfg<MODE>::LDS, "hipFuncSetAttribute(probe_stream)");
        if (st_attr != CNN_OK) return st_attr;
    }
    {
        cnn::ProfScope ps(ctx, name, 0.0);
        hipLaunchKernelGGL(k_probe_stream<MODE>, dim3((unsigned)groups), dim3(kStreamBlock), StreamCfg<MODE>::LDS, ctx->stream,
                           n4, src, dst);
    }
    return cnn::launch_check(ctx, "probe_stream");
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int cnn_probe_mfma(cnn_ctx* ctx, int iters, float* sink, double* flops) {
    if (!ctx || !sink || iters <= 0 || iters > (1 << 24)) return CNN_EINVAL;
    const double fl = (double)kMfmaGroups * 4 * (double)iters * kMfmaChains * 4096.0;   // 32*32*2*2 FLOP per wave MFMA
    if (flops) *flops = fl;
    cnn::ProfScope ps(ctx, "k_probe_mfma", fl);
    hipLaunchKernelGGL(k_probe_mfma, dim3(kMfmaGroups), dim3(256), 0, ctx->stream, iters, 0.5f, sink);
    return cnn::launch_check(ctx, "probe_mfma");
}

int cnn_probe_stream(cnn_ctx* ctx, int mode, size_t n, const float* src, float* dst) {
    if (!ctx || n < 4 || (n & 3) || mode < CNN_STREAM_READ || mode > CNN_STREAM_COPY) return CNN_EINVAL;
    if (mode != CNN_STREAM_WRITE && (!src || !aligned16(src))) return CNN_EINVAL;
    if (!dst || !aligned16(dst)) return CNN_EINVAL;
    const size_t n4 = n >> 2;
    if (mode == CNN_STREAM_READ) return launch_stream<CNN_STREAM_READ>(ctx, "k_probe_stream<read>", n4, src, dst);
    if (mode == CNN_STREAM_WRITE) return launch_stream<CNN_STREAM_WRITE>(ctx, "k_probe_stream<write>", n4, src, dst);
    return launch_stream<CNN_STREAM_COPY>(ctx, "k_probe_stream<copy>", n4, src, dst);
}

}  // extern "C"
