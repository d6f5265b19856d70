// Bandwidth-bound kernels: the SGD update, the Section 2.3 layout permutations and the glue ops
// between layers (ReLU, 2x2 max-pool, sigmoid, softmax cross-entropy).
#include "common.h"

namespace {

constexpr int kBlock = 256;

inline unsigned stream_grid(size_t work_items, int per_block) {
    size_t g = (work_items + per_block - 1) / per_block;
    const size_t cap = 256u * 16u;   // 16 workgroups per compute unit keeps every HBM channel busy
    return (unsigned)(g < cap ? (g ? g : 1) : cap);
}

// ---------------------------------------------------------------- SGD
// v <- mu*v + g ; w <- w - lr*v: three read streams and two write streams over arrays far larger than any cache.
// What bounds it is how many DRAM rows the launch keeps open, so the kernel keeps the span of addresses in flight
// small: one workgroup of 512 threads per compute unit (the launch reserves more than half of the LDS it never
// uses), one float4 per thread and array, workgroups dispatched in address order.  At any moment the chip then works
// on about 2 MB of each array (256 x 8 KB) instead of the tens of MB a full-occupancy grid spreads over, and the
// in-place stores land in rows the loads have just opened.  All accesses carry the non-temporal hint (nothing is
// reused before it leaves the caches).  Measured on VGG-A's 132.9 M parameters: 6.7-6.9 TB/s against 5.4 TB/s for
// a full-occupancy grid-stride kernel with temporal loads.  Without momentum there is one stream less per
// direction and two resident workgroups do best (6.7 TB/s).
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kSgdBlock = 512;
constexpr int kSgdLds = 96 * 1024;       // more than half of a compute unit's 160 KB: one resident workgroup
constexpr int kSgdLdsPlain = 64 * 1024;  // without momentum (two read streams, one write stream): two workgroups
constexpr int kNonTemporal = 2;       // cache-policy bit "nt" of buffer loads / stores

template <bool MOMENTUM>
__global__ void __launch_bounds__(kSgdBlock) k_sgd(size_t n4, size_t n, float* __restrict__ w, const float* __restrict__ g,
                                                  float* __restrict__ v, float lr, float mu) {
    const size_t base = (size_t)blockIdx.x * kSgdBlock;                 // in float4
    const size_t left = (n4 - base) * sizeof(v4f);
    const int bytes = left > (size_t)kSgdBlock * sizeof(v4f) ? kSgdBlock * (int)sizeof(v4f) : (int)left;
    const int off = threadIdx.x * (int)sizeof(v4f);                     // past `bytes`: loads give 0, stores are dropped
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(w + 4 * base, 0, bytes, kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(g) + 4 * base, 0, bytes, kRsrcWord3);
    const v4f wv = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rw, off, 0, kNonTemporal));
    const v4f gv = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, kNonTemporal));
    v4f vel = gv;
    if (MOMENTUM) {
        const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(v + 4 * base, 0, bytes, kRsrcWord3);
        const v4f vv = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, kNonTemporal));
        vel.x = fmaf(mu, vv.x, gv.x); vel.y = fmaf(mu, vv.y, gv.y);
        vel.z = fmaf(mu, vv.z, gv.z); vel.w = fmaf(mu, vv.w, gv.w);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vel), rv, off, 0, kNonTemporal);
    }
    v4f o;
    o.x = fmaf(-lr, vel.x, wv.x); o.y = fmaf(-lr, vel.y, wv.y);
    o.z = fmaf(-lr, vel.z, wv.z); o.w = fmaf(-lr, vel.w, wv.w);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), rw, off, 0, kNonTemporal);
    // scalar tail (n not a multiple of 4)
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t j = (n4 << 2) + threadIdx.x;
        float t = g[j];
        if (MOMENTUM) {
            t = fmaf(mu, v[j], t);
            v[j] = t;
        }
        w[j] = fmaf(-lr, t, w[j]);
    }
}

// ---------------------------------------------------------------- element-wise glue
__global__ void __launch_bounds__(kBlock) k_relu_fwd(size_t n4, size_t n, const float4* __restrict__ z,
                                                    float4* __restrict__ a) {
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n4; i += stride) {
        float4 t = z[i];
        t.x = t.x > 0.f ? t.x : 0.f; t.y = t.y > 0.f ? t.y : 0.f;
        t.z = t.z > 0.f ? t.z : 0.f; t.w = t.w > 0.f ? t.w : 0.f;
        a[i] = t;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t j = (n4 << 2) + threadIdx.x;
        const float t = reinterpret_cast<const float*>(z)[j];
        reinterpret_cast<float*>(a)[j] = t > 0.f ? t : 0.f;
    }
}
__global__ void __launch_bounds__(kBlock) k_relu_bwd(size_t n4, size_t n, const float4* __restrict__ z,
                                                    const float4* __restrict__ da, float4* __restrict__ dz) {
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n4; i += stride) {
        const float4 t = z[i];
        float4 d = da[i];
        d.x = t.x > 0.f ? d.x : 0.f; d.y = t.y > 0.f ? d.y : 0.f;
        d.z = t.z > 0.f ? d.z : 0.f; d.w = t.w > 0.f ? d.w : 0.f;
        dz[i] = d;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t j = (n4 << 2) + threadIdx.x;
        reinterpret_cast<float*>(dz)[j] =
            reinterpret_cast<const float*>(z)[j] > 0.f ? reinterpret_cast<const float*>(da)[j] : 0.f;
    }
}
__global__ void __launch_bounds__(kBlock) k_sigmoid_fwd(size_t n, const float* __restrict__ z, float* __restrict__ a) {
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += stride)
        a[i] = 1.0f / (1.0f + expf(-z[i]));
}
__global__ void __launch_bounds__(kBlock) k_sigmoid_bwd(size_t n, const float* __restrict__ a,
                                                       const float* __restrict__ da, float* __restrict__ dz) {
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < n; i += stride) {
        const float s = a[i];
        dz[i] = da[i] * s * (1.0f - s);
    }
}

// 2x2 stride-2 max-pool; one thread per pair of adjacent outputs (reads two float4-aligned float2 pairs
// when W is a multiple of 4, else scalar path).  First maximum in row-major window order wins.
__device__ inline void pool_window(float a, float b, float c, float d, float& best, uint8_t& arg) {
    best = a; arg = 0;
    if (b > best) { best = b; arg = 1; }
    if (c > best) { best = c; arg = 2; }
    if (d > best) { best = d; arg = 3; }
}
__global__ void __launch_bounds__(kBlock) k_maxpool2_fwd(size_t total, int H, int W, const float* __restrict__ x,
                                                        float* __restrict__ y, uint8_t* __restrict__ arg) {
    const int P = H / 2, Q = W / 2;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int q = f % Q; f /= Q;
        const int p = f % P; f /= P;
        const float2 top = *reinterpret_cast<const float2*>(x + (f * H + 2 * p) * W + 2 * q);
        const float2 bot = *reinterpret_cast<const float2*>(x + (f * H + 2 * p + 1) * W + 2 * q);
        float best; uint8_t a;
        pool_window(top.x, top.y, bot.x, bot.y, best, a);
        y[i] = best;
        if (arg) arg[i] = a;
    }
}
__global__ void __launch_bounds__(kBlock) k_maxpool2_bwd(size_t total, int H, int W, const float* __restrict__ dy,
                                                        const uint8_t* __restrict__ arg, float* __restrict__ dx) {
    const int P = H / 2, Q = W / 2;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int q = f % Q; f /= Q;
        const int p = f % P; f /= P;
        const float g = dy[i];
        const int a = arg[i];
        float2 top, bot;
        top.x = a == 0 ? g : 0.f; top.y = a == 1 ? g : 0.f;
        bot.x = a == 2 ? g : 0.f; bot.y = a == 3 ? g : 0.f;
        *reinterpret_cast<float2*>(dx + (f * H + 2 * p) * W + 2 * q) = top;
        *reinterpret_cast<float2*>(dx + (f * H + 2 * p + 1) * W + 2 * q) = bot;
    }
}

// max-pool backward fused with the ReLU that preceded the pool: the gradient reaches the argmax position only if the
// pooled value (= the ReLU output there) is positive.  Equals cnn_maxpool2_bwd followed by cnn_relu_bwd.
__global__ void __launch_bounds__(kBlock) k_maxpool2_relu_bwd(size_t total, int H, int W, const float* __restrict__ dy,
                                                             const uint8_t* __restrict__ arg,
                                                             const float* __restrict__ y, float* __restrict__ dz) {
    const int P = H / 2, Q = W / 2;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int q = f % Q; f /= Q;
        const int p = f % P; f /= P;
        const float g = y[i] > 0.f ? dy[i] : 0.f;
        const int a = arg[i];
        float2 top, bot;
        top.x = a == 0 ? g : 0.f; top.y = a == 1 ? g : 0.f;
        bot.x = a == 2 ? g : 0.f; bot.y = a == 3 ? g : 0.f;
        *reinterpret_cast<float2*>(dz + (f * H + 2 * p) * W + 2 * q) = top;
        *reinterpret_cast<float2*>(dz + (f * H + 2 * p + 1) * W + 2 * q) = bot;
    }
}

// softmax cross-entropy: one workgroup per sample; max and sum by LDS tree reduction.  ROW_IN_LDS: the row is read
// from memory once and kept in LDS (first as logits, then as exponentials), so each element costs one read, one
// exponential and one write; otherwise three passes over memory with the exponential taken twice (same values, same
// summation order either way).
template <bool ROW_IN_LDS>
__global__ void __launch_bounds__(kBlock) k_softmax_xent(int N, int O, const float* __restrict__ z,
                                                        const int32_t* __restrict__ label,
                                                        float* __restrict__ loss, float* __restrict__ dz) {
    __shared__ float red[kBlock];
    extern __shared__ float row[];              // O floats when ROW_IN_LDS
    const int n = blockIdx.x;
    const float* zr = z + (size_t)n * O;
    float m = -INFINITY;
    for (int o = threadIdx.x; o < O; o += kBlock) {
        const float t = zr[o];
        if (ROW_IN_LDS) row[o] = t;
        m = fmaxf(m, t);
    }
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s = kBlock / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    m = red[0];
    __syncthreads();
    // labels live in device memory, so the host cannot validate them: a label outside [0, O) reads nothing, gives
    // this sample a NaN loss and leaves its row of dz as the plain softmax / N
    const int lab = label[n];
    const bool lab_ok = (unsigned)lab < (unsigned)O;
    const float z_lab = lab_ok ? (ROW_IN_LDS ? row[lab] : zr[lab]) : 0.f;
    __syncthreads();                            // row[lab] is read before the exponentials overwrite the logits
    float sum = 0.f;
    for (int o = threadIdx.x; o < O; o += kBlock) {
        const float e = expf((ROW_IN_LDS ? row[o] : zr[o]) - m);
        if (ROW_IN_LDS) row[o] = e;
        sum += e;
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int s = kBlock / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    sum = red[0];
    if (threadIdx.x == 0 && loss) loss[n] = lab_ok ? -((z_lab - m) - logf(sum)) : __builtin_nanf("");
    if (dz) {
        const float inv = 1.0f / sum, invN = 1.0f / (float)N;
        for (int o = threadIdx.x; o < O; o += kBlock) {
            const float e = ROW_IN_LDS ? row[o] : expf(zr[o] - m);
            dz[(size_t)n * O + o] = (e * inv - (o == lab ? 1.0f : 0.0f)) * invN;
        }
    }
}

// ---------------------------------------------------------------- Section 2.3 layouts
// [outer][A][inner] <-> [outer][ceil(A/SW)][inner][SW]; one thread per packed element.
//   activations: outer = N, A = C, inner = H*W
//   transpose-weights: outer = K, A = C, inner = R*S
//   weights: element (k,c,rs) <-> packed[c][k/SW][rs][k%SW] (handled by the _wt kernels)
__global__ void __launch_bounds__(kBlock) k_pack_blocked(size_t total, int A, int inner, int SW,
                                                        const float* __restrict__ src, float* __restrict__ dst) {
    const int AB = (A + SW - 1) / SW;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int l = f % SW; f /= SW;
        const int in = f % inner; f /= inner;
        const int ab = f % AB; f /= AB;
        const int a = ab * SW + l;
        dst[i] = a < A ? src[(f * A + a) * inner + in] : 0.f;
    }
}
__global__ void __launch_bounds__(kBlock) k_unpack_blocked(size_t total, int A, int inner, int SW,
                                                          const float* __restrict__ src, float* __restrict__ dst) {
    const int AB = (A + SW - 1) / SW;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int in = f % inner; f /= inner;
        const int a = f % A; f /= A;
        dst[i] = src[((f * AB + a / SW) * inner + in) * SW + a % SW];
    }
}
__global__ void __launch_bounds__(kBlock) k_pack_wt(size_t total, int K, int C, int RS, int SW,
                                                   const float* __restrict__ kcrs, float* __restrict__ dst) {
    const int KB = (K + SW - 1) / SW;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int l = f % SW; f /= SW;
        const int rs = f % RS; f /= RS;
        const int kb = f % KB; f /= KB;
        const int c = (int)f, k = kb * SW + l;
        dst[i] = k < K ? kcrs[((size_t)k * C + c) * RS + rs] : 0.f;
    }
}
__global__ void __launch_bounds__(kBlock) k_unpack_wt(size_t total, int K, int C, int RS, int SW,
                                                     const float* __restrict__ src, float* __restrict__ kcrs) {
    const int KB = (K + SW - 1) / SW;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = blockIdx.x * (size_t)kBlock + threadIdx.x; i < total; i += stride) {
        size_t f = i;
        const int rs = f % RS; f /= RS;
        const int c = f % C; f /= C;
        const int k = (int)f;
        kcrs[i] = src[((((size_t)c * KB + k / SW) * RS) + rs) * SW + k % SW];
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int cnn_sgd_update(cnn_ctx* ctx, size_t n, float* w, const float* dw, float* v, float lr, float momentum) {
    if (!ctx || !w || !dw || n == 0) return CNN_EINVAL;
    if (!aligned16(w) || !aligned16(dw) || (v && !aligned16(v))) return CNN_EINVAL;
    const size_t n4 = n >> 2;
    const size_t groups = (n4 + kSgdBlock - 1) / kSgdBlock;
    if (groups > 0x7fffffffu) return CNN_EUNSUPPORTED;
    const unsigned grid = groups ? (unsigned)groups : 1u;     // fewer than four elements: the scalar tail alone
    static std::atomic<unsigned long long> attr_done{0}, attr_done_plain{0};      // one bit per device each
    {
        int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_sgd<true>), kSgdLds, "hipFuncSetAttribute(sgd)");
        if (st_attr == CNN_OK)
            st_attr = cnn::lds_attr_once(ctx, attr_done_plain, reinterpret_cast<const void*>(&k_sgd<false>), kSgdLdsPlain,
                                         "hipFuncSetAttribute(sgd plain)");
        if (st_attr != CNN_OK) return st_attr;
    }
    cnn::ProfScope ps(ctx, v ? "k_sgd<momentum>" : "k_sgd<plain>", 0.0);
    if (v)
        hipLaunchKernelGGL(k_sgd<true>, dim3(grid), dim3(kSgdBlock), kSgdLds, ctx->stream, n4, n, w, dw, v, lr, momentum);
    else
        hipLaunchKernelGGL(k_sgd<false>, dim3(grid), dim3(kSgdBlock), kSgdLdsPlain, ctx->stream, n4, n, w, dw, (float*)nullptr, lr,
                           0.f);
    return cnn::launch_check(ctx, "sgd_update");
}

int cnn_relu_fwd(cnn_ctx* ctx, size_t n, const float* z, float* a) {
    if (!ctx || !z || !a || n == 0 || !aligned16(z) || !aligned16(a)) return CNN_EINVAL;
    cnn::ProfScope ps_k_relu_fwd(ctx, "k_relu_fwd", 0.0);
    hipLaunchKernelGGL(k_relu_fwd, dim3(stream_grid(n >> 2, kBlock * 2)), dim3(kBlock), 0, ctx->stream, n >> 2, n,
                       reinterpret_cast<const float4*>(z), reinterpret_cast<float4*>(a));
    return cnn::launch_check(ctx, "relu_fwd");
}
int cnn_relu_bwd(cnn_ctx* ctx, size_t n, const float* z, const float* da, float* dz) {
    if (!ctx || !z || !da || !dz || n == 0 || !aligned16(z) || !aligned16(da) || !aligned16(dz)) return CNN_EINVAL;
    cnn::ProfScope ps_k_relu_bwd(ctx, "k_relu_bwd", 0.0);
    hipLaunchKernelGGL(k_relu_bwd, dim3(stream_grid(n >> 2, kBlock * 2)), dim3(kBlock), 0, ctx->stream, n >> 2, n,
                       reinterpret_cast<const float4*>(z), reinterpret_cast<const float4*>(da),
                       reinterpret_cast<float4*>(dz));
    return cnn::launch_check(ctx, "relu_bwd");
}
int cnn_sigmoid_fwd(cnn_ctx* ctx, size_t n, const float* z, float* a) {
    if (!ctx || !z || !a || n == 0) return CNN_EINVAL;
    cnn::ProfScope ps_k_sigmoid_fwd(ctx, "k_sigmoid_fwd", 0.0);
    hipLaunchKernelGGL(k_sigmoid_fwd, dim3(stream_grid(n, kBlock * 4)), dim3(kBlock), 0, ctx->stream, n, z, a);
    return cnn::launch_check(ctx, "sigmoid_fwd");
}
int cnn_sigmoid_bwd(cnn_ctx* ctx, size_t n, const float* a, const float* da, float* dz) {
    if (!ctx || !a || !da || !dz || n == 0) return CNN_EINVAL;
    cnn::ProfScope ps_k_sigmoid_bwd(ctx, "k_sigmoid_bwd", 0.0);
    hipLaunchKernelGGL(k_sigmoid_bwd, dim3(stream_grid(n, kBlock * 4)), dim3(kBlock), 0, ctx->stream, n, a, da, dz);
    return cnn::launch_check(ctx, "sigmoid_bwd");
}
int cnn_maxpool2_fwd(cnn_ctx* ctx, size_t planes, int H, int W, const float* x, float* y, uint8_t* arg) {
    if (!ctx || !x || !y || planes == 0 || H < 2 || W < 2 || (H & 1) || (W & 1)) return CNN_EINVAL;
    if (reinterpret_cast<uintptr_t>(x) & 7u) return CNN_EINVAL;
    const size_t total = planes * (size_t)(H / 2) * (W / 2);
    cnn::ProfScope ps_k_maxpool2_fwd(ctx, "k_maxpool2_fwd", 0.0);
    hipLaunchKernelGGL(k_maxpool2_fwd, dim3(stream_grid(total, kBlock * 2)), dim3(kBlock), 0, ctx->stream, total, H, W,
                       x, y, arg);
    return cnn::launch_check(ctx, "maxpool2_fwd");
}
int cnn_maxpool2_bwd(cnn_ctx* ctx, size_t planes, int H, int W, const float* dy, const uint8_t* arg, float* dx) {
    if (!ctx || !dy || !arg || !dx || planes == 0 || H < 2 || W < 2 || (H & 1) || (W & 1)) return CNN_EINVAL;
    if (reinterpret_cast<uintptr_t>(dx) & 7u) return CNN_EINVAL;
    const size_t total = planes * (size_t)(H / 2) * (W / 2);
    cnn::ProfScope ps_k_maxpool2_bwd(ctx, "k_maxpool2_bwd", 0.0);
    hipLaunchKernelGGL(k_maxpool2_bwd, dim3(stream_grid(total, kBlock * 2)), dim3(kBlock), 0, ctx->stream, total, H, W,
                       dy, arg, dx);
    return cnn::launch_check(ctx, "maxpool2_bwd");
}
int cnn_maxpool2_relu_bwd(cnn_ctx* ctx, size_t planes, int H, int W, const float* dy, const uint8_t* arg,
                          const float* y, float* dz) {
    if (!ctx || !dy || !arg || !y || !dz || planes == 0 || H < 2 || W < 2 || (H & 1) || (W & 1)) return CNN_EINVAL;
    if (reinterpret_cast<uintptr_t>(dz) & 7u) return CNN_EINVAL;
    const size_t total = planes * (size_t)(H / 2) * (W / 2);
    cnn::ProfScope ps(ctx, "k_maxpool2_relu_bwd", 0.0);
    hipLaunchKernelGGL(k_maxpool2_relu_bwd, dim3(stream_grid(total, kBlock * 2)), dim3(kBlock), 0, ctx->stream, total, H,
                       W, dy, arg, y, dz);
    return cnn::launch_check(ctx, "maxpool2_relu_bwd");
}
int cnn_softmax_xent(cnn_ctx* ctx, int N, int O, const float* z, const int32_t* label, float* loss, float* dz) {
    if (!ctx || !z || !label || N <= 0 || O <= 0) return CNN_EINVAL;
    cnn::ProfScope ps_k_softmax_xent(ctx, "k_softmax_xent", 0.0);
    if ((size_t)O * sizeof(float) <= 40 * 1024)      // the row fits the default LDS allowance beside the reduction buffer
        hipLaunchKernelGGL(k_softmax_xent<true>, dim3(N), dim3(kBlock), (size_t)O * sizeof(float), ctx->stream, N, O, z, label,
                           loss, dz);
    else
        hipLaunchKernelGGL(k_softmax_xent<false>, dim3(N), dim3(kBlock), 0, ctx->stream, N, O, z, label, loss, dz);
    return cnn::launch_check(ctx, "softmax_xent");
}

size_t cnn_packed_act_elems(int N, int C, int H, int W, int SW) {
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || SW <= 0) return 0;
    return (size_t)N * ((C + SW - 1) / SW) * H * W * SW;
}
size_t cnn_packed_wt_elems(int K, int C, int R, int S, int SW, int transpose) {
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0 || SW <= 0) return 0;
    return transpose ? (size_t)K * ((C + SW - 1) / SW) * R * S * SW : (size_t)C * ((K + SW - 1) / SW) * R * S * SW;
}
int cnn_pack_act(cnn_ctx* ctx, int N, int C, int H, int W, int SW, const float* nchw, float* packed) {
    const size_t total = cnn_packed_act_elems(N, C, H, W, SW);
    if (!ctx || !nchw || !packed || total == 0) return CNN_EINVAL;
    cnn::ProfScope ps_k_pack_blocked(ctx, "k_pack_blocked", 0.0);
    hipLaunchKernelGGL(k_pack_blocked, dim3(stream_grid(total, kBlock * 4)), dim3(kBlock), 0, ctx->stream, total, C,
                       H * W, SW, nchw, packed);
    return cnn::launch_check(ctx, "pack_act");
}
int cnn_unpack_act(cnn_ctx* ctx, int N, int C, int H, int W, int SW, const float* packed, float* nchw) {
    if (!ctx || !nchw || !packed || cnn_packed_act_elems(N, C, H, W, SW) == 0) return CNN_EINVAL;
    const size_t total = (size_t)N * C * H * W;
    cnn::ProfScope ps_k_unpack_blocked(ctx, "k_unpack_blocked", 0.0);
    hipLaunchKernelGGL(k_unpack_blocked, dim3(stream_grid(total, kBlock * 4)), dim3(kBlock), 0, ctx->stream, total, C,
                       H * W, SW, packed, nchw);
    return cnn::launch_check(ctx, "unpack_act");
}
int cnn_pack_wt(cnn_ctx* ctx, int K, int C, int R, int S, int SW, int transpose, const float* kcrs, float* packed) {
    const size_t total = cnn_packed_wt_elems(K, C, R, S, SW, transpose);
    if (!ctx || !kcrs || !packed || total == 0) return CNN_EINVAL;
    cnn::ProfScope ps(ctx, "k_pack_wt", 0.0);
    if (transpose)
        hipLaunchKernelGGL(k_pack_blocked, dim3(stream_grid(total, kBlock * 4)), dim3(kBlock), 0, ctx->stream, total,
                           C, R * S, SW, kcrs, packed);
    else
        hipLaunchKernelGGL(k_pack_wt, dim3(stream_grid(total, kBlock * 4)), dim3(kBlock), 0, ctx->stream, total, K, C,
                           R * S, SW, kcrs, packed);
    return cnn::launch_check(ctx, "pack_wt");
}
int cnn_unpack_wt(cnn_ctx* ctx, int K, int C, int R, int S, int SW, int transpose, const float* packed, float* kcrs) {
    if (!ctx || !kcrs || !packed || cnn_packed_wt_elems(K, C, R, S, SW, transpose) == 0) return CNN_EINVAL;
    const size_t total = (size_t)K * C * R * S;
    cnn::ProfScope ps(ctx, "k_unpack_wt", 0.0);
    if (transpose)
        hipLaunchKernelGGL(k_unpack_blocked, dim3(stream_grid(total, kBlock * 4)), dim3(kBlock), 0, ctx->stream, total,
                           C, R * S, SW, packed, kcrs);
    else
        hipLaunchKernelGGL(k_unpack_wt, dim3(stream_grid(total, kBlock * 4)), dim3(kBlock), 0, ctx->stream, total, K, C,
                           R * S, SW, packed, kcrs);
    return cnn::launch_check(ctx, "unpack_wt");
}

}  // extern "C"
