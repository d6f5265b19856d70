// Cache-blocking model of Section 2.2: bytes-to-FLOPs ratios and the exhaustive search for the block of least B/F
// that fits the on-chip memory, run as a GPU kernel (the paper's "multithreaded brute-force state space search";
// here one thread per row of the candidate space and a two-stage minimum).
//
// Single-cache model as printed: block = (b1_0 images, b1_1 output features, b2_0 input features, b1_2 x b1_3
// output pixels, b2_2 x b2_3 kernel taps);
//   BS = 4 * (b1_0*b1_1*b1_2*b1_3 + b2_0*b1_1*b2_2*b2_3 + b1_0*b2_0*(b1_2*s + b2_2 - 1)*(b1_3*s + b2_3 - 1))
//   CPB = 2 * b1_0*b1_1*b2_0*b1_2*b1_3*b2_2*b2_3 (input features included: the whole-layer ratio needs them)
//   minimise BS / CPB subject to BS < cache_bytes, b1_1 a multiple of the SIMD width.
// Traversal model (the section's remark that walking along the input features precludes reading the output block),
// the form that fits a GPU: the output block stays in accumulator registers, weights and inputs stream through a
// double-buffered staging memory (LDS) one chunk of input features at a time:
//   bytes = 4 * (b1_0*b1_1*b1_2*b1_3 + ifm*(b1_1*k_h*k_w + b1_0*in_h*in_w)), FLOPs = 2*b1_0*b1_1*ifm*b1_2*b1_3*k_h*k_w
//   subject to 4*b1_0*b1_1*b1_2*b1_3 <= acc_bytes and 2*4*b2_0*(b1_1*k_h*k_w + b1_0*in_h*in_w) <= stage_bytes.
// Candidates are numbered in loop order (b1_0, b1_1, b2_0, b1_2, b1_3, b2_2, b2_3; leftmost slowest); among equal
// ratios the lowest number wins, so the result does not depend on how the space is spread over threads.
#include "common.h"

namespace {

struct Layer {
    int n, c, k, p, q, r, s, stride;
    int nkb, simd;          // blocks of output features: (i + 1) * simd, or the single block k when k < simd
    int ncb, chunk;         // traversal model: chunks of input features
};

struct Key {
    double bf;
    unsigned long long idx;     // ~0: nothing found
};
__device__ __forceinline__ bool better(const Key& a, const Key& b) {
    if (a.idx == ~0ull) return false;
    if (b.idx == ~0ull) return true;
    return a.bf < b.bf || (a.bf == b.bf && a.idx < b.idx);
}

struct Partial {
    double bf;
    unsigned long long idx;
    unsigned long long feasible;
};

constexpr int kThreads = 256;
constexpr int kMaxGroups = 2048;

__device__ __forceinline__ int ofm_block(const Layer& L, int i) { return L.k < L.simd ? L.k : (i + 1) * L.simd; }

// workgroup minimum of (key, count) -> partial[blockIdx.x]
__device__ void group_reduce(Key best, unsigned long long feasible, Partial* __restrict__ partial) {
    __shared__ Partial sh[kThreads / 64];
    for (int off = 32; off > 0; off >>= 1) {
        Key o;
        o.bf = __shfl_down(best.bf, off);
        o.idx = __shfl_down(best.idx, off);
        feasible += __shfl_down(feasible, off);
        if (better(o, best)) best = o;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) sh[wave] = Partial{best.bf, best.idx, feasible};
    __syncthreads();
    if (threadIdx.x == 0) {
        Partial t = sh[0];
        for (int w = 1; w < kThreads / 64; ++w) {
            t.feasible += sh[w].feasible;
            if (better(Key{sh[w].bf, sh[w].idx}, Key{t.bf, t.idx})) { t.bf = sh[w].bf; t.idx = sh[w].idx; }
        }
        partial[blockIdx.x] = t;
    }
}

// One thread per row (b1_0, b1_1, b2_0, b1_2) of the candidate space, grid-strided; the row's b1_3, b2_2, b2_3 are
// walked in order.  BS grows with every block dimension, so a row ends at the first b1_3 whose smallest block
// (one tap) no longer fits.
__global__ void __launch_bounds__(kThreads) k_block_search(Layer L, long long cache_bytes, unsigned long long rows,
                                                          Partial* __restrict__ partial) {
    Key best{0.0, ~0ull};
    unsigned long long feasible = 0;
    for (unsigned long long row = blockIdx.x * (unsigned long long)kThreads + threadIdx.x; row < rows;
         row += (unsigned long long)gridDim.x * kThreads) {
        unsigned long long t = row;
        const long long bp = (long long)(t % L.p) + 1; t /= L.p;
        const long long bc = (long long)(t % L.c) + 1; t /= L.c;
        const long long bk = ofm_block(L, (int)(t % L.nkb)); t /= L.nkb;
        const long long bn = (long long)t + 1;
        const unsigned long long row_idx = row * L.q * L.r * L.s;
        for (long long bq = 1; bq <= L.q; ++bq) {
            const long long out = bn * bk * bp * bq;
            if (!(4 * (out + bc * bk + bn * bc * (bp * L.stride) * (bq * L.stride)) < cache_bytes)) break;
            for (long long br = 1; br <= L.r; ++br)
                for (long long bs = 1; bs <= L.s; ++bs) {
                    const long long bytes = 4 * (out + bc * bk * br * bs +
                                                 bn * bc * (bp * L.stride + br - 1) * (bq * L.stride + bs - 1));
                    if (!(bytes < cache_bytes)) continue;
                    ++feasible;
                    const long long flops = 2 * bn * bk * bc * bp * bq * br * bs;
                    const Key cand{(double)bytes / (double)flops,
                                   row_idx + (unsigned long long)(((bq - 1) * L.r + (br - 1)) * L.s + (bs - 1))};
                    if (better(cand, best)) best = cand;
                }
        }
    }
    group_reduce(best, feasible, partial);
}

// Traversal model: one thread per (b1_0, b1_1, b2_0, b1_2), walking b1_3.
__global__ void __launch_bounds__(kThreads) k_block_search_trav(Layer L, long long acc_bytes, long long stage_bytes,
                                                               unsigned long long rows, Partial* __restrict__ partial) {
    Key best{0.0, ~0ull};
    unsigned long long feasible = 0;
    for (unsigned long long row = blockIdx.x * (unsigned long long)kThreads + threadIdx.x; row < rows;
         row += (unsigned long long)gridDim.x * kThreads) {
        unsigned long long t = row;
        const long long bp = (long long)(t % L.p) + 1; t /= L.p;
        const long long bc = ((long long)(t % L.ncb) + 1) * L.chunk; t /= L.ncb;
        const long long bk = ofm_block(L, (int)(t % L.nkb)); t /= L.nkb;
        const long long bn = (long long)t + 1;
        const long long in_h = bp * L.stride + L.r - 1;
        for (long long bq = 1; bq <= L.q; ++bq) {
            const long long out = bn * bk * bp * bq;
            if (4 * out > acc_bytes) break;                        // grows with b1_3
            const long long in = in_h * (bq * L.stride + L.s - 1);
            if (2 * 4 * bc * (bk * L.r * L.s + bn * in) > stage_bytes) break;
            ++feasible;
            const long long bytes = 4 * (out + (long long)L.c * (bk * L.r * L.s + bn * in));
            const long long flops = 2 * bn * bk * L.c * bp * bq * L.r * L.s;
            const Key cand{(double)bytes / (double)flops, row * L.q + (unsigned long long)(bq - 1)};
            if (better(cand, best)) best = cand;
        }
    }
    group_reduce(best, feasible, partial);
}

// Second stage: minimum over the workgroups' partials, then the winning number is turned back into a block.
__global__ void __launch_bounds__(kThreads) k_block_search_finish(Layer L, int traversal, int groups,
                                                                 const Partial* __restrict__ partial,
                                                                 cnn_block_result* __restrict__ result) {
    __shared__ Partial total;
    Key best{0.0, ~0ull};
    unsigned long long feasible = 0;
    for (int g = threadIdx.x; g < groups; g += kThreads) {
        const Partial t = partial[g];
        feasible += t.feasible;
        if (better(Key{t.bf, t.idx}, best)) best = Key{t.bf, t.idx};
    }
    group_reduce(best, feasible, &total);        // launched as one workgroup: blockIdx.x == 0
    __syncthreads();
    if (threadIdx.x != 0) return;
    cnn_block_result r;
    for (int i = 0; i < 7; ++i) r.block[i] = 0;
    r.found = total.idx != ~0ull;
    r.bf = r.found ? total.bf : 0.0;
    r.feasible = total.feasible;
    if (r.found) {
        unsigned long long t = total.idx;
        if (!traversal) {
            r.block[6] = (int)(t % L.s) + 1; t /= L.s;
            r.block[5] = (int)(t % L.r) + 1; t /= L.r;
        }
        r.block[4] = (int)(t % L.q) + 1; t /= L.q;
        r.block[3] = (int)(t % L.p) + 1; t /= L.p;
        if (traversal) { r.block[2] = ((int)(t % L.ncb) + 1) * L.chunk; t /= L.ncb; }
        else { r.block[2] = (int)(t % L.c) + 1; t /= L.c; }
        r.block[1] = ofm_block(L, (int)(t % L.nkb)); t /= L.nkb;
        r.block[0] = (int)t + 1;
    }
    *result = r;
}

bool fill_layer(int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride, int simd, int chunk,
                Layer* L) {
    if (minibatch <= 0 || ifm <= 0 || ofm <= 0 || out_h <= 0 || out_w <= 0 || k_h <= 0 || k_w <= 0 || stride <= 0 ||
        simd <= 0 || chunk <= 0)
        return false;
    *L = Layer{minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride, ofm < simd ? 1 : ofm / simd, simd,
               (ifm + chunk - 1) / chunk, chunk};
    return true;
}

// every product formed in the kernels stays below 2^62
bool in_range(const Layer& L) {
    const double in = ((double)L.p * L.stride + L.r) * ((double)L.q * L.stride + L.s);
    const double big = 8.0 * L.n * ((double)L.k + L.simd) * ((double)L.c + L.chunk) * in * L.r * L.s;
    return big < 4.0e18;
}

int launch_search(cnn_ctx* ctx, const Layer& L, int traversal, long long a, long long b, cnn_block_result* result) {
    if (!ctx->ws || ctx->ws_bytes < kMaxGroups * sizeof(Partial)) return CNN_EWORKSPACE;
    const unsigned long long rows = (unsigned long long)L.n * L.nkb * (traversal ? L.ncb : L.c) * L.p;
    unsigned long long groups = (rows + kThreads - 1) / kThreads;
    if (groups > kMaxGroups) groups = kMaxGroups;
    Partial* partial = reinterpret_cast<Partial*>(ctx->ws);
    {
        cnn::ProfScope ps(ctx, traversal ? "k_block_search_trav" : "k_block_search", 0.0);
        if (traversal)
            hipLaunchKernelGGL(k_block_search_trav, dim3((unsigned)groups), dim3(kThreads), 0, ctx->stream, L, a, b, rows,
                               partial);
        else
            hipLaunchKernelGGL(k_block_search, dim3((unsigned)groups), dim3(kThreads), 0, ctx->stream, L, a, rows, partial);
    }
    int st = cnn::launch_check(ctx, "block_search");
    if (st != CNN_OK) return st;
    hipLaunchKernelGGL(k_block_search_finish, dim3(1), dim3(kThreads), 0, ctx->stream, L, traversal, (int)groups, partial,
                       result);
    return cnn::launch_check(ctx, "block_search_finish");
}

}  // namespace

namespace cnn {
size_t block_search_ws() { return kMaxGroups * sizeof(Partial); }
}  // namespace cnn

extern "C" {

double cnn_bf_plane(int out_h, int out_w, int k_h, int k_w, int stride) {
    if (out_h <= 0 || out_w <= 0 || k_h <= 0 || k_w <= 0 || stride <= 0) return -1.0;
    const double in = ((double)out_h * stride + k_h - 1) * ((double)out_w * stride + k_w - 1);
    return 4.0 * ((double)out_h * out_w + in + (double)k_h * k_w) / (2.0 * k_h * k_w * out_h * out_w);
}

double cnn_bf_layer(int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride) {
    if (minibatch <= 0 || ifm <= 0 || ofm <= 0 || out_h <= 0 || out_w <= 0 || k_h <= 0 || k_w <= 0 || stride <= 0)
        return -1.0;
    const double in = ((double)out_h * stride + k_h - 1) * ((double)out_w * stride + k_w - 1);
    const double px = (double)out_h * out_w, taps = (double)k_h * k_w;
    return 4.0 * (minibatch * ofm * px + minibatch * ifm * in + ifm * ofm * taps) / (2.0 * minibatch * ofm * ifm * taps * px);
}

double cnn_bf_block_traversal(int ifm, int k_h, int k_w, int stride, int images, int ofm_block, int rows, int cols) {
    if (ifm <= 0 || k_h <= 0 || k_w <= 0 || stride <= 0 || images <= 0 || ofm_block <= 0 || rows <= 0 || cols <= 0)
        return -1.0;
    const double in = ((double)rows * stride + k_h - 1) * ((double)cols * stride + k_w - 1);
    const double out = (double)images * ofm_block * rows * cols, taps = (double)k_h * k_w;
    return 4.0 * (out + ifm * (ofm_block * taps + images * in)) / (2.0 * out * ifm * taps);
}

int cnn_block_search(cnn_ctx* ctx, int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride,
                     int64_t cache_bytes, int simd, cnn_block_result* result) {
    Layer L;
    if (!ctx || !result || (reinterpret_cast<uintptr_t>(result) & 7u) || cache_bytes <= 0 ||
        !fill_layer(minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride, simd, 1, &L))
        return CNN_EINVAL;
    if (!in_range(L)) return CNN_EUNSUPPORTED;
    return launch_search(ctx, L, 0, cache_bytes, 0, result);
}

int cnn_block_search_traversal(cnn_ctx* ctx, int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w,
                               int stride, int64_t acc_bytes, int64_t stage_bytes, int simd, int chunk,
                               cnn_block_result* result) {
    Layer L;
    if (!ctx || !result || (reinterpret_cast<uintptr_t>(result) & 7u) || acc_bytes <= 0 || stage_bytes <= 0 ||
        !fill_layer(minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride, simd, chunk, &L))
        return CNN_EINVAL;
    if (!in_range(L)) return CNN_EUNSUPPORTED;
    return launch_search(ctx, L, 1, acc_bytes, stage_bytes, result);
}

}  // extern "C"
