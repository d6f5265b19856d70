// Forward propagation (Section 2.1, Algorithm 1) for a strided first layer: three input feature maps, a large
// kernel and stride > 1 (OverFeat-FAST's 11x11 / stride 4).  The generic tiled kernel needs stride 1; here
//   D[k][pixel] = sum_j w[k][j] * x[c_j][p*ST + r_j][q*ST + s_j],   j = (c, r, s)
// runs on the fp32 matrix cores with A = filters (lane = output feature), B = input gathered from an LDS tile
// (lane = output pixel), one kernel row r per chunk (j' = (c, s): C*S of them, split between the wave halves).
// With stride ST the 32 lanes of a B operand would read every ST-th word (ST-way bank conflicts), so the tile is
// stored de-interleaved by column phase: x[c][row][w] -> xl[c][row][w % ST][w / ST]; lane q then reads
// consecutive words for any tap.  The input tile (all rows the TH output rows need) is loaded once per workgroup,
// the filter chunk of the next kernel row is fetched while the current one is multiplied.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int R_, int S_, int ST_, int TH_, int WI_, int KBK_, int NT_>
struct C3Cfg {
    static constexpr int R = R_, S = S_, ST = ST_, TH = TH_, WI = WI_, KBK = KBK_, NT = NT_, C = 3;
    static constexpr int WO = (WI - S) / ST + 1;
    static constexpr int ROWS = (TH - 1) * ST + R;               // input rows of one tile
    static constexpr int PW = (WI + ST - 1) / ST;                 // words per column phase
    static constexpr int ROWP = ST * PW;                          // LDS words per input row
    static constexpr int PLANE = ROWS * ROWP;
    static constexpr int JC = C * S;                              // contraction entries per kernel row
    static constexpr int HALF = (JC + 1) / 2;                     // per wave half (the last one may be a zero dummy)
    static constexpr int WSTR = 2 * HALF + 1;                     // odd LDS row stride of the filter chunk
    static constexpr int KROWS = 32 * KBK;
    static constexpr int T = 64 * KBK;
    static constexpr int NPIX = TH * WO;
    static constexpr int WSL = (KROWS * JC + T - 1) / T;          // filter elements fetched per thread per chunk
    static constexpr int LDS_BYTES = (C * PLANE + 2 * KROWS * WSTR) * 4;
    static_assert(NT * 32 >= NPIX && NT * 32 - NPIX < 32, "pixel tile padded by less than one block");
};

template <class G>
__global__ void __launch_bounds__(G::T)
k_conv_c3_strided(int N, int K, int HI, int HO, int row_tiles, int relu, const float* __restrict__ x,
                  const float* __restrict__ w, float* __restrict__ y) {
    constexpr int R = G::R, S = G::S, ST = G::ST, NT = G::NT, T = G::T, C = G::C;
    extern __shared__ float lds[];
    float* xl = lds;                       // [C][ROWS][ST][PW]
    float* wl = lds + C * G::PLANE;        // [2][KROWS][WSTR]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int n = blockIdx.x / row_tiles, p0 = (blockIdx.x % row_tiles) * G::TH;

    // ---- input tile, de-interleaved by column phase (rows past the image are zero)
    const float* xs = x + (size_t)n * C * HI * G::WI;
    for (int e = tid; e < C * G::ROWS * G::WI; e += T) {
        const int c = e / (G::ROWS * G::WI), rem = e % (G::ROWS * G::WI), row = rem / G::WI, col = rem % G::WI;
        const int h = p0 * ST + row;
        xl[c * G::PLANE + row * G::ROWP + (col % ST) * G::PW + col / ST] =
            h < HI ? xs[((size_t)c * HI + h) * G::WI + col] : 0.f;
    }

    // ---- filter chunk staging: element e of the chunk -> (feature k, j' = c*S + s)
    float wr[G::WSL];
    auto fetch_w = [&](int r) {
#pragma unroll
        for (int i = 0; i < G::WSL; ++i) {
            const int e = tid + i * T;
            float v = 0.f;
            if (e < G::KROWS * G::JC) {
                const int k = e / G::JC, jj = e % G::JC, c = jj / S, s = jj % S;
                if (k < K) v = w[(((size_t)k * C + c) * R + r) * S + s];
            }
            wr[i] = v;
        }
    };
    auto stage_w = [&](int buf) {
#pragma unroll
        for (int i = 0; i < G::WSL; ++i) {
            const int e = tid + i * T;
            if (e < G::KROWS * G::JC) wl[(buf * G::KROWS + e / G::JC) * G::WSTR + e % G::JC] = wr[i];
        }
    };
    // the dummy entry (j' = JC when JC is odd) must be zero in both buffers
    if (2 * G::HALF > G::JC)
        for (int e = tid; e < 2 * G::KROWS; e += T) wl[e * G::WSTR + G::JC] = 0.f;

    const int a_base = (wave * 32 + l32) * G::WSTR + half * G::HALF;
    int b_base[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = j * 32 + l32;
        b_base[j] = i < G::NPIX ? (i / G::WO) * ST * G::ROWP + i % G::WO : 0;
    }
    f32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    fetch_w(0);
    stage_w(0);
    if (R > 1) fetch_w(1);
    __syncthreads();
    for (int r = 0; r < R; ++r) {
        const int buf = r & 1;
        if (r + 1 < R) stage_w(buf ^ 1);           // next kernel row's filters into the other buffer
        if (r + 2 < R) fetch_w(r + 2);
        const float* wb = wl + buf * G::KROWS * G::WSTR + a_base;
        const float* xb = xl + r * G::ROWP;
#pragma unroll
        for (int t = 0; t < G::HALF; ++t) {
            // low half: j' = t, high half: j' = t + HALF (compile-time offsets, selected per lane)
            constexpr int dummy = 0;
            const int jl = t, jh = t + G::HALF < G::JC ? t + G::HALF : dummy;
            const int ol = (jl / S) * G::PLANE + ((jl % S) % ST) * G::PW + (jl % S) / ST;
            const int oh = (jh / S) * G::PLANE + ((jh % S) % ST) * G::PW + (jh % S) / ST;
            const int off = half ? oh : ol;
            const float a = wb[t];
            float b[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = xb[b_base[j] + off];
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[j], acc[j], 0, 0, 0);
        }
        __syncthreads();
    }

    const size_t out_plane = (size_t)HO * G::WO;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = j * 32 + l32;
        if (i >= G::NPIX) continue;
        const int p = p0 + i / G::WO, q = i % G::WO;
        if (p >= HO) continue;
        float* o = y + ((size_t)n * K) * out_plane + (size_t)p * G::WO + q;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = wave * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (k < K) {
                float rr = acc[j][v];
                if (relu) rr = rr > 0.f ? rr : 0.f;
                o[(size_t)k * out_plane] = rr;
            }
        }
    }
}

}  // namespace

namespace cnn {

int c3_strided_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* y, int relu) {
    // OverFeat-FAST's first layer: 3 x 231 x 231 -> 96 x 56 x 56, 11x11, stride 4, pad 0
    using G = C3Cfg<11, 11, 4, 4, 231, 3, 7>;
    if (s.C != 3 || s.R != G::R || s.S != G::S || s.stride != G::ST || s.pad != 0 || s.W != G::WI || s.H != s.W ||
        s.K > G::KROWS)
        return CNN_EUNSUPPORTED;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_conv_c3_strided<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (e != hipSuccess) return hip_check(ctx, e, "hipFuncSetAttribute(conv_c3_strided)");
        attr_done = true;
    }
    const int row_tiles = (s.P + G::TH - 1) / G::TH;
    {
        ProfScope ps(ctx, "k_conv_c3_strided<11x11 s4 TH4 W231>", conv_flops(s));
        hipLaunchKernelGGL(k_conv_c3_strided<G>, dim3((unsigned)(s.N * row_tiles)), dim3(G::T), G::LDS_BYTES, ctx->stream, s.N,
                           s.K, s.H, s.P, row_tiles, relu, x, w, y);
    }
    return launch_check(ctx, "conv_c3_strided");
}

}  // namespace cnn
