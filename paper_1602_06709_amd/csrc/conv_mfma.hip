// Stride-1 convolution as an implicit contraction over (channel, kernel row, kernel col) on the fp32
// matrix cores of gfx950 (v_mfma_f32_32x32x2_f32).  One kernel serves
//   forward propagation  (Section 2.1, Algorithm 1):  out = y,  in = x,  contraction over ifm
//   backpropagation      (Section 2.1):               out = dx, in = dy, contraction over ofm,
//                                                      kernel taps mirrored, pad' = R-1-pad
// which is the paper's remark that the passes share one loop nest and one blocking strategy.
//
// Tiling (per workgroup): MB = 32*WM output features x NPIX = NB*TH*WO output pixels
// (NB images x TH full-width output rows).  Each wave owns 32 output features x NT blocks of
// 32 pixels: NT accumulators of 16 VGPRs.  The contraction runs over chunks of CB channels:
//   LDS  wl[MB][CB*R*S + 1]      filter tile, row stride odd  -> the 32 lanes of an A operand
//                                (one output feature each) hit 32 different banks
//   LDS  xl[CB][NB][TH+R-1][WI+2*PADE]   input tile with its halo, zeros where the image ends;
//                                lanes of a B operand are consecutive pixels -> consecutive words
// The two halves of the 64-lane wave feed k = 0 and k = 1 of the MFMA: the low half walks channels
// [0, CB/2) of the chunk and the high half [CB/2, CB), so both halves use the same immediate offsets.
// The next chunk is fetched from HBM into registers while the current one is multiplied.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int R_, int S_, int PADE_, int CB_, int WM_, int WN_, int NT_, int NB_, int TH_, int WI_>
struct ConvCfg {
    static constexpr int R = R_, S = S_, PADE = PADE_, CB = CB_, WM = WM_, WN = WN_, NT = NT_, NB = NB_, TH = TH_, WI = WI_;
    static constexpr int RS = R * S;
    static constexpr int WO = WI + 2 * PADE - S + 1;
    static constexpr int THI = TH + R - 1;
    static constexpr int WLD = WI + 2 * PADE;
    static constexpr int PLANE = NB * THI * WLD;
    static constexpr int MB = 32 * WM;
    static constexpr int NPIX = NB * TH * WO;
    static constexpr int NPIXB = WN * NT * 32;              // padded to whole MFMA column blocks
    static constexpr int T = WM * WN * 64;
    static constexpr int KCH = CB * RS;                      // contraction length of one chunk
    static constexpr int WSTR = (KCH % 2 == 0) ? KCH + 1 : KCH;
    static constexpr int XTOT = CB * PLANE;
    static constexpr int XP = (PLANE + T - 1) / T;           // input-tile positions per thread (per channel)
    static constexpr int Q4 = KCH / 4;                       // float4s per filter row
    static constexpr int RPP = T / Q4;                       // filter rows fetched per pass of the workgroup
    static constexpr int WSL = (MB + RPP - 1) / RPP;         // passes
    static constexpr int LDS_BYTES = (MB * WSTR + XTOT) * 4;
    static_assert(CB % 2 == 0, "the two wave halves split the chunk's channels");
    static_assert(KCH % 4 == 0, "filter tile is fetched as float4");
    static_assert(NPIXB >= NPIX && NPIXB - NPIX < 32 * WN, "pixel tile padded by less than one block per wave column");
};

template <class G>
__global__ void __launch_bounds__(G::T, 2)
k_conv_s1(int N, int J, int M, int HI, int HO, int row_tiles,
          const float* __restrict__ in, const float* __restrict__ wt, float* __restrict__ out) {
    constexpr int R = G::R, S = G::S, RS = G::RS, CB = G::CB, NT = G::NT, T = G::T;
    extern __shared__ float lds[];
    float* wl = lds;
    float* xl = lds + G::MB * G::WSTR;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm = wave % G::WM, wn = wave / G::WM;

    const int ptile = blockIdx.x;
    const int n0 = (ptile / row_tiles) * G::NB;
    const int p0 = (ptile % row_tiles) * G::TH;
    const int m0 = blockIdx.y * G::MB;

    const size_t in_img = (size_t)J * HI * G::WI;      // elements per image of `in`
    const float* in_base = in + (size_t)n0 * in_img;
    const int plane_g = HI * G::WI;

    // ---- input tile staging: each thread owns XP positions of the (image, row, col) plane and fetches
    //      them for every channel of the chunk (-1 = outside the image: zero fill)
    int xoff[G::XP];
#pragma unroll
    for (int j = 0; j < G::XP; ++j) {
        const int e = tid + j * T;
        int off = -1;
        if (e < G::PLANE) {
            const int nb = e / (G::THI * G::WLD), rem = e % (G::THI * G::WLD);
            const int row = rem / G::WLD, col = rem % G::WLD;
            const int h = p0 - G::PADE + row, w = col - G::PADE;
            if (n0 + nb < N && h >= 0 && h < HI && w >= 0 && w < G::WI) off = nb * (int)in_img + h * G::WI + w;
        }
        xoff[j] = off;
    }
    // ---- filter tile staging: thread = (row m_sub, float4 kq) of a pass over RPP rows
    const int w_msub = tid / G::Q4, w_kq = tid % G::Q4;
    const bool w_thread = tid < G::RPP * G::Q4;
    const float* w_src = wt + ((size_t)(m0 + w_msub) * J) * RS + w_kq * 4;
    float* w_dst = wl + w_msub * G::WSTR + w_kq * 4;

    // ---- per-lane LDS read bases
    const int a_base = (wm * 32 + l32) * G::WSTR + half * (CB / 2) * RS;
    int b_base[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = (wn * NT + j) * 32 + l32;
        int o = 0;
        if (i < G::NPIX) {
            const int nb = i / (G::TH * G::WO), rem = i % (G::TH * G::WO);
            o = (nb * G::THI + rem / G::WO) * G::WLD + rem % G::WO;
        }
        b_base[j] = o + half * (CB / 2) * G::PLANE;
    }

    f32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    float xr[CB][G::XP];
    float4 wr[G::WSL];

    auto fetch = [&](int c0) {
        const float* src = in_base + (size_t)c0 * plane_g;
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int j = 0; j < G::XP; ++j) xr[c][j] = xoff[j] >= 0 ? src[xoff[j] + c * plane_g] : 0.f;
        // w[m][c0 .. c0+CB)[R][S]: CB*R*S contiguous floats per output feature
#pragma unroll
        for (int i = 0; i < G::WSL; ++i) {
            const int m = w_msub + i * G::RPP;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (w_thread && m < G::MB && m0 + m < M)
                v = *reinterpret_cast<const float4*>(w_src + ((size_t)i * G::RPP * J + c0) * RS);
            wr[i] = v;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int j = 0; j < G::XP; ++j)
                if (tid + j * T < G::PLANE) xl[c * G::PLANE + tid + j * T] = xr[c][j];
#pragma unroll
        for (int i = 0; i < G::WSL; ++i) {
            if (w_thread && w_msub + i * G::RPP < G::MB) {
                float* d = w_dst + i * G::RPP * G::WSTR;
                d[0] = wr[i].x; d[1] = wr[i].y; d[2] = wr[i].z; d[3] = wr[i].w;
            }
        }
    };

    const int nchunks = J / CB;
    fetch(0);
    for (int ch = 0; ch < nchunks; ++ch) {
        stage();
        __syncthreads();
        if (ch + 1 < nchunks) fetch((ch + 1) * CB);
#pragma unroll
        for (int cc = 0; cc < CB / 2; ++cc)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    const float a = wl[a_base + cc * RS + r * S + s];
                    float b[NT];
#pragma unroll
                    for (int j = 0; j < NT; ++j) b[j] = xl[b_base[j] + cc * G::PLANE + r * G::WLD + s];
#pragma unroll
                    for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[j], acc[j], 0, 0, 0);
                }
        __syncthreads();
    }

    // ---- epilogue: lane = pixel (coalesced along the row), register v = output feature
    const size_t out_plane = (size_t)HO * G::WO;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = (wn * NT + j) * 32 + l32;
        if (i >= G::NPIX) continue;
        const int nb = i / (G::TH * G::WO), rem = i % (G::TH * G::WO);
        const int p = p0 + rem / G::WO, q = rem % G::WO;
        if (n0 + nb >= N || p >= HO) continue;
        float* o = out + ((size_t)(n0 + nb) * M) * out_plane + (size_t)p * G::WO + q;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (m < M) o[(size_t)m * out_plane] = acc[j][v];
        }
    }
}

// wT[c][k][r][s] = w[k][c][R-1-r][S-1-s]: the "transpose-weights" of Section 2.3 with the taps mirrored, so that
// backpropagation is a forward convolution of dy with wT.  One workgroup moves a 32(k) x 32(c) block through LDS;
// both the reads (32*RS contiguous floats per k) and the writes (32*RS per c) are coalesced.
__global__ void __launch_bounds__(256) k_transpose_flip(int K, int C, int RS, const float* __restrict__ w,
                                                       float* __restrict__ wT) {
    extern __shared__ float tl[];               // [32 k][32*RS + 1]
    const int k0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const int row = 32 * RS, str = row + 1;
    const int cn = min(32, C - c0), kn = min(32, K - k0);
    for (int e = threadIdx.x; e < 32 * row; e += 256) {
        const int k = e / row, o = e % row;
        if (k < kn && o < cn * RS) tl[k * str + o] = w[((size_t)(k0 + k) * C + c0) * RS + o];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 32 * row; e += 256) {
        const int c = e / row, o = e % row, k = o / RS, t = o % RS;
        if (c < cn && k < kn) wT[((size_t)(c0 + c) * K + k0) * RS + o] = tl[k * str + c * RS + (RS - 1 - t)];
    }
}

template <class G>
int launch(cnn_ctx* ctx, int N, int J, int M, int HI, int HO, const float* in, const float* wt, float* out) {
    static bool attr_done = false;
    if (!attr_done && G::LDS_BYTES > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_conv_s1<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (e != hipSuccess) return cnn::hip_check(ctx, e, "hipFuncSetAttribute(conv_s1)");
        attr_done = true;
    }
    const int row_tiles = (HO + G::TH - 1) / G::TH;
    const int img_tiles = (N + G::NB - 1) / G::NB;
    dim3 grid((unsigned)(row_tiles * img_tiles), (unsigned)((M + G::MB - 1) / G::MB));
    static char name[96] = "";
    if (!name[0])
        snprintf(name, sizeof(name), "k_conv_s1<%dx%d pad%d CB%d WM%d WN%d NT%d NB%d TH%d W%d>", G::R, G::S, G::PADE, G::CB,
                 G::WM, G::WN, G::NT, G::NB, G::TH, G::WI);
    {
        cnn::ProfScope ps(ctx, name, 2.0 * N * J * M * G::RS * HO * G::WO);
        hipLaunchKernelGGL(k_conv_s1<G>, grid, dim3(G::T), G::LDS_BYTES, ctx->stream, N, J, M, HI, HO, row_tiles, in, wt, out);
    }
    return cnn::launch_check(ctx, "conv_s1");
}

// Geometry table: (R, S, effective pad, CB, WM, WN, NT, NB, TH, WI).  Every entry needs
//   J % CB == 0, (J*R*S) % 4 == 0, HO == HI + 2*PADE - R + 1.
// probe != 0: only report whether the shape is covered (CNN_OK) without launching anything.
int dispatch(cnn_ctx* ctx, int probe, int R, int S, int pade, int N, int J, int M, int HI, int WI, const float* in,
             const float* wt, float* out) {
    const int HO = HI + 2 * pade - R + 1;
    if (HO <= 0) return CNN_EUNSUPPORTED;
    if ((J * R * S) % 4 != 0) return CNN_EUNSUPPORTED;
#define TRY(R_, S_, P_, CB_, WM_, WN_, NT_, NB_, TH_, WI_)                                                  \
    if (R == R_ && S == S_ && pade == P_ && WI == WI_ && J % CB_ == 0)                                       \
        return probe ? CNN_OK                                                                                \
                     : launch<ConvCfg<R_, S_, P_, CB_, WM_, WN_, NT_, NB_, TH_, WI_>>(ctx, N, J, M, HI, HO, in, wt, out);
    if (M <= 64) {
        TRY(3, 3, 1, 8, 2, 2, 7, 1, 4, 112)
        TRY(3, 3, 1, 8, 2, 2, 7, 1, 8, 56)
    }
    TRY(3, 3, 1, 8, 4, 1, 7, 1, 2, 112)
    TRY(3, 3, 1, 8, 4, 1, 7, 1, 4, 56)
    TRY(3, 3, 1, 8, 4, 1, 7, 2, 4, 28)
    TRY(3, 3, 1, 8, 4, 1, 7, 1, 14, 14)
    TRY(3, 3, 1, 4, 4, 1, 9, 2, 12, 12)
    TRY(5, 5, 0, 4, 2, 2, 3, 1, 8, 28)      // 28x28 -> 24x24 forward
    TRY(5, 5, 4, 4, 2, 2, 7, 2, 8, 24)      // 24x24 -> 28x28: backpropagation of the above
#undef TRY
    return CNN_EUNSUPPORTED;
}

}  // namespace

namespace cnn {

int mfma_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* y) {
    if (s.stride != 1 || s.H != s.W) return CNN_EUNSUPPORTED;
    return dispatch(ctx, 0, s.R, s.S, s.pad, s.N, s.C, s.K, s.H, s.W, x, w, y);
}

size_t mfma_conv_bwd_data_ws(const ConvShape& s) {
    if (s.stride != 1 || s.H != s.W || s.R != s.S || s.R - 1 - s.pad < 0) return 0;
    if (dispatch(nullptr, 1, s.R, s.S, s.R - 1 - s.pad, s.N, s.K, s.C, s.P, s.Q, nullptr, nullptr, nullptr) != CNN_OK) return 0;
    return (size_t)s.K * s.C * s.R * s.S * sizeof(float);
}

// dx = forward convolution of dy (P x Q, K channels) with the mirrored transpose-weights, pad' = R-1-pad.
int mfma_conv_bwd_data(cnn_ctx* ctx, const ConvShape& s, const float* dy, const float* w, float* dx) {
    if (s.stride != 1 || s.H != s.W || s.R != s.S || s.R - 1 - s.pad < 0) return CNN_EUNSUPPORTED;
    if (s.P + 2 * (s.R - 1 - s.pad) - s.R + 1 != s.H) return CNN_EUNSUPPORTED;
    // probe the table before touching the workspace: an unsupported shape must fall through untouched
    if (dispatch(ctx, 1, s.R, s.S, s.R - 1 - s.pad, s.N, s.K, s.C, s.P, s.Q, dy, w, dx) != CNN_OK) return CNN_EUNSUPPORTED;
    if (!ctx->ws || ctx->ws_bytes < mfma_conv_bwd_data_ws(s)) return CNN_EWORKSPACE;
    float* wT = reinterpret_cast<float*>(ctx->ws);
    const int RS = s.R * s.S;
    dim3 grid((unsigned)((s.K + 31) / 32), (unsigned)((s.C + 31) / 32));
    const size_t tl_bytes = (32 * (32 * RS + 1)) * sizeof(float);
    static size_t tl_attr = 48 * 1024;
    if (tl_bytes > tl_attr) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_transpose_flip),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)tl_bytes);
        if (e != hipSuccess) return hip_check(ctx, e, "hipFuncSetAttribute(transpose_flip)");
        tl_attr = tl_bytes;
    }
    {
        ProfScope ps(ctx, "k_transpose_flip", 0.0);
        hipLaunchKernelGGL(k_transpose_flip, grid, dim3(256), tl_bytes, ctx->stream, s.K, s.C, RS, w, wT);
    }
    int st = launch_check(ctx, "transpose_flip");
    if (st != CNN_OK) return st;
    return dispatch(ctx, 0, s.R, s.S, s.R - 1 - s.pad, s.N, s.K, s.C, s.P, s.Q, dy, wT, dx);
}

}  // namespace cnn
