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
// Two LDS buffers: while chunk ch is multiplied, chunk ch+1 moves from registers into the other buffer and chunk
// ch+2 from HBM into those registers, one staging item between every MFMA step (no staging phase, one barrier per
// chunk).  LDS row / image strides are padded so that consecutive pixels stay in consecutive banks across row ends.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

// epilogues: plain store; ReLU of the result; result where aux > 0 else 0 (ReLU derivative, aux = the ReLU's output)
enum { EPI_NONE = 0, EPI_RELU = 1, EPI_MASK = 2 };

// VEC = 4: filter rows are fetched as float4 (needs J % CB == 0 and 16-byte aligned rows); VEC = 1: element-wise
// fetch with the channels past J zero-filled (first layers: J = 3).
template <int R_, int S_, int PADE_, int CB_, int WM_, int WN_, int NT_, int NB_, int TH_, int WI_, int VEC_ = 4>
struct ConvCfg {
    static constexpr int R = R_, S = S_, PADE = PADE_, CB = CB_, WM = WM_, WN = WN_, NT = NT_, NB = NB_, TH = TH_, WI = WI_;
    static constexpr int VEC = VEC_;
    static constexpr int RS = R * S;
    static constexpr int WO = WI + 2 * PADE - S + 1;
    static constexpr int THI = TH + R - 1;
    static constexpr int WLD = WI + 2 * PADE;
    static constexpr int PLANE = NB * THI * WLD;            // staged elements per channel
    // LDS strides.  Consecutive output pixels must fall into consecutive banks also across the end of a row and of
    // an image, or every operand read that spans two rows pays a bank conflict: row stride = WO (mod 32), image
    // stride = TH*WO (mod 32).
    static constexpr int WLDP = WO + 32 * ((WLD - WO + 31) / 32);
    static constexpr int IMG0 = THI * WLDP;
    static constexpr int IMGSTR = IMG0 + ((((TH - 1) * WLDP + WO - IMG0) % 32) + 32) % 32;
    static constexpr int PLANEP = NB * IMGSTR;               // LDS elements per channel
    static constexpr int MB = 32 * WM;
    static constexpr int NPIX = NB * TH * WO;
    static constexpr int NPIXB = WN * NT * 32;              // padded to whole MFMA column blocks
    static constexpr int T = WM * WN * 64;
    static constexpr int KCH = CB * RS;                      // contraction length of one chunk
    static constexpr int WSTR = (KCH % 2 == 0) ? KCH + 1 : KCH;
    static constexpr int XTOT = CB * PLANEP;
    static constexpr int XP = (PLANE + T - 1) / T;           // input-tile positions per thread (per channel)
    static constexpr int Q4 = KCH / VEC;                     // fetch units (float4 or float) per filter row
    static constexpr int RPP = T / Q4;                       // filter rows fetched per pass of the workgroup
    static constexpr int WSL = (MB + RPP - 1) / RPP;         // passes
    static constexpr int LDS_BUF = MB * WSTR + XTOT;         // elements of one (filter tile, input tile) buffer
    static constexpr int LDS_BYTES = LDS_BUF * 4 * 2;
    static_assert(CB % 2 == 0, "the two wave halves split the chunk's channels");
    static_assert(KCH % VEC == 0 && (VEC == 1 || VEC == 4), "filter tile is fetched as float4 or float");
    static_assert(NPIXB >= NPIX && NPIXB - NPIX < 32 * WN, "pixel tile padded by less than one block per wave column");
};

template <class G>
__global__ void __launch_bounds__(G::T, 2)
k_conv_s1(int N, int J, int M, int HI, int HO, int row_tiles, int chunks_per_split, int epi,
          const float* __restrict__ in, const float* __restrict__ wt, const float* __restrict__ aux,
          float* __restrict__ out_base) {
    constexpr int R = G::R, S = G::S, RS = G::RS, CB = G::CB, NT = G::NT, T = G::T;
    extern __shared__ float lds[];
    float* wl = lds;
    float* xl = lds + G::MB * G::WSTR;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm = wave % G::WM, wn = wave / G::WM;

    // Workgroups are handed to the 8 XCDs round-robin by linear id.  Give each XCD (its own L2) a contiguous range
    // of pixel tiles and run the output-feature tiles of one pixel tile back to back on it, so the input tile, and
    // the halo rows it shares with the next tile, come from HBM once instead of once per feature tile.
    const int ptiles = row_tiles * ((N + G::NB - 1) / G::NB), mtiles = (M + G::MB - 1) / G::MB;
    const int per_xcd = (ptiles + 7) / 8;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int ptile = xcd * per_xcd + seq / mtiles;
    if (seq / mtiles >= per_xcd || ptile >= ptiles) return;      // whole workgroup leaves: no barrier is left behind
    const int m0 = (seq % mtiles) * G::MB;
    const int n0 = (ptile / row_tiles) * G::NB;
    const int p0 = (ptile % row_tiles) * G::TH;

    const size_t in_img = (size_t)J * HI * G::WI;      // elements per image of `in`
    const float* in_base = in + (size_t)n0 * in_img;
    const int plane_g = HI * G::WI;

    // ---- input tile staging: each thread owns XP positions of the (image, row, col) plane and fetches
    //      them for every channel of the chunk (-1 = outside the image: zero fill)
    int xoff[G::XP], xpos[G::XP];
#pragma unroll
    for (int j = 0; j < G::XP; ++j) {
        const int e = tid + j * T;
        int off = -1, pos = 0;
        if (e < G::PLANE) {
            const int nb = e / (G::THI * G::WLD), rem = e % (G::THI * G::WLD);
            const int row = rem / G::WLD, col = rem % G::WLD;
            const int h = p0 - G::PADE + row, w = col - G::PADE;
            pos = nb * G::IMGSTR + row * G::WLDP + col;
            if (n0 + nb < N && h >= 0 && h < HI && w >= 0 && w < G::WI) off = nb * (int)in_img + h * G::WI + w;
        }
        xoff[j] = off;
        xpos[j] = pos;
    }
    // ---- filter tile staging: thread = (row m_sub, float4 kq) of a pass over RPP rows
    const int w_msub = tid / G::Q4, w_kq = tid % G::Q4;
    const bool w_thread = tid < G::RPP * G::Q4;
    const float* w_src = wt + ((size_t)(m0 + w_msub) * J) * RS + w_kq * G::VEC;
    float* w_dst = wl + w_msub * G::WSTR + w_kq * G::VEC;

    // ---- per-lane LDS read bases
    const int a_base = (wm * 32 + l32) * G::WSTR + half * (CB / 2) * RS;
    int b_base[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = (wn * NT + j) * 32 + l32;
        int o = 0;
        if (i < G::NPIX) {
            const int nb = i / (G::TH * G::WO), rem = i % (G::TH * G::WO);
            o = nb * G::IMGSTR + (rem / G::WO) * G::WLDP + rem % G::WO;
        }
        b_base[j] = o + half * (CB / 2) * G::PLANEP;
    }

    f32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    float xr[CB][G::XP];
    float4 wr[G::WSL];

    // Staging is cut into items (one input-tile register or one filter-tile float4 each) so that it can be spread
    // over the MFMA steps of a chunk instead of forming a phase of its own.
    constexpr int NX = CB * G::XP, NITEMS = NX + G::WSL;
    auto fetch_item = [&](int it, int c0) {
        if (it < NX) {
            const int c = it / G::XP, j = it % G::XP;
            const float* src = in_base + (size_t)c0 * plane_g;
            xr[c][j] = (xoff[j] >= 0 && (G::VEC == 4 || c0 + c < J)) ? src[xoff[j] + c * plane_g] : 0.f;
        } else {
            // w[m][c0 .. c0+CB)[R][S]: CB*R*S contiguous floats per output feature
            const int i = it - NX, m = w_msub + i * G::RPP;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (w_thread && m < G::MB && m0 + m < M) {
                if (G::VEC == 4) v = *reinterpret_cast<const float4*>(w_src + ((size_t)i * G::RPP * J + c0) * RS);
                else if (c0 * RS + w_kq < J * RS) v.x = w_src[((size_t)i * G::RPP * J + c0) * RS];
            }
            wr[i] = v;
        }
    };
    auto stage_item = [&](int it, int buf) {
        if (it < NX) {
            const int c = it / G::XP, j = it % G::XP;
            if (tid + j * T < G::PLANE) xl[buf * G::LDS_BUF + c * G::PLANEP + xpos[j]] = xr[c][j];
        } else {
            const int i = it - NX;
            if (w_thread && w_msub + i * G::RPP < G::MB) {
                float* d = w_dst + buf * G::LDS_BUF + i * G::RPP * G::WSTR;
                d[0] = wr[i].x;
                if (G::VEC == 4) { d[1] = wr[i].y; d[2] = wr[i].z; d[3] = wr[i].w; }
            }
        }
    };

    // Two LDS buffers.  While chunk ch is multiplied out of buffer ch&1, chunk ch+1 goes from registers into the
    // other buffer and chunk ch+2 from HBM into those registers, item by item between the MFMA steps, so neither
    // the LDS writes nor the global-load issue ever stall the matrix pipe for a whole phase.  One barrier per chunk.
    // The last iterations stage and fetch a clamped chunk again instead of branching (harmless: that buffer is
    // never read), which keeps the chunk body one basic block.
    // blockIdx.z selects a slice of the contraction (used when the output alone gives too few workgroups);
    // each slice writes its own partial output, added up afterwards in slice order.
    const int ch_begin = blockIdx.z * chunks_per_split;
    const int ch_end = min(ch_begin + chunks_per_split, (J + CB - 1) / CB);
    float* out = out_base + (size_t)blockIdx.z * N * M * HO * G::WO;
    constexpr int STEPS = (CB / 2) * RS, IPS = (NITEMS + STEPS - 1) / STEPS;
#pragma unroll
    for (int it = 0; it < NITEMS; ++it) fetch_item(it, ch_begin * CB);
#pragma unroll
    for (int it = 0; it < NITEMS; ++it) stage_item(it, 0);
    {
        const int c1 = min(ch_begin + 1, ch_end - 1) * CB;
#pragma unroll
        for (int it = 0; it < NITEMS; ++it) fetch_item(it, c1);
    }
    __syncthreads();
    for (int ch = ch_begin; ch < ch_end; ++ch) {
        const int buf = (ch - ch_begin) & 1;
        const int c2 = min(ch + 2, ch_end - 1) * CB;
        const float* wb = wl + buf * G::LDS_BUF;
        const float* xb = xl + buf * G::LDS_BUF;
#pragma unroll
        for (int cc = 0; cc < CB / 2; ++cc)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    const int step = (cc * R + r) * S + s;
#pragma unroll
                    for (int u = 0; u < IPS; ++u) {
                        const int it = step * IPS + u;
                        if (it < NITEMS) {
                            stage_item(it, buf ^ 1);
                            fetch_item(it, c2);
                        }
                    }
                    const float a = wb[a_base + cc * RS + r * S + s];
                    float b[NT];
#pragma unroll
                    for (int j = 0; j < NT; ++j) b[j] = xb[b_base[j] + cc * G::PLANEP + r * G::WLDP + s];
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
        const size_t o0 = ((size_t)(n0 + nb) * M) * out_plane + (size_t)p * G::WO + q;
        float* o = out + o0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (m < M) {
                float r = acc[j][v];
                if (epi == EPI_RELU) r = r > 0.f ? r : 0.f;                                   // fused ReLU
                else if (epi == EPI_MASK) r = aux[o0 + (size_t)m * out_plane] > 0.f ? r : 0.f;   // fused ReLU derivative
                o[(size_t)m * out_plane] = r;
            }
        }
    }
}

// wT[c][k][r][s] = w[k][c][R-1-r][S-1-s]: the "transpose-weights" of Section 2.3 with the taps mirrored, so that
// backpropagation is a forward convolution of dy with wT.  One workgroup moves an 8(k) x 32(c) block through LDS;
// the reads (32*RS contiguous floats per k) are coalesced, the writes are runs of 8*RS floats per c.
constexpr int kTfK = 8;
__global__ void __launch_bounds__(256) k_transpose_flip(int K, int C, int RS, const float* __restrict__ w,
                                                       float* __restrict__ wT) {
    extern __shared__ float tl[];               // [kTfK][32*RS + 1]
    const int k0 = blockIdx.x * kTfK, c0 = blockIdx.y * 32;
    const int row = 32 * RS, str = row + 1;
    const int cn = min(32, C - c0), kn = min(kTfK, K - k0);
    for (int e = threadIdx.x; e < kTfK * row; e += 256) {
        const int k = e / row, o = e % row;
        if (k < kn && o < cn * RS) tl[k * str + o] = w[((size_t)(k0 + k) * C + c0) * RS + o];
    }
    __syncthreads();
    const int orow = kTfK * RS;
    for (int e = threadIdx.x; e < 32 * orow; e += 256) {
        const int c = e / orow, o = e % orow, k = o / RS, t = o % RS;
        if (c < cn && k < kn) wT[((size_t)(c0 + c) * K + k0) * RS + o] = tl[k * str + c * RS + (RS - 1 - t)];
    }
}

// out[i] = sum over slices of partial[slice][i], in slice order.
__global__ void __launch_bounds__(256) k_slice_reduce(int nslice, size_t n, int epi, const float* __restrict__ partial,
                                                     const float* __restrict__ aux, float* __restrict__ out) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        float s0 = 0.f, s1 = 0.f;
        int s = 0;
        for (; s + 1 < nslice; s += 2) {
            s0 += partial[(size_t)s * n + i];
            s1 += partial[(size_t)(s + 1) * n + i];
        }
        if (s < nslice) s0 += partial[(size_t)s * n + i];
        float r = s0 + s1;
        if (epi == EPI_RELU) r = r > 0.f ? r : 0.f;
        else if (epi == EPI_MASK) r = aux[i] > 0.f ? r : 0.f;
        out[i] = r;
    }
}

struct LaunchArgs {
    int N, J, M, HI, HO, nsplit, chunks_per_split, epi;
    const float *in, *wt, *aux;
    float* out;       // final output, or the partial buffer when nsplit > 1
};
typedef int (*LaunchFn)(cnn_ctx*, const LaunchArgs&);

template <class G>
int launch(cnn_ctx* ctx, const LaunchArgs& a) {
    static bool attr_done = false;
    if (!attr_done && G::LDS_BYTES > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_conv_s1<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (e != hipSuccess) return cnn::hip_check(ctx, e, "hipFuncSetAttribute(conv_s1)");
        attr_done = true;
    }
    const int row_tiles = (a.HO + G::TH - 1) / G::TH;
    const int img_tiles = (a.N + G::NB - 1) / G::NB;
    dim3 grid((unsigned)(8 * ((row_tiles * img_tiles + 7) / 8) * ((a.M + G::MB - 1) / G::MB)), 1, (unsigned)a.nsplit);
    static char name[96] = "";
    if (!name[0])
        snprintf(name, sizeof(name), "k_conv_s1<%dx%d pad%d CB%d WM%d WN%d NT%d NB%d TH%d W%d%s>", G::R, G::S, G::PADE, G::CB,
                 G::WM, G::WN, G::NT, G::NB, G::TH, G::WI, G::VEC == 1 ? " v1" : "");
    {
        cnn::ProfScope ps(ctx, name, 2.0 * a.N * a.J * a.M * G::RS * a.HO * G::WO);
        hipLaunchKernelGGL(k_conv_s1<G>, grid, dim3(G::T), G::LDS_BYTES, ctx->stream, a.N, a.J, a.M, a.HI, a.HO, row_tiles,
                           a.chunks_per_split, a.epi, a.in, a.wt, a.aux, a.out);
    }
    return cnn::launch_check(ctx, "conv_s1");
}

// One table row per input geometry the tiled kernel is instantiated for.  Each row has a 128-feature tile
// (4 waves) and a 64-feature tile (2 waves, same pixel tile); `big`/`small` may be null.
struct Geo {
    int R, S, pade, WI, CB, NB, TH, vec;
    int mb_big;
    LaunchFn big;
    int mb_small;
    LaunchFn small;
};
#define CFG(R_, S_, P_, CB_, WM_, WN_, NT_, NB_, TH_, WI_, V_) launch<ConvCfg<R_, S_, P_, CB_, WM_, WN_, NT_, NB_, TH_, WI_, V_>>
const Geo kGeo[] = {
    // first layer: three input feature maps, element-wise filter fetch
    {3, 3, 1, 224, 4, 1, 2, 1, 0, nullptr, 64, CFG(3, 3, 1, 4, 2, 2, 7, 1, 2, 224, 1)},
    {3, 3, 1, 112, 4, 1, 2, 4, 128, CFG(3, 3, 1, 4, 4, 1, 7, 1, 2, 112, 4), 64, CFG(3, 3, 1, 4, 2, 1, 7, 1, 2, 112, 4)},
    {3, 3, 1, 56, 4, 1, 4, 4, 128, CFG(3, 3, 1, 4, 4, 1, 7, 1, 4, 56, 4), 64, CFG(3, 3, 1, 4, 2, 1, 7, 1, 4, 56, 4)},
    {3, 3, 1, 28, 4, 2, 4, 4, 128, CFG(3, 3, 1, 4, 4, 1, 7, 2, 4, 28, 4), 64, CFG(3, 3, 1, 4, 2, 1, 7, 2, 4, 28, 4)},
    {3, 3, 1, 14, 4, 1, 14, 4, 128, CFG(3, 3, 1, 4, 4, 1, 7, 1, 14, 14, 4), 64, CFG(3, 3, 1, 4, 2, 1, 7, 1, 14, 14, 4)},
    {3, 3, 1, 12, 4, 2, 12, 4, 128, CFG(3, 3, 1, 4, 4, 1, 9, 2, 12, 12, 4), 64, CFG(3, 3, 1, 4, 2, 1, 9, 2, 12, 12, 4)},
    {5, 5, 0, 28, 4, 1, 8, 4, 0, nullptr, 64, CFG(5, 5, 0, 4, 2, 2, 3, 1, 8, 28, 4)},     // 28x28 -> 24x24 forward
    {5, 5, 4, 24, 4, 2, 8, 4, 0, nullptr, 64, CFG(5, 5, 4, 4, 2, 2, 7, 2, 8, 24, 4)},     // its backpropagation
};
#undef CFG

struct ConvPlan {
    const Geo* g;
    bool use_small;
    int nsplit, chunks_per_split;
    size_t partial_bytes;
};

// Picks the tile height (128 output features, or 64 for narrow layers) and slices the contraction when the output
// alone gives fewer workgroups than the chip runs at once.
bool make_plan(int R, int S, int pade, int N, int J, int M, int HI, int WI, ConvPlan* p) {
    const int HO = HI + 2 * pade - R + 1;
    if (HO <= 0) return false;
    for (const Geo& g : kGeo) {
        if (g.R != R || g.S != S || g.pade != pade || g.WI != WI) continue;
        if (g.vec == 4 ? (J % g.CB != 0 || (J * R * S) % 4 != 0) : J >= 4) continue;
        const long ptiles = (long)((N + g.NB - 1) / g.NB) * ((HO + g.TH - 1) / g.TH);
        const int kCU = 256;
        p->g = &g;
        // the 64-feature tile re-stages the same input tile for half the MFMA work (measured ~30 % slower per
        // FLOP), so it is used only when the layer has no more than 64 output features
        p->use_small = !g.big || (g.small && M <= g.mb_small);
        const int mb = p->use_small ? g.mb_small : g.mb_big;
        const long wgs = ptiles * ((M + mb - 1) / mb);
        const long concurrent = (long)kCU * 8 / ((p->use_small && g.big) ? 2 : 4);   // 8 waves per compute unit
        const int nchunks = (J + g.CB - 1) / g.CB;
        int want = 1;
        if (wgs < concurrent) want = (int)((concurrent + wgs - 1) / wgs);
        int max_split = nchunks / 8;                     // at least 8 chunks per slice
        if (max_split < 1) max_split = 1;
        if (want > max_split) want = max_split;
        p->chunks_per_split = (nchunks + want - 1) / want;
        p->nsplit = (nchunks + p->chunks_per_split - 1) / p->chunks_per_split;
        const int WO = WI + 2 * pade - S + 1;
        p->partial_bytes = p->nsplit > 1 ? (size_t)p->nsplit * N * M * HO * WO * sizeof(float) : 0;
        return true;
    }
    return false;
}

// ws: scratch for the partial outputs (only touched when the plan slices the contraction)
int run_plan(cnn_ctx* ctx, const ConvPlan& p, int N, int J, int M, int HI, int HO, int WO, const float* in, const float* wt,
             float* out, float* ws, int epi, const float* aux) {
    // with a sliced contraction the epilogue belongs to the kernel that adds the slices
    LaunchArgs a{N, J, M, HI, HO, p.nsplit, p.chunks_per_split, p.nsplit > 1 ? EPI_NONE : epi, in, wt, aux,
                 p.nsplit > 1 ? ws : out};
    int st = (p.use_small ? p.g->small : p.g->big)(ctx, a);
    if (st != CNN_OK || p.nsplit == 1) return st;
    const size_t n = (size_t)N * M * HO * WO;
    size_t g = (n + 255) / 256;
    if (g > 8192) g = 8192;
    {
        cnn::ProfScope ps(ctx, "k_slice_reduce", 0.0);
        hipLaunchKernelGGL(k_slice_reduce, dim3((unsigned)g), dim3(256), 0, ctx->stream, p.nsplit, n, epi, ws, aux, out);
    }
    return cnn::launch_check(ctx, "slice_reduce");
}

}  // namespace

namespace cnn {

size_t mfma_conv_fwd_ws(const ConvShape& s) {
    ConvPlan p;
    if (s.stride != 1 || s.H != s.W || !make_plan(s.R, s.S, s.pad, s.N, s.C, s.K, s.H, s.W, &p)) return 0;
    return p.partial_bytes;
}

int mfma_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* y, int relu) {
    ConvPlan p;
    if (s.stride != 1 || s.H != s.W || !make_plan(s.R, s.S, s.pad, s.N, s.C, s.K, s.H, s.W, &p)) return CNN_EUNSUPPORTED;
    if (p.partial_bytes && (!ctx->ws || ctx->ws_bytes < p.partial_bytes)) return CNN_EWORKSPACE;
    return run_plan(ctx, p, s.N, s.C, s.K, s.H, s.P, s.Q, x, w, y, reinterpret_cast<float*>(ctx->ws),
                    relu ? EPI_RELU : EPI_NONE, nullptr);
}

static bool bwd_plan(const ConvShape& s, ConvPlan* p) {
    if (s.stride != 1 || s.H != s.W || s.R != s.S || s.R - 1 - s.pad < 0) return false;
    if (s.P + 2 * (s.R - 1 - s.pad) - s.R + 1 != s.H) return false;
    return make_plan(s.R, s.S, s.R - 1 - s.pad, s.N, s.K, s.C, s.P, s.Q, p);
}

static size_t wt_bytes(const ConvShape& s) {   // mirrored transpose of the weights, rounded up to 256 bytes
    return ((size_t)s.K * s.C * s.R * s.S * sizeof(float) + 255) / 256 * 256;
}

size_t mfma_conv_bwd_data_ws(const ConvShape& s) {
    ConvPlan p;
    if (!bwd_plan(s, &p)) return 0;
    return wt_bytes(s) + p.partial_bytes;
}

// dx = forward convolution of dy (P x Q, K channels) with the mirrored transpose-weights, pad' = R-1-pad.
// act != NULL: dx is zeroed where act <= 0 (act = the ReLU output that was this layer's forward input).
int mfma_conv_bwd_data(cnn_ctx* ctx, const ConvShape& s, const float* dy, const float* w, float* dx, const float* act) {
    ConvPlan p;
    if (!bwd_plan(s, &p)) return CNN_EUNSUPPORTED;      // decided before the workspace is touched
    if (!ctx->ws || ctx->ws_bytes < wt_bytes(s) + p.partial_bytes) return CNN_EWORKSPACE;
    float* wT = reinterpret_cast<float*>(ctx->ws);
    float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(ctx->ws) + wt_bytes(s));
    const int RS = s.R * s.S;
    dim3 grid((unsigned)((s.K + kTfK - 1) / kTfK), (unsigned)((s.C + 31) / 32));
    const size_t tl_bytes = (kTfK * (32 * RS + 1)) * sizeof(float);
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
    return run_plan(ctx, p, s.N, s.K, s.C, s.P, s.H, s.W, dy, wT, dx, partial, act ? EPI_MASK : EPI_NONE, act);
}

}  // namespace cnn
