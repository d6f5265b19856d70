// Weight gradient of a stride-1 convolution (Section 2.1, "Weight-gradient Update") on the fp32
// matrix cores:  dw[k][c][r][s] = sum_{n,p,q} dy[n][k][p][q] * x[n][c][p+r-pad][q+s-pad].
//
// The output is tiny and the contraction (all pixels of the per-GPU minibatch) is huge, so, as the paper
// does for its C1-type layers (Section 2.5), the contraction is split across workgroups, each keeps a
// private partial sum, and a second kernel adds the partials in a fixed order (bitwise repeatable).
//
// One workgroup owns KB = 32*KW output features x CBK = 32*CW input features x all R*S taps and walks a
// range of output rows.  Per tap one accumulator D[k][c] (16 VGPRs per wave): A = dy (lane = output
// feature), B = x shifted by the tap (lane = input feature), the MFMA's k index = pixel.
// The walk goes along the image height, so each step brings in ONE new input row and one dy row while
// the R-1 rows above stay in an LDS ring (the row-reuse of Section 2.2's traversal argument):
//   LDS xl[CBK][NBI][NSLOT][TW+2*pad]   ring of input rows (halo columns kept at zero)
//   LDS dyl[2][KB][NBI*TW]              double-buffered dy row
// Row strides are odd so the 32 lanes of an operand (32 features) read 32 different banks.
// Narrow images are processed NBI at a time (one ring each) to keep >= 48 pixels per step.
// Wide rows are cut into column tiles of TW; each column tile is one more split.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int R_, int S_, int PAD_, int TW_, int NBI_, int KW_, int CW_, int RW_, int NSLOT_>
struct WgCfg {
    static constexpr int R = R_, S = S_, PAD = PAD_, TW = TW_, NBI = NBI_, KW = KW_, CW = CW_, RW = RW_, NSLOT = NSLOT_;
    static constexpr int RS = R * S, RPW = R / RW;
    static constexpr int WLD = TW + S - 1;                 // input columns feeding TW output columns
    static constexpr int KB = 32 * KW, CBK = 32 * CW;
    static constexpr int T = 64 * KW * CW * RW;
    static constexpr int XROW = NBI * NSLOT * WLD;
    static constexpr int XSTR = (XROW % 2 == 0) ? XROW + 1 : XROW;
    static constexpr int DROW = NBI * TW;
    static constexpr int DSTR = (DROW % 2 == 0) ? DROW + 1 : DROW;
    static constexpr int XL = CBK * XSTR, DL = 2 * KB * DSTR;
    static constexpr int LDS_BYTES = (XL + DL) * 4;
    static constexpr int NWAVE = T / 64;
    static constexpr int XS = (CBK + NWAVE - 1) / NWAVE, DS = (KB + NWAVE - 1) / NWAVE;   // rows staged per wave per step
    static_assert(NBI * WLD <= 64 && NBI * TW <= 64, "one wave instruction fetches one feature's row(s)");
    // pixel pairs of one step: the low wave half takes pixel i, the high half pixel i + HALF_DELTA
    static constexpr int NLOW = NBI * TW / 2;
    static_assert(R % RW == 0 && NSLOT >= R + 1 && (NSLOT & (NSLOT - 1)) == 0, "ring geometry");
    static_assert(NBI == 1 ? TW % 2 == 0 : NBI % 2 == 0, "the wave halves split the step's pixels evenly");
};

template <class G>
__global__ void __launch_bounds__(G::T)
k_wgrad(int N, int C, int K, int HI, int WI, int HO, int WO, int rows_per_split, int total_rows,
        const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ partial) {
    constexpr int R = G::R, S = G::S, PAD = G::PAD, TW = G::TW, NBI = G::NBI, NSLOT = G::NSLOT, T = G::T, WLD = G::WLD;
    extern __shared__ float lds[];
    float* xl = lds;
    float* dyl = lds + G::XL;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int kw = wave % G::KW, cw = (wave / G::KW) % G::CW, rw = wave / (G::KW * G::CW);

    const int col_tiles = WO / TW;
    const int split = blockIdx.x / col_tiles, q0 = (blockIdx.x % col_tiles) * TW;
    const int c0 = blockIdx.y * G::CBK, k0 = blockIdx.z * G::KB;

    // output rows are numbered g = group*HO + p over image groups of NBI images
    const int g_begin = split * rows_per_split;
    const int g_end = min(g_begin + rows_per_split, total_rows);
    const int V = HO + R - 1;                         // input rows of one image incl. the zero rows above/below

    // zero the whole ring once: halo columns stay zero for the life of the kernel
    for (int e = tid; e < G::XL; e += T) xl[e] = 0.f;

    // staging: wave w fetches feature rows w, w+NWAVE, ...; lane = position in the row(s) of the NBI images
    int xo = -1, xlds = 0;
    {
        const int b = lane / WLD, col = lane % WLD, w = q0 - PAD + col;
        if (lane < NBI * WLD) {
            xlds = wave * G::XSTR + b * NSLOT * WLD + col;
            if (w >= 0 && w < WI) xo = (b * C + c0 + wave) * HI * WI + w;
        }
    }
    const int xb = lane / WLD;
    int dyo = -1, dlds = 0;
    {
        const int b = lane / TW, q = lane % TW;
        if (lane < NBI * TW) {
            dlds = wave * G::DSTR + b * TW + q;
            dyo = (b * K + k0 + wave) * HO * WO + q0 + q;
        }
    }
    const int db = lane / TW;

    f32x16 acc[G::RPW][S];
#pragma unroll
    for (int r = 0; r < G::RPW; ++r)
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][s][v] = 0.f;

    // LDS read bases.  pixel i of the step: image b = i / TW, column q = i % TW
    constexpr int A_DELTA = G::NLOW;                                           // in dyl: pixels are contiguous
    constexpr int B_DELTA = NBI == 1 ? TW / 2 : (NBI / 2) * NSLOT * WLD;       // in xl
    const int a_base = (kw * 32 + l32) * G::DSTR + half * A_DELTA;
    const int b_base = (cw * 32 + l32) * G::XSTR + half * B_DELTA;

    float xr[G::XS], dr[G::DS];
    const size_t x_grp = (size_t)NBI * C * HI * WI, dy_grp = (size_t)NBI * K * HO * WO;

    // step u (virtual input row): image group = u / V, row within the zero-extended image = u % V
    auto fetch = [&](int u) {
        const int grp = u / V, vr = u % V;
        const int h = vr - PAD, p = vr - (R - 1);
        const int nleft = N - grp * NBI;                 // images of this group that exist
        const bool hv = h >= 0 && h < HI && xo >= 0 && xb < nleft;
        const float* xs = x + grp * x_grp + (size_t)(h >= 0 && h < HI ? h : 0) * WI;
#pragma unroll
        for (int i = 0; i < G::XS; ++i) {
            const int c = wave + i * G::NWAVE;
            xr[i] = (hv && c < G::CBK && c0 + c < C) ? xs[xo + i * G::NWAVE * HI * WI] : 0.f;
        }
        const int g = grp * HO + p;
        const bool rowv = p >= 0 && g >= g_begin && g < g_end;
        const bool pv = rowv && dyo >= 0 && db < nleft;
        const float* ds = dy + grp * dy_grp + (size_t)(rowv ? p : 0) * WO;
#pragma unroll
        for (int i = 0; i < G::DS; ++i) {
            const int k = wave + i * G::NWAVE;
            dr[i] = (pv && k < G::KB && k0 + k < K) ? ds[dyo + i * G::NWAVE * HO * WO] : 0.f;
        }
    };

    if (g_begin < g_end) {
        const int u_begin = (g_begin / HO) * V + (g_begin % HO);
        const int u_last = ((g_end - 1) / HO) * V + ((g_end - 1) % HO) + R - 1;
        __syncthreads();   // ring zeroed
        fetch(u_begin);
        for (int u = u_begin; u <= u_last; ++u) {
            const int slot = u & (NSLOT - 1), buf = u & 1;
            if (lane < NBI * WLD) {
#pragma unroll
                for (int i = 0; i < G::XS; ++i)
                    if (wave + i * G::NWAVE < G::CBK) xl[xlds + i * G::NWAVE * G::XSTR + slot * WLD] = xr[i];
            }
            if (lane < NBI * TW) {
#pragma unroll
                for (int i = 0; i < G::DS; ++i)
                    if (wave + i * G::NWAVE < G::KB) dyl[buf * G::KB * G::DSTR + dlds + i * G::NWAVE * G::DSTR] = dr[i];
            }
            __syncthreads();
            if (u < u_last) fetch(u + 1);
            const int vr = u % V, p = vr - (R - 1);
            const int g = (u / V) * HO + p;
            if (p >= 0 && g >= g_begin) {     // an output row completes at this step (g < g_end by construction)
                const float* ap = dyl + buf * G::KB * G::DSTR + a_base;
                const float* bp = xl + b_base;
                int so[G::RPW];
#pragma unroll
                for (int r = 0; r < G::RPW; ++r) so[r] = ((u - (R - 1) + rw * G::RPW + r) & (NSLOT - 1)) * WLD;
                if (NBI == 1) {
#pragma unroll 2
                    for (int q = 0; q < TW / 2; ++q) {
                        const float a = ap[q];
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s)
                                acc[r][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bp[so[r] + q + s], acc[r][s], 0, 0, 0);
                    }
                } else {
                    for (int b = 0; b < NBI / 2; ++b) {
#pragma unroll 2
                        for (int q = 0; q < TW; ++q) {
                            const float a = ap[b * TW + q];
#pragma unroll
                            for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                                for (int s = 0; s < S; ++s)
                                    acc[r][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                        a, bp[b * NSLOT * WLD + so[r] + q + s], acc[r][s], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    // partial[blockIdx.x][tap][K][C]: lane = input feature (contiguous), register = output feature
    float* out = partial + (size_t)blockIdx.x * G::RS * K * C;
    const int c = c0 + cw * 32 + l32;
    if (c < C) {
#pragma unroll
        for (int r = 0; r < G::RPW; ++r)
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const int tap = (rw * G::RPW + r) * S + s;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = k0 + kw * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    if (k < K) out[((size_t)tap * K + k) * C + c] = acc[r][s][v];
                }
            }
    }
}

// dw[(k*C + c)*RS + tap] = sum over splits of partial[split][tap][k*C + c], added in split order.
__global__ void __launch_bounds__(256) k_wgrad_reduce(int nsplit, int RS, int KC, const float* __restrict__ partial,
                                                     float* __restrict__ dw) {
    const size_t total = (size_t)RS * KC;
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int tap = (int)(i / KC), kc = (int)(i % KC);
        float s0 = 0.f, s1 = 0.f;
        int s = 0;
        for (; s + 1 < nsplit; s += 2) {
            s0 += partial[(size_t)s * total + i];
            s1 += partial[(size_t)(s + 1) * total + i];
        }
        if (s < nsplit) s0 += partial[(size_t)s * total + i];
        dw[(size_t)kc * RS + tap] = s0 + s1;
    }
}

struct Plan {
    int nsplit, col_tiles, rows_per_split, total_rows, ktiles, ctiles;
    size_t ws_bytes;
};

template <class G>
Plan make_plan(const ConvShape& s) {
    Plan p;
    p.col_tiles = s.Q / G::TW;
    p.ktiles = (s.K + G::KB - 1) / G::KB;
    p.ctiles = (s.C + G::CBK - 1) / G::CBK;
    const int groups = (s.N + G::NBI - 1) / G::NBI;
    p.total_rows = groups * s.P;
    const int tiles = p.ktiles * p.ctiles * p.col_tiles;
    // Choose the number of row splits that minimises the time of the slowest compute unit, counted in steps (one
    // output row each): a split of n rows costs n + R - 1 steps (ring warm-up), the workgroups run 256 at a time
    // (one per compute unit, the LDS ring fills it), and every split adds one private copy of dw to write and read
    // back (a step moves about as many bytes as 70 MB of that traffic takes).
    const double copy_steps = (double)G::RS * s.K * s.C * 8.0 / 70e6;
    double best = 1e30;
    int best_split = 1;
    for (int ns = 1; ns <= p.total_rows; ++ns) {
        const int rps = (p.total_rows + ns - 1) / ns;
        const int real = (p.total_rows + rps - 1) / rps;
        if (real != ns) continue;
        const long rounds = ((long)tiles * ns + 255) / 256;
        const double cost = (double)rounds * (rps + G::R - 1) + copy_steps * ns;
        if (cost < best) { best = cost; best_split = ns; }
        if (rps == 1) break;
    }
    p.nsplit = best_split;
    p.rows_per_split = (p.total_rows + best_split - 1) / best_split;
    p.ws_bytes = (size_t)p.nsplit * p.col_tiles * G::RS * s.K * s.C * sizeof(float);
    return p;
}

template <class G>
int launch(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, float* dw) {
    const Plan p = make_plan<G>(s);
    if (ctx->ws_bytes < p.ws_bytes || !ctx->ws) return CNN_EWORKSPACE;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wgrad<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (e != hipSuccess) return cnn::hip_check(ctx, e, "hipFuncSetAttribute(wgrad)");
        attr_done = true;
    }
    float* partial = reinterpret_cast<float*>(ctx->ws);
    dim3 grid((unsigned)(p.nsplit * p.col_tiles), (unsigned)p.ctiles, (unsigned)p.ktiles);
    static char name[96] = "";
    if (!name[0])
        snprintf(name, sizeof(name), "k_wgrad<%dx%d pad%d TW%d NBI%d KW%d CW%d RW%d>", G::R, G::S, G::PAD, G::TW, G::NBI,
                 G::KW, G::CW, G::RW);
    {
        cnn::ProfScope ps(ctx, name, cnn::conv_flops(s));
        hipLaunchKernelGGL(k_wgrad<G>, grid, dim3(G::T), G::LDS_BYTES, ctx->stream, s.N, s.C, s.K, s.H, s.W, s.P, s.Q,
                           p.rows_per_split, p.total_rows, x, dy, partial);
    }
    int st = cnn::launch_check(ctx, "wgrad");
    if (st != CNN_OK) return st;
    const size_t total = (size_t)G::RS * s.K * s.C;
    size_t g = (total + 255) / 256;
    if (g > 4096) g = 4096;
    {
        cnn::ProfScope ps(ctx, "k_wgrad_reduce", 0.0);
        hipLaunchKernelGGL(k_wgrad_reduce, dim3((unsigned)g), dim3(256), 0, ctx->stream, p.nsplit * p.col_tiles, G::RS,
                           s.K * s.C, partial, dw);
    }
    return cnn::launch_check(ctx, "wgrad_reduce");
}

// (R, S, pad, TW, NBI, KW, CW, RW, NSLOT)
#define WG_TABLE(X)                                   \
    X(3, 3, 1, 56, 1, 4, 2, 1, 4)                      \
    X(3, 3, 1, 28, 2, 4, 2, 1, 4)                      \
    X(3, 3, 1, 14, 4, 4, 2, 1, 4)                      \
    X(3, 3, 1, 12, 4, 4, 2, 1, 4)                      \
    X(5, 5, 0, 24, 2, 2, 1, 5, 8)

template <class F>
int select(const ConvShape& s, F&& f) {
    if (s.stride != 1 || s.C < 16) return CNN_EUNSUPPORTED;
    if (s.P != s.H + 2 * s.pad - s.R + 1 || s.Q != s.W + 2 * s.pad - s.S + 1) return CNN_EUNSUPPORTED;
#define X(R_, S_, P_, TW_, NBI_, KW_, CW_, RW_, NS_)                                                     \
    if (s.R == R_ && s.S == S_ && s.pad == P_ && s.Q % TW_ == 0 && (s.Q == TW_ || TW_ >= 56))            \
        return f(WgCfg<R_, S_, P_, TW_, NBI_, KW_, CW_, RW_, NS_>{});
    WG_TABLE(X)
#undef X
    return CNN_EUNSUPPORTED;
}

}  // namespace

namespace cnn {

size_t mfma_conv_bwd_weight_ws(const ConvShape& s) {
    size_t bytes = 0;
    select(s, [&](auto g) {
        bytes = make_plan<decltype(g)>(s).ws_bytes;
        return CNN_OK;
    });
    return bytes;
}

int mfma_conv_bwd_weight(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, float* dw) {
    return select(s, [&](auto g) { return launch<decltype(g)>(ctx, s, x, dy, dw); });
}

}  // namespace cnn
