// Weight gradient for layers with very few input feature maps (the first layer of a CNN: C = 3), any
// kernel size, stride and pad (Section 2.1 "Weight-gradient Update"; Section 2.5's C1 case: few
// (ifm, ofm) jobs, so the minibatch/pixel contraction is split, privatised and reduced).
//
// With C this small the MFMA's column index cannot be the input feature; it is the whole
// (input feature, kernel row, kernel col) triple j = (c, r, s), J = C*R*S of them:
//     D[k][j] += sum_pixels dy[k][pixel] * x[c_j][p*stride + r_j - pad][q*stride + s_j - pad]
// A = dy (lane = output feature k), B = x gathered through a per-lane offset (lane = j), MFMA k = pixel:
// the low wave half takes output column q, the high half column q + TW/2 of the same output row.
// The walk is along output rows; input rows stay in an LDS ring of NSLOT >= R + stride rows, so each
// step brings `stride` new input rows and one dy row (fetched into registers during the previous step).
// The layer is HBM-bound (it streams dy once); the matrix cores only have to keep up.
#include <stdio.h>

#include "common.h"

namespace {


struct SmallcArgs {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
    int TW;              // output columns per column tile (even, divides Q)
    int col_tiles;
    int WLD;             // input columns staged per row: (TW-1)*stride + S
    int nslot;           // ring slots (power of two >= R + stride)
    int cpl;             // LDS elements per input feature: nslot * WLD
    int dstr;            // LDS row stride of the dy tile (odd)
    int rows_per_split, total_rows;
};

// KBK: 32-blocks of output features; JB: 32-blocks of j per wave; JW x PW waves: JW split j, PW split the row's
// pixel pairs; CC input features; ST stride; NPASS = ceil(TW / 64) lanes-passes over a dy row.
// POOL: dy is the gradient behind a 2x2 max-pool, [N][K][P/2][Q/2], with the window positions parg of the pool's
// forward pass: the full-size gradient row (zero except at each window's recorded position) is formed on the way
// into LDS and never exists in memory.
template <int KBK, int JB, int JW, int PW, int CC, int ST, int NPASS, bool POOL>
__global__ void __launch_bounds__(256)
k_wgrad_smallc(SmallcArgs a, const float* __restrict__ x, const float* __restrict__ dy, const unsigned char* __restrict__ parg,
               float* __restrict__ partial) {
    constexpr int KROWS = 32 * KBK, RPWV = KROWS / 4;       // dy rows per wave
    extern __shared__ float lds[];
    float* xl = lds;                              // [CC][nslot][WLD]
    float* dyl = lds + CC * a.cpl;                // [2][KROWS][dstr]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int jw = wave % JW, pw = wave / JW;
    const int split = blockIdx.x / a.col_tiles, q0 = (blockIdx.x % a.col_tiles) * a.TW;
    const int g_begin = split * a.rows_per_split;
    const int g_end = min(g_begin + a.rows_per_split, a.total_rows);      // rows g = n*P + p
    const int RS = a.R * a.S, J = CC * RS;
    const int mask = a.nslot - 1;

    // input staging: thread = LDS column (tid < WLD), looping over (row, feature)
    const int xcol_w = q0 * ST - a.pad + tid;                             // input column of this thread
    const bool xcol_ok = tid < a.WLD && xcol_w >= 0 && xcol_w < a.W;
    // dy staging: wave = rows wave, wave+4, ...; lane (+64) = column
    // per-lane gather geometry
    int jr[JB], joff[JB];
#pragma unroll
    for (int b = 0; b < JB; ++b) {
        const int j = (jw * JB + b) * 32 + l32;
        const int jj = j < J ? j : 0;
        jr[b] = (jj % RS) / a.S;
        joff[b] = (jj / RS) * a.cpl + (jj % a.S) + half * (a.TW / 2) * ST;
    }
    const int a_lane = l32 * a.dstr + half * (a.TW / 2);

    f32x16 acc[KBK][JB];
#pragma unroll
    for (int i = 0; i < KBK; ++i)
#pragma unroll
        for (int b = 0; b < JB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][b][v] = 0.f;

    float xr[ST][CC], dr[RPWV][NPASS];
    int da[POOL ? RPWV : 1][1];      // POOL: the window position recorded for the fetched element

    // the ST newest input rows of output row p (image n): rows p*ST - pad + R - ST + i
    auto fetch_x = [&](int n, int p) {
        const float* xs = x + (size_t)n * CC * a.H * a.W;
        const int hb = p * ST - a.pad + a.R - ST;
#pragma unroll
        for (int i = 0; i < ST; ++i) {
            const int h = hb + i;
            const bool ok = xcol_ok && h >= 0 && h < a.H;
#pragma unroll
            for (int c = 0; c < CC; ++c) xr[i][c] = ok ? xs[((size_t)c * a.H + h) * a.W + xcol_w] : 0.f;
        }
    };
    auto fetch_dy = [&](int n, int p) {
        if (POOL) {
            // lane l takes the pooled element of columns (2l, 2l+1), row p/2: one read serves two columns and both
            // rows of the pair
            const int PP = a.P / 2, QP = a.Q / 2;
#pragma unroll
            for (int i = 0; i < RPWV; ++i) {
                const int k = wave + 4 * i;
                const bool ok = k < a.K && 2 * lane < a.TW;
                const size_t e = ok ? (((size_t)n * a.K + k) * PP + (p >> 1)) * QP + (q0 >> 1) + lane : 0;
                dr[i][0] = dy[e];
                da[POOL ? i : 0][0] = parg[e];
            }
            return;
        }
        const float* ds = dy + ((size_t)n * a.K * a.P + p) * a.Q + q0;
#pragma unroll
        for (int i = 0; i < RPWV; ++i) {
            const int k = wave + 4 * i;
#pragma unroll
            for (int h = 0; h < NPASS; ++h) {
                const int q = lane + 64 * h;
                dr[i][h] = (k < a.K && q < a.TW) ? ds[(size_t)k * a.P * a.Q + q] : 0.f;
            }
        }
    };

    if (g_begin < g_end) {
        fetch_dy(g_begin / a.P, g_begin % a.P);
        bool fresh = true;                        // the whole R-row window must be (re)loaded
        for (int g = g_begin; g < g_end; ++g) {
            const int n = g / a.P, p = g % a.P, buf = g & 1;
            if (fresh) {
                // start of the range or of an image: all R rows straight into the ring (no prefetch)
                __syncthreads();                  // nobody still reads the previous image's rows
                const float* xs = x + (size_t)n * CC * a.H * a.W;
                if (tid < a.WLD) {
                    // rows in batches of 4: all loads of a batch are issued before its first LDS write (one trip to
                    // HBM per batch instead of one per element)
                    for (int r0 = 0; r0 < a.R; r0 += 4) {
                        float t[4][CC];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int h = p * ST - a.pad + r0 + i;
                            const bool ok = xcol_ok && r0 + i < a.R && h >= 0 && h < a.H;
#pragma unroll
                            for (int c = 0; c < CC; ++c) t[i][c] = ok ? xs[((size_t)c * a.H + h) * a.W + xcol_w] : 0.f;
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int h = p * ST - a.pad + r0 + i;
                            if (r0 + i < a.R)
#pragma unroll
                                for (int c = 0; c < CC; ++c) xl[c * a.cpl + ((h + a.pad) & mask) * a.WLD + tid] = t[i][c];
                        }
                    }
                }
            } else if (tid < a.WLD) {
                const int hb = p * ST - a.pad + a.R - ST;
#pragma unroll
                for (int i = 0; i < ST; ++i)
#pragma unroll
                    for (int c = 0; c < CC; ++c) xl[c * a.cpl + ((hb + i + a.pad) & mask) * a.WLD + tid] = xr[i][c];
            }
            if (POOL) {
                // the gradient belongs to the window position 2 * (row parity) + (column parity); the other column gets 0
                if (2 * lane < a.TW) {
#pragma unroll
                    for (int i = 0; i < RPWV; ++i) {
                        const bool live = wave + 4 * i < a.K;
                        const int pos = da[POOL ? i : 0][0] - 2 * (p & 1);
                        float* d = dyl + (buf * KROWS + wave + 4 * i) * a.dstr + 2 * lane;
                        d[0] = (live && pos == 0) ? dr[i][0] : 0.f;
                        d[1] = (live && pos == 1) ? dr[i][0] : 0.f;
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < RPWV; ++i)
#pragma unroll
                    for (int h = 0; h < NPASS; ++h)
                        if (lane + 64 * h < a.TW) dyl[(buf * KROWS + wave + 4 * i) * a.dstr + lane + 64 * h] = dr[i][h];
            }
            __syncthreads();
            fresh = false;
            if (g + 1 < g_end) {
                const int n1 = (g + 1) / a.P, p1 = (g + 1) % a.P;
                if (!POOL || !(p1 & 1)) fetch_dy(n1, p1);     // POOL: an odd row reads what the even row before it read
                if (p1 == 0 || ST >= a.R) fresh = true;
                else fetch_x(n1, p1);
            }
            // multiply: this wave's share of the row's pixel pairs
            const int pairs = a.TW / 2, ppw = (pairs + PW - 1) / PW;
            const int qa = pw * ppw, qb = min(qa + ppw, pairs);
            int boff[JB];
#pragma unroll
            for (int b = 0; b < JB; ++b) boff[b] = joff[b] + ((p * ST + jr[b]) & mask) * a.WLD;
            const float* ap = dyl + buf * KROWS * a.dstr + a_lane;
            // seven pixel pairs at a time: their operands are all read before the first MFMA, so the reads of one
            // group complete under the MFMAs of the previous one (a single pair per trip exposes the LDS latency).
            // Measured: a gain for the 9-MFMA pairs of the strided layers, none for the 2-MFMA pairs of stride 1.
            int q = qa;
            for (; KBK * JB >= 4 && q + 7 <= qb; q += 7) {
                float av[7][KBK], bv[7][JB];
#pragma unroll
                for (int u = 0; u < 7; ++u) {
#pragma unroll
                    for (int i = 0; i < KBK; ++i) av[u][i] = ap[i * 32 * a.dstr + q + u];
#pragma unroll
                    for (int b = 0; b < JB; ++b) bv[u][b] = xl[boff[b] + (q + u) * ST];
                }
#pragma unroll
                for (int u = 0; u < 7; ++u)
#pragma unroll
                    for (int i = 0; i < KBK; ++i)
#pragma unroll
                        for (int b = 0; b < JB; ++b)
                            acc[i][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][i], bv[u][b], acc[i][b], 0, 0, 0);
            }
            for (; q < qb; ++q) {
                float av[KBK], bv[JB];
#pragma unroll
                for (int i = 0; i < KBK; ++i) av[i] = ap[i * 32 * a.dstr + q];
#pragma unroll
                for (int b = 0; b < JB; ++b) bv[b] = xl[boff[b] + q * ST];
#pragma unroll
                for (int i = 0; i < KBK; ++i)
#pragma unroll
                    for (int b = 0; b < JB; ++b)
                        acc[i][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[b], acc[i][b], 0, 0, 0);
            }
            // One barrier per step suffices between ordinary steps: the next step writes the ST ring slots that no
            // wave still reads (nslot >= R + ST) and the other dy buffer, and a wave cannot run two steps ahead.
        }
    }

    // the PW waves that shared the row's pixels hold partial sums of the same elements: add them through LDS
    // (fixed order), then write one private copy per workgroup: partial[blockIdx.x][tap][k*C + c]
    if (PW > 1) {
        __syncthreads();                           // everyone is done with the tiles; reuse LDS as [PW][KBK*JB*16][64]
        float* red = lds;
#pragma unroll
        for (int i = 0; i < KBK; ++i)
#pragma unroll
            for (int b = 0; b < JB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[(pw * KBK * JB * 16 + (i * JB + b) * 16 + v) * 64 + lane] = acc[i][b][v];
        __syncthreads();
        if (pw == 0) {
#pragma unroll
            for (int i = 0; i < KBK; ++i)
#pragma unroll
                for (int b = 0; b < JB; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float t = acc[i][b][v];
                        for (int w = 1; w < PW; ++w) t += red[(w * KBK * JB * 16 + (i * JB + b) * 16 + v) * 64 + lane];
                        acc[i][b][v] = t;
                    }
        }
    }
    if (PW == 1 || pw == 0) {
        float* out = partial + (size_t)blockIdx.x * RS * a.K * CC;
#pragma unroll
        for (int b = 0; b < JB; ++b) {
            const int j = (jw * JB + b) * 32 + l32;
            if (j >= J) continue;
            const int c = j / RS, tap = j % RS;
#pragma unroll
            for (int i = 0; i < KBK; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    if (k < a.K) out[((size_t)tap * a.K + k) * CC + c] = acc[i][b][v];
                }
        }
    }
}

// dw[(k*C + c)*RS + tap] = sum over splits of partial[split][tap][k*C + c].  The output is tiny (a few thousand
// elements) and the splits many, so one workgroup sums 64 consecutive elements with 4 threads per element striding
// over the splits (coalesced 256-byte reads), then adds the 4 strided sums in a fixed order.
__global__ void __launch_bounds__(256) k_wgrad_reduce2(int nsplit, int RS, int KC, const float* __restrict__ partial,
                                                      GradSink sink) {
    __shared__ float red[4][64];
    const int total = RS * KC;
    const int e = blockIdx.x * 64 + (threadIdx.x & 63), part = threadIdx.x >> 6;
    float s0 = 0.f, s1 = 0.f;
    if (e < total) {
        int s = part;
        for (; s + 4 < nsplit; s += 8) {
            s0 += partial[(size_t)s * total + e];
            s1 += partial[(size_t)(s + 4) * total + e];
        }
        if (s < nsplit) s0 += partial[(size_t)s * total + e];
    }
    red[part][threadIdx.x & 63] = s0 + s1;
    __syncthreads();
    if (part == 0 && e < total) {
        const int l = threadIdx.x & 63;
        const float t = (red[0][l] + red[1][l]) + (red[2][l] + red[3][l]);
        sink_store(sink, (size_t)(e % KC) * RS + e / KC, t);
    }
}

struct SmallcPlan {
    SmallcArgs a;
    int variant;          // 0: K <= 32, J <= 32; 1: K <= 64, J <= 32; 2: K <= 96, J <= 384, stride 4; 3: ... stride 2
    int pw, nsplit;
    size_t lds_bytes, ws_bytes;
    bool ok;
};

SmallcPlan plan(const ConvShape& s) {
    SmallcPlan p{};
    p.ok = false;
    const int J = s.C * s.R * s.S;
    if (s.C != 3 || (s.Q & 1)) return p;
    int kbk;
    if (J <= 32 && s.K <= 32 && s.stride == 1) { p.variant = 0; kbk = 1; p.pw = 4; }
    else if (J <= 32 && s.K <= 64 && s.stride == 1) { p.variant = 1; kbk = 2; p.pw = 4; }
    else if (J <= 384 && s.K <= 96 && s.stride == 4) { p.variant = 2; kbk = 3; p.pw = 1; }
    else if (J <= 384 && s.K <= 96 && s.stride == 2) { p.variant = 3; kbk = 3; p.pw = 1; }
    else return p;
    SmallcArgs& a = p.a;
    a.N = s.N; a.C = s.C; a.H = s.H; a.W = s.W; a.K = s.K; a.R = s.R; a.S = s.S; a.stride = s.stride; a.pad = s.pad;
    a.P = s.P; a.Q = s.Q;
    // column tile: largest even divisor of Q within the lanes the dy staging covers (128 for stride 1, 64 else)
    const int tw_max = p.variant >= 2 ? 64 : 112;
    int tw = 0;
    for (int t = 2; t <= s.Q && t <= tw_max; t += 2)
        if (s.Q % t == 0) tw = t;
    if (!tw) return p;
    a.TW = tw;
    a.col_tiles = s.Q / tw;
    a.WLD = (tw - 1) * s.stride + s.S;
    if (a.WLD > 256) return p;                 // one thread per staged input column
    int ns = 1;
    while (ns < s.R + s.stride) ns <<= 1;
    a.nslot = ns;
    a.cpl = ns * a.WLD;
    a.dstr = (tw & 1) ? tw : tw + 1;
    a.total_rows = s.N * s.P;
    p.lds_bytes = ((size_t)s.C * a.cpl + 2 * 32 * kbk * a.dstr) * sizeof(float);
    // one round of workgroups: as many as the chip holds at once (one or two per compute unit, by LDS size)
    const int resident = p.lds_bytes <= 78 * 1024 ? 512 : 256;
    int want = (resident + a.col_tiles - 1) / a.col_tiles;
    const int warm = (s.R + s.stride - 1) / s.stride;      // steps' worth of rows a fresh window costs
    int min_rows = 4 * warm > 8 ? 4 * warm : 8;
    int max_split = a.total_rows / min_rows;
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    a.rows_per_split = (a.total_rows + want - 1) / want;
    p.nsplit = (a.total_rows + a.rows_per_split - 1) / a.rows_per_split;
    const size_t red_bytes = p.pw > 1 ? (size_t)p.pw * kbk * 16 * 64 * sizeof(float) : 0;   // cross-wave reduction scratch
    if (p.lds_bytes < red_bytes) p.lds_bytes = red_bytes;
    if (p.lds_bytes > 150 * 1024) return p;
    p.ws_bytes = (size_t)p.nsplit * a.col_tiles * s.R * s.S * s.K * s.C * sizeof(float);
    p.ok = true;
    return p;
}

template <int KBK, int JB, int JW, int PW, int CC, int ST, int NPASS, bool POOL = false>
int launch(cnn_ctx* ctx, const SmallcPlan& p, const ConvShape& s, const float* x, const float* dy, const GradSink& sink,
           const unsigned char* parg = nullptr) {
    auto kern = &k_wgrad_smallc<KBK, JB, JW, PW, CC, ST, NPASS, POOL>;
    static std::atomic<unsigned long long> attr_done{0};     // one bit per device: the attribute is the device's
    {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(kern), 150 * 1024, "hipFuncSetAttribute(wgrad_smallc)");
        if (st_attr != CNN_OK) return st_attr;
    }
    float* partial = reinterpret_cast<float*>(ctx->ws);
    static const std::string name_s = strf("k_wgrad_smallc<KB%d JB%d JW%d PW%d ST%d%s>", KBK, JB, JW, PW, ST, POOL ? " unpool" : "");
    const char* const name = name_s.c_str();
    {
        cnn::ProfScope ps(ctx, name, cnn::conv_flops(s));
        hipLaunchKernelGGL(kern, dim3((unsigned)(p.nsplit * p.a.col_tiles)), dim3(256), p.lds_bytes, ctx->stream, p.a, x, dy,
                           parg, partial);
    }
    int st = cnn::launch_check(ctx, "wgrad_smallc");
    if (st != CNN_OK) return st;
    const size_t total = (size_t)s.R * s.S * s.K * s.C;
    {
        cnn::ProfScope ps(ctx, sink.w ? "k_wgrad_reduce2<sgd>" : "k_wgrad_reduce2", 0.0);
        hipLaunchKernelGGL(k_wgrad_reduce2, dim3((unsigned)((total + 63) / 64)), dim3(256), 0, ctx->stream,
                           p.nsplit * p.a.col_tiles, s.R * s.S, s.K * s.C, partial, sink);
    }
    return cnn::launch_check(ctx, "wgrad_reduce2");
}

}  // namespace

namespace cnn {

size_t smallc_conv_bwd_weight_ws(const ConvShape& s) {
    const SmallcPlan p = plan(s);
    return p.ok ? p.ws_bytes : 0;
}

// dw = conv_bwd_weight(x, maxpool2_bwd(dpool, arg)): the stride-1 variants (3x3 first layers), even output sizes
bool smallc_unpool_serves(const ConvShape& s) {
    const SmallcPlan p = plan(s);
    return p.ok && p.variant <= 1 && !((s.P | s.Q) & 1);
}

int smallc_conv_bwd_weight_unpool(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dpool, const unsigned char* arg,
                                  const GradSink& dw) {
    if (!smallc_unpool_serves(s)) return CNN_EUNSUPPORTED;
    const SmallcPlan p = plan(s);
    if (!ctx->ws || ctx->ws_bytes < p.ws_bytes) return CNN_EWORKSPACE;
    if (p.variant == 0) return launch<1, 1, 1, 4, 3, 1, 2, true>(ctx, p, s, x, dpool, dw, arg);
    return launch<2, 1, 1, 4, 3, 1, 2, true>(ctx, p, s, x, dpool, dw, arg);
}

int smallc_conv_bwd_weight(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, const GradSink& dw) {
    const SmallcPlan p = plan(s);
    if (!p.ok) return CNN_EUNSUPPORTED;
    if (!ctx->ws || ctx->ws_bytes < p.ws_bytes) return CNN_EWORKSPACE;
    if (p.variant == 0) return launch<1, 1, 1, 4, 3, 1, 2>(ctx, p, s, x, dy, dw);
    if (p.variant == 1) return launch<2, 1, 1, 4, 3, 1, 2>(ctx, p, s, x, dy, dw);
    if (p.variant == 2) return launch<3, 3, 4, 1, 3, 4, 1>(ctx, p, s, x, dy, dw);
    return launch<3, 3, 4, 1, 3, 2, 1>(ctx, p, s, x, dy, dw);
}

}  // namespace cnn
