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
//   LDS xl[CBK][NBI][NSLOT][TW+S-1]   ring of input rows (columns outside the image are zero)
//   LDS dyl[2][KB][NBI*TW]            double-buffered dy row
// Row strides are odd so the 32 lanes of an operand (32 features) read 32 different banks.
// Narrow images are processed NBI at a time (one ring each) to keep about 56 pixels per step; wide rows are
// cut into column tiles of TW, each one more split.  TW, NBI, pad and all image sizes are run-time values.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct WgGeo {
    int N, C, K, HI, WI, HO, WO, pad;
    int TW, NBI, WLD;            // output columns per tile, images per step, staged input columns per row (TW+S-1)
    int XSTR, DSTR;              // odd LDS strides per input feature / output feature
    int col_tiles, rows_per_split, total_rows;
};

template <int R_, int S_, int KW_, int CW_, int RW_, int NSLOT_>
struct WgCfg {
    static constexpr int R = R_, S = S_, KW = KW_, CW = CW_, RW = RW_, NSLOT = NSLOT_;
    static constexpr int RS = R * S, RPW = R / RW;
    static constexpr int KB = 32 * KW, CBK = 32 * CW;
    static constexpr int T = 64 * KW * CW * RW;
    static constexpr int NWAVE = T / 64;
    static constexpr int XS = (CBK + NWAVE - 1) / NWAVE, DS = (KB + NWAVE - 1) / NWAVE;   // rows staged per wave per step
    static_assert(R % RW == 0 && NSLOT >= R + 1 && (NSLOT & (NSLOT - 1)) == 0, "ring geometry");
};

template <class G>
__global__ void __launch_bounds__(G::T)
k_wgrad(WgGeo g, const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ partial) {
    constexpr int R = G::R, S = G::S, NSLOT = G::NSLOT, T = G::T;
    const int N = g.N, C = g.C, K = g.K, HI = g.HI, WI = g.WI, HO = g.HO, WO = g.WO, PAD = g.pad;
    const int TW = g.TW, NBI = g.NBI, WLD = g.WLD;
    extern __shared__ float lds[];
    float* xl = lds;                                  // [CBK][XSTR]
    float* dyl = lds + G::CBK * g.XSTR;               // [2][KB][DSTR]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int kw = wave % G::KW, cw = (wave / G::KW) % G::CW, rw = wave / (G::KW * G::CW);

    const int split = blockIdx.x / g.col_tiles, q0 = (blockIdx.x % g.col_tiles) * TW;
    const int c0 = blockIdx.y * G::CBK, k0 = blockIdx.z * G::KB;

    // output rows are numbered gr = group*HO + p over image groups of NBI images
    const int g_begin = split * g.rows_per_split;
    const int g_end = min(g_begin + g.rows_per_split, g.total_rows);
    const int V = HO + R - 1;                         // input rows of one image incl. the zero rows above/below

    // zero the whole ring once (slots never written are never read, but must not hold NaN patterns)
    for (int e = tid; e < G::CBK * g.XSTR; e += T) xl[e] = 0.f;

    // staging: wave w fetches feature rows w, w+NWAVE, ...; lane = position in the row(s) of the NBI images
    int xo = -1, xlds = 0;
    const int xb = lane / WLD;
    {
        const int col = lane % WLD, w = q0 - PAD + col;
        if (lane < NBI * WLD) {
            xlds = wave * g.XSTR + xb * NSLOT * WLD + col;
            if (w >= 0 && w < WI) xo = (xb * C + c0 + wave) * HI * WI + w;
        }
    }
    int dyo = -1, dlds = 0;
    const int db = lane / TW;
    {
        const int q = lane % TW;
        if (lane < NBI * TW) {
            dlds = wave * g.DSTR + db * TW + q;
            dyo = (db * K + k0 + wave) * HO * WO + q0 + q;
        }
    }

    f32x16 acc[G::RPW][S];
#pragma unroll
    for (int r = 0; r < G::RPW; ++r)
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][s][v] = 0.f;

    // LDS read bases.  Pixel i of the step: image b = i / TW, column q = i % TW.  The low wave half takes the
    // first half of the step's pixels, the high half the second: the other half of the columns (one image per
    // step) or the other half of the images.
    const int a_delta = NBI * TW / 2;                                          // in dyl: pixels are contiguous
    const int b_delta = NBI == 1 ? TW / 2 : (NBI / 2) * NSLOT * WLD;           // in xl
    const int nb_loop = NBI == 1 ? 1 : NBI / 2, q_loop = NBI == 1 ? TW / 2 : TW;
    const int a_base = (kw * 32 + l32) * g.DSTR + half * a_delta;
    const int b_base = (cw * 32 + l32) * g.XSTR + half * b_delta;

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
        const int gr = grp * HO + p;
        const bool rowv = p >= 0 && gr >= g_begin && gr < g_end;
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
                    if (wave + i * G::NWAVE < G::CBK) xl[xlds + i * G::NWAVE * g.XSTR + slot * WLD] = xr[i];
            }
            if (lane < NBI * TW) {
#pragma unroll
                for (int i = 0; i < G::DS; ++i)
                    if (wave + i * G::NWAVE < G::KB) dyl[buf * G::KB * g.DSTR + dlds + i * G::NWAVE * g.DSTR] = dr[i];
            }
            __syncthreads();
            if (u < u_last) fetch(u + 1);
            const int vr = u % V, p = vr - (R - 1);
            const int gr = (u / V) * HO + p;
            if (p >= 0 && gr >= g_begin) {    // an output row completes at this step (gr < g_end by construction)
                const float* ap = dyl + buf * G::KB * g.DSTR + a_base;
                const float* bp = xl + b_base;
                int so[G::RPW];
#pragma unroll
                for (int r = 0; r < G::RPW; ++r) so[r] = ((u - (R - 1) + rw * G::RPW + r) & (NSLOT - 1)) * WLD;
                for (int b = 0; b < nb_loop; ++b) {
                    const float* apb = ap + b * TW;
                    const float* bpb = bp + b * NSLOT * WLD;
                    // two pixels' operands are fetched before their 2 x RPW x S MFMAs are issued
                    int q = 0;
                    for (; q + 1 < q_loop; q += 2) {
                        const float a0 = apb[q], a1 = apb[q + 1];
                        float b0[G::RPW][S], b1[G::RPW][S];
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s) {
                                b0[r][s] = bpb[so[r] + q + s];
                                b1[r][s] = bpb[so[r] + q + 1 + s];
                            }
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s)
                                acc[r][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0[r][s], acc[r][s], 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s)
                                acc[r][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1[r][s], acc[r][s], 0, 0, 0);
                    }
                    if (q < q_loop) {
                        const float a = apb[q];
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                            for (int s = 0; s < S; ++s)
                                acc[r][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bpb[so[r] + q + s], acc[r][s], 0, 0, 0);
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
    WgGeo g;
    int nsplit, ktiles, ctiles;
    size_t lds_bytes, ws_bytes;
};

// Column tile TW (a divisor of Q with TW+S-1 <= 64 staged columns) and images per step NBI in {1, 2, 4}: the pair
// that gives the most pixels per step within the 64 lanes that stage one feature's row(s); then the number of row
// splits that minimises the time of the slowest compute unit.
template <class G>
bool make_plan(const ConvShape& s, Plan* p) {
    if (s.stride != 1 || s.C < 16 || s.R != G::R || s.S != G::S) return false;
    if (s.P != s.H + 2 * s.pad - s.R + 1 || s.Q != s.W + 2 * s.pad - s.S + 1) return false;
    int best_tw = 0, best_nbi = 0;
    double best_score = 0.0;
    for (int tw = 1; tw <= s.Q && tw + G::S - 1 <= 64; ++tw) {
        if (s.Q % tw) continue;
        for (int nbi = 1; nbi <= 4; nbi *= 2) {
            if (nbi * (tw + G::S - 1) > 64) continue;
            if (nbi == 1 && (tw & 1)) continue;                      // the wave halves split the step's pixels evenly
            double score = (double)nbi * tw;
            if (nbi > s.N) score *= (double)s.N / nbi;               // images that do not exist are wasted lanes
            score *= 1.0 - 0.02 * (s.Q / tw - 1);                    // column tiles re-read halo columns
            if (score > best_score + 1e-9) { best_score = score; best_tw = tw; best_nbi = nbi; }
        }
    }
    if (!best_tw) return false;
    WgGeo& g = p->g;
    g.N = s.N; g.C = s.C; g.K = s.K; g.HI = s.H; g.WI = s.W; g.HO = s.P; g.WO = s.Q; g.pad = s.pad;
    g.TW = best_tw; g.NBI = best_nbi; g.WLD = best_tw + G::S - 1;
    const int xrow = g.NBI * G::NSLOT * g.WLD, drow = g.NBI * g.TW;
    g.XSTR = (xrow & 1) ? xrow : xrow + 1;
    g.DSTR = (drow & 1) ? drow : drow + 1;
    g.col_tiles = s.Q / g.TW;
    p->ktiles = (s.K + G::KB - 1) / G::KB;
    p->ctiles = (s.C + G::CBK - 1) / G::CBK;
    const int groups = (s.N + g.NBI - 1) / g.NBI;
    g.total_rows = groups * s.P;
    const int tiles = p->ktiles * p->ctiles * g.col_tiles;
    // Row splits: a split of n rows costs n + R - 1 steps (ring warm-up), the workgroups run 256 at a time (one per
    // compute unit, the LDS ring fills it), and every split adds one private copy of dw to write and read back
    // (a step moves about as many bytes as 70 MB of that traffic takes).
    const double copy_steps = (double)G::RS * s.K * s.C * 8.0 / 70e6;
    double best = 1e30;
    int best_split = 1;
    for (int ns = 1; ns <= g.total_rows; ++ns) {
        const int rps = (g.total_rows + ns - 1) / ns;
        const int real = (g.total_rows + rps - 1) / rps;
        if (real != ns) continue;
        const long rounds = ((long)tiles * ns + 255) / 256;
        const double cost = (double)rounds * (rps + G::R - 1) + copy_steps * ns;
        if (cost < best) { best = cost; best_split = ns; }
        if (rps == 1) break;
    }
    p->nsplit = best_split;
    g.rows_per_split = (g.total_rows + best_split - 1) / best_split;
    p->lds_bytes = ((size_t)G::CBK * g.XSTR + 2 * (size_t)G::KB * g.DSTR) * sizeof(float);
    p->ws_bytes = (size_t)p->nsplit * g.col_tiles * G::RS * s.K * s.C * sizeof(float);
    return p->lds_bytes <= 156 * 1024;
}

template <class G>
int launch(cnn_ctx* ctx, const Plan& p, const ConvShape& s, const float* x, const float* dy, float* dw) {
    if (ctx->ws_bytes < p.ws_bytes || !ctx->ws) return CNN_EWORKSPACE;
    static size_t attr_bytes = 48 * 1024;
    if (p.lds_bytes > attr_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wgrad<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds_bytes);
        if (e != hipSuccess) return cnn::hip_check(ctx, e, "hipFuncSetAttribute(wgrad)");
        attr_bytes = p.lds_bytes;
    }
    float* partial = reinterpret_cast<float*>(ctx->ws);
    dim3 grid((unsigned)(p.nsplit * p.g.col_tiles), (unsigned)p.ctiles, (unsigned)p.ktiles);
    static char name[96] = "";
    if (!name[0]) snprintf(name, sizeof(name), "k_wgrad<%dx%d KW%d CW%d RW%d>", G::R, G::S, G::KW, G::CW, G::RW);
    {
        cnn::ProfScope ps(ctx, name, cnn::conv_flops(s));
        hipLaunchKernelGGL(k_wgrad<G>, grid, dim3(G::T), p.lds_bytes, ctx->stream, p.g, x, dy, partial);
    }
    int st = cnn::launch_check(ctx, "wgrad");
    if (st != CNN_OK) return st;
    const size_t total = (size_t)G::RS * s.K * s.C;
    size_t gsz = (total + 255) / 256;
    if (gsz > 4096) gsz = 4096;
    {
        cnn::ProfScope ps(ctx, "k_wgrad_reduce", 0.0);
        hipLaunchKernelGGL(k_wgrad_reduce, dim3((unsigned)gsz), dim3(256), 0, ctx->stream, p.nsplit * p.g.col_tiles, G::RS,
                           s.K * s.C, partial, dw);
    }
    return cnn::launch_check(ctx, "wgrad_reduce");
}

// (R, S, KW, CW, RW, NSLOT): 3x3 -> 128 k x 64 c x 9 taps per workgroup (8 waves); 5x5 -> 64 k x 32 c, one kernel
// row per wave (10 waves)
using Wg3 = WgCfg<3, 3, 4, 2, 1, 4>;
using Wg5 = WgCfg<5, 5, 2, 1, 5, 8>;

}  // namespace

namespace cnn {

size_t mfma_conv_bwd_weight_ws(const ConvShape& s) {
    Plan p;
    if (make_plan<Wg3>(s, &p) || make_plan<Wg5>(s, &p)) return p.ws_bytes;
    return 0;
}

int mfma_conv_bwd_weight(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, float* dw) {
    Plan p;
    if (make_plan<Wg3>(s, &p)) return launch<Wg3>(ctx, p, s, x, dy, dw);
    if (make_plan<Wg5>(s, &p)) return launch<Wg5>(ctx, p, s, x, dy, dw);
    return CNN_EUNSUPPORTED;
}

}  // namespace cnn
