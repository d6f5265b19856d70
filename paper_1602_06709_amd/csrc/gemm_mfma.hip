// fp32 GEMM on the gfx950 matrix cores for the fully-connected layers (Section 2.1: the convolution loop
// nest with k_h = k_w = out_h = out_w = 1; the paper's "block-SGEMM", Section 4).
//   C[M][Nn] = sum_k A(m,k) * B(n,k)
// Either operand may be stored with the contraction index contiguous ([rows][Kd]) or with it outermost
// ([Kd][rows]); the three FC passes are three such combinations and need no transposed copy of anything:
//   forward   y  = x  . w^T   A = x  [N][I],          B = w [O][I]
//   bwd-data  dx = dy . w     A = dy [N][O],          B = w [O][I] read as [Kd = O][Nn = I]
//   bwd-wt    dw = dy^T . x   A = dy [N][O] as [Kd = N][M = O],  B = x [N][I] as [Kd = N][Nn = I]
// Tiles go through LDS in a form whose operand reads are bank-conflict free: contraction-contiguous tiles
// as [row][KC+1] (odd stride across the 32 lanes), row-contiguous tiles as [k][rows].  The output has
// lane = column n (coalesced stores).  A small minibatch leaves few output tiles, so the contraction is
// split across workgroups and the partial products are added by a second kernel in a fixed order.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KC = 32;   // contraction elements per LDS chunk

template <int MT_, int NT_, int WGM_, int WGN_, bool AKM_, bool BKM_>
struct GemmCfg {
    static constexpr int MT = MT_, NT = NT_, WGM = WGM_, WGN = WGN_;
    static constexpr bool AKM = AKM_, BKM = BKM_;
    static constexpr int TM = 32 * MT * WGM, TN = 32 * NT * WGN, T = 64 * WGM * WGN;
    static constexpr int A_LDS = AKM ? KC * TM : TM * (KC + 1);
    static constexpr int B_LDS = BKM ? KC * TN : TN * (KC + 1);
    static constexpr int A4 = TM * KC / 4, B4 = TN * KC / 4;
    static constexpr int AS = (A4 + T - 1) / T, BS = (B4 + T - 1) / T;
};

// One operand tile: fetch `rows` x KC elements starting at (row0, k0) into registers, then into LDS.
template <bool KM, int ROWS, int T, int SLOTS>
struct Stager {
    // KM == false: src[row][Kd], float4 along k.  KM == true: src[Kd][rows_total], float4 along the row index.
    __device__ static void fetch(const float* __restrict__ src, int rows_total, int Kd, int row0, int k0, int k_end,
                                 int tid, float4 (&reg)[SLOTS]) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int f = tid + i * T;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (f < ROWS * KC / 4) {
                if (!KM) {
                    const int r = f / (KC / 4), kq = f % (KC / 4);
                    const int k = k0 + kq * 4;
                    if (row0 + r < rows_total && k < k_end)
                        v = *reinterpret_cast<const float4*>(src + (size_t)(row0 + r) * Kd + k);
                } else {
                    const int k = f / (ROWS / 4), rq = f % (ROWS / 4);
                    const int r = row0 + rq * 4;
                    if (r < rows_total && k0 + k < k_end)
                        v = *reinterpret_cast<const float4*>(src + (size_t)(k0 + k) * rows_total + r);
                }
            }
            reg[i] = v;
        }
    }
    __device__ static void stage(float* __restrict__ l, int tid, const float4 (&reg)[SLOTS]) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int f = tid + i * T;
            if (f < ROWS * KC / 4) {
                if (!KM) {
                    const int r = f / (KC / 4), kq = f % (KC / 4);
                    float* d = l + r * (KC + 1) + kq * 4;
                    d[0] = reg[i].x; d[1] = reg[i].y; d[2] = reg[i].z; d[3] = reg[i].w;
                } else {
                    const int k = f / (ROWS / 4), rq = f % (ROWS / 4);
                    *reinterpret_cast<float4*>(l + k * ROWS + rq * 4) = reg[i];
                }
            }
        }
    }
};

template <class G>
__global__ void __launch_bounds__(G::T, 2)
k_gemm(int M, int Nn, int Kd, int k_per_split, const float* __restrict__ A, const float* __restrict__ B,
       float* __restrict__ Cout) {
    constexpr int MT = G::MT, NT = G::NT, T = G::T;
    __shared__ __attribute__((aligned(16))) float al[G::A_LDS];
    __shared__ __attribute__((aligned(16))) float bl[G::B_LDS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm = wave % G::WGM, wn = wave / G::WGM;
    const int n0 = blockIdx.x * G::TN, m0 = blockIdx.y * G::TM;
    const int k_begin = blockIdx.z * k_per_split;
    const int k_end = min(k_begin + k_per_split, Kd);

    using SA = Stager<G::AKM, G::TM, T, G::AS>;
    using SB = Stager<G::BKM, G::TN, T, G::BS>;
    float4 ar[G::AS], br[G::BS];

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // LDS read addresses: element (row, k) at row*sr + k*sk; the high wave half starts KC/2 further along k
    constexpr int a_sr = G::AKM ? 1 : KC + 1, a_sk = G::AKM ? G::TM : 1;
    constexpr int b_sr = G::BKM ? 1 : KC + 1, b_sk = G::BKM ? G::TN : 1;
    int a_base[MT], b_base[NT];
#pragma unroll
    for (int i = 0; i < MT; ++i) a_base[i] = ((wm * MT + i) * 32 + l32) * a_sr + half * (KC / 2) * a_sk;
#pragma unroll
    for (int j = 0; j < NT; ++j) b_base[j] = ((wn * NT + j) * 32 + l32) * b_sr + half * (KC / 2) * b_sk;

    if (k_begin < k_end) {
        SA::fetch(A, M, Kd, m0, k_begin, k_end, tid, ar);
        SB::fetch(B, Nn, Kd, n0, k_begin, k_end, tid, br);
        for (int k0 = k_begin; k0 < k_end; k0 += KC) {
            SA::stage(al, tid, ar);
            SB::stage(bl, tid, br);
            __syncthreads();
            if (k0 + KC < k_end) {
                SA::fetch(A, M, Kd, m0, k0 + KC, k_end, tid, ar);
                SB::fetch(B, Nn, Kd, n0, k0 + KC, k_end, tid, br);
            }
#pragma unroll
            for (int kk = 0; kk < KC / 2; ++kk) {
                float a[MT], b[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i) a[i] = al[a_base[i] + kk * a_sk];
#pragma unroll
                for (int j = 0; j < NT; ++j) b[j] = bl[b_base[j] + kk * b_sk];
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        }
    }

    float* out = Cout + (size_t)blockIdx.z * M * Nn;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int n = n0 + (wn * NT + j) * 32 + l32;
            if (n >= Nn) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * MT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (m < M) out[(size_t)m * Nn + n] = acc[i][j][v];
            }
        }
}

// C[i] = sum over splits of partial[split][i], in split order (float4 lanes; MN % 4 == 0 not required).
__global__ void __launch_bounds__(256) k_splitk_reduce(int nsplit, size_t MN, const float* __restrict__ partial,
                                                      float* __restrict__ C) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < MN; i += (size_t)gridDim.x * 256) {
        float s0 = 0.f, s1 = 0.f;
        int s = 0;
        for (; s + 1 < nsplit; s += 2) {
            s0 += partial[(size_t)s * MN + i];
            s1 += partial[(size_t)(s + 1) * MN + i];
        }
        if (s < nsplit) s0 += partial[(size_t)s * MN + i];
        C[i] = s0 + s1;
    }
}

struct GemmPlan {
    int tm, tn, nsplit, k_per_split;
    size_t ws_bytes;
};

GemmPlan plan_gemm(int M, int Nn, int Kd) {
    GemmPlan p;
    p.tm = M <= 64 ? 64 : 128;
    p.tn = 128;
    const long tiles = (long)((M + p.tm - 1) / p.tm) * ((Nn + p.tn - 1) / p.tn);
    int want = tiles >= 256 ? 1 : (int)((512 + tiles - 1) / tiles);
    const int chunks = (Kd + KC - 1) / KC;
    int max_split = chunks / 8;            // at least 8 chunks (256 contraction elements) per split
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    const int cps = (chunks + want - 1) / want;
    p.k_per_split = cps * KC;
    p.nsplit = (Kd + p.k_per_split - 1) / p.k_per_split;
    p.ws_bytes = p.nsplit > 1 ? (size_t)p.nsplit * M * Nn * sizeof(float) : 0;
    return p;
}

template <class G>
int launch(cnn_ctx* ctx, const GemmPlan& p, int M, int Nn, int Kd, const float* A, const float* B, float* C) {
    float* dst = p.nsplit > 1 ? reinterpret_cast<float*>(ctx->ws) : C;
    dim3 grid((unsigned)((Nn + G::TN - 1) / G::TN), (unsigned)((M + G::TM - 1) / G::TM), (unsigned)p.nsplit);
    static char name[96] = "";
    if (!name[0])
        snprintf(name, sizeof(name), "k_gemm<%dx%d %s%s>", G::TM, G::TN, G::AKM ? "At" : "A", G::BKM ? "B" : "Bt");
    {
        cnn::ProfScope ps(ctx, name, 2.0 * M * Nn * Kd);
        hipLaunchKernelGGL(k_gemm<G>, grid, dim3(G::T), 0, ctx->stream, M, Nn, Kd, p.k_per_split, A, B, dst);
    }
    int st = cnn::launch_check(ctx, "gemm");
    if (st != CNN_OK || p.nsplit == 1) return st;
    const size_t MN = (size_t)M * Nn;
    size_t g = (MN + 255) / 256;
    if (g > 4096) g = 4096;
    {
        cnn::ProfScope ps(ctx, "k_splitk_reduce", 0.0);
        hipLaunchKernelGGL(k_splitk_reduce, dim3((unsigned)g), dim3(256), 0, ctx->stream, p.nsplit, MN, dst, C);
    }
    return cnn::launch_check(ctx, "splitk_reduce");
}

}  // namespace

namespace cnn {

size_t mfma_gemm_ws(int M, int Nn, int Kd) {
    if (M <= 0 || Nn <= 0 || Kd <= 0) return 0;
    return plan_gemm(M, Nn, Kd).ws_bytes;
}

int mfma_gemm(cnn_ctx* ctx, int M, int Nn, int Kd, const float* A, int akm, const float* B, int bkm, float* C) {
    // float4 fetches along the contiguous index of each operand
    if ((akm ? M : Kd) % 4 != 0 || (bkm ? Nn : Kd) % 4 != 0) return CNN_EUNSUPPORTED;
    const GemmPlan p = plan_gemm(M, Nn, Kd);
    if (p.ws_bytes && (!ctx->ws || ctx->ws_bytes < p.ws_bytes)) return CNN_EWORKSPACE;
#define GO(MT, NT, WGM, WGN)                                                                               \
    do {                                                                                                   \
        if (!akm && !bkm) return launch<GemmCfg<MT, NT, WGM, WGN, false, false>>(ctx, p, M, Nn, Kd, A, B, C); \
        if (!akm && bkm) return launch<GemmCfg<MT, NT, WGM, WGN, false, true>>(ctx, p, M, Nn, Kd, A, B, C);   \
        if (akm && bkm) return launch<GemmCfg<MT, NT, WGM, WGN, true, true>>(ctx, p, M, Nn, Kd, A, B, C);     \
        return launch<GemmCfg<MT, NT, WGM, WGN, true, false>>(ctx, p, M, Nn, Kd, A, B, C);                    \
    } while (0)
    if (p.tm == 64) GO(2, 1, 1, 4);
    GO(2, 2, 2, 2);
#undef GO
}

}  // namespace cnn
