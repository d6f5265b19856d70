// Forward propagation (Section 2.1, Algorithm 1) for a strided first layer: three input feature maps, a large
// kernel and stride > 1 (OverFeat-FAST's 11x11 / stride 4).  The generic tiled kernel needs stride 1 for its
// conflict-free LDS reads; here
//   D[k][pixel] = sum_{c,r,s} w[k][c][r][s] * x[c][p*ST + r][q*ST + s]
// runs on the fp32 matrix cores with A = filters (lane = output feature), B = input gathered from an LDS tile
// (lane = output pixel).  With stride ST the 32 lanes of a B operand would read every ST-th word (ST-way bank
// conflicts), so the tile is stored de-interleaved by column phase: x[c][row][w] -> xl[c][row][w % ST][w / ST];
// lane q then reads consecutive words for any tap.
// The contraction runs over chunks of two kernel rows: the low wave half (MFMA k = 0) takes row r, the high half row
// r + 1, and both walk the same (channel, kernel column) sequence, so every operand offset inside a chunk is an
// immediate and the halves differ by a constant folded into the per-lane base (R odd: the last chunk pairs the last
// row with a row of zero weights read against a row of zeros).  The input tile (all rows the TH output rows need)
// is loaded once per workgroup by raw buffer loads (rows past the image read 0).  The filters never touch LDS: an A
// operand is one filter element per lane, so every lane loads the elements of its own output feature and kernel
// row straight from HBM / L2 into registers, one chunk ahead, one load per MFMA step; the B operands of each step
// are read one step ahead.  After the tile is in LDS there is no barrier.
#include <stdio.h>

#include "common.h"

namespace {



template <int R_, int S_, int ST_, int TH_, int WI_, int KBK_, int NT_>
struct C3Cfg {
    static constexpr int R = R_, S = S_, ST = ST_, TH = TH_, WI = WI_, KBK = KBK_, NT = NT_, C = 3;
    static constexpr int WO = (WI - S) / ST + 1;
    static constexpr int NCH = (R + 1) / 2;                       // chunks: pairs of kernel rows
    static constexpr int ROWS = (TH - 1) * ST + 2 * NCH;          // input rows of one tile (incl. the zero-weight row)
    static constexpr int PW = (WI + ST - 1) / ST;                 // words per column phase
    static constexpr int ROWP = ST * PW;                          // LDS words per input row
    static constexpr int PLANE = ROWS * ROWP;
    static constexpr int JC = C * S;                              // MFMA steps per chunk: (channel, kernel column)
    static constexpr int KROWS = 32 * KBK;
    static constexpr int T = 64 * KBK;
    static constexpr int NPIX = TH * WO;
    static constexpr int XPASS = (WI + 63) / 64;                  // column passes of a wave over one input row
    static constexpr int LDS_BYTES = C * PLANE * 4;
    static_assert(NT * 32 >= NPIX && NT * 32 - NPIX < 32, "pixel tile padded by less than one block");
    static_assert((C * ROWS) % (T / 64) == 0, "the waves share the input rows evenly");
};

template <class G>
__global__ void __launch_bounds__(G::T, 2)      // two waves per SIMD: two workgroups per compute unit
k_conv_c3_strided(int N, int K, int HI, int HO, int row_tiles, int relu, const float* __restrict__ x,
                  const float* __restrict__ w, float* __restrict__ y) {
    constexpr int R = G::R, S = G::S, ST = G::ST, NT = G::NT, C = G::C, JC = G::JC;
    extern __shared__ float lds[];
    float* xl = lds;                       // [C][ROWS][ST][PW]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int n = blockIdx.x / row_tiles, p0 = (blockIdx.x % row_tiles) * G::TH;

    // ---- input tile, de-interleaved by column phase: wave w takes (channel, row) pairs w, w + NW, ...; its lanes
    //      walk the columns.  Rows past the image (and the extra row under the zero weights) read 0.
    {
        const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(x) + (size_t)n * C * HI * G::WI, 0, C * HI * G::WI * (int)sizeof(float), kRsrcWord3);
        int cvo[G::XPASS], cl[G::XPASS];
#pragma unroll
        for (int t = 0; t < G::XPASS; ++t) {
            const int col = lane + 64 * t;
            cvo[t] = col < G::WI ? col * (int)sizeof(float) : kOutOfRange;      // the words past the last column get 0
            cl[t] = (col % ST) * G::PW + col / ST;
        }
        constexpr int NW = G::T / 64, PAIRS = C * G::ROWS / NW;
        // the loads of half the wave's rows are issued before their first LDS write (two trips to HBM instead of one
        // per row; all at once would cost the registers a second wave per SIMD needs)
        constexpr int BATCH = PAIRS / 2;
        static_assert(PAIRS % 2 == 0, "two equal batches");
#pragma unroll
        for (int b0 = 0; b0 < PAIRS; b0 += BATCH) {
            float v[BATCH][G::XPASS];
#pragma unroll
            for (int pp = 0; pp < BATCH; ++pp) {
                const int pr = wave + (b0 + pp) * NW, c = pr / G::ROWS, row = pr % G::ROWS;
                const int h = p0 * ST + row;
                const bool live = h < HI && row < G::ROWS - 1;          // the last row stays zero (see the last chunk)
#pragma unroll
                for (int t = 0; t < G::XPASS; ++t)
                    v[pp][t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                             rs_x, live ? cvo[t] : kOutOfRange,
                                                             (c * HI + (live ? h : 0)) * G::WI * (int)sizeof(float), 0));
            }
#pragma unroll
            for (int pp = 0; pp < BATCH; ++pp) {
                const int pr = wave + (b0 + pp) * NW, c = pr / G::ROWS, row = pr % G::ROWS;
                float* d = xl + c * G::PLANE + row * G::ROWP;
#pragma unroll
                for (int t = 0; t < G::XPASS; ++t)
                    if (lane + 64 * t < G::ROWP) d[cl[t]] = v[pp][t];
            }
        }
    }

    // ---- filters: lane (half, l32) of wave w needs w[k = 32w + l32][c][2*ch + half][s] in chunk ch, step (c, s)
    const int kf = wave * 32 + l32;
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(w), 0, K * C * R * S * (int)sizeof(float), kRsrcWord3);
    const int w_vo = kf < K ? (kf * C * R * S + half * S) * (int)sizeof(float) : kOutOfRange;
    float wcur[JC];      // refreshed in place: element t of the next chunk is requested right after step t used it
    auto fetch_w = [&](int j, int ch, float (&dst)[JC]) {     // element j = (c, s) of chunk ch
        const int c = j / S, s = j % S;
        const int vo = 2 * ch + half < R ? w_vo : kOutOfRange;     // the row under the last odd row: zeros
        dst[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                               rs_w, vo + (c * R * S + s) * (int)sizeof(float), 2 * ch * S * (int)sizeof(float), 0));
    };
#pragma unroll
    for (int j = 0; j < JC; ++j) fetch_w(j, 0, wcur);

    // ---- per-lane B operand bases: the high half reads the pair's second kernel row
    const lds_float* bp[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = j * 32 + l32;
        bp[j] = (const lds_float*)(xl + (i < G::NPIX ? (i / G::WO) * ST * G::ROWP + i % G::WO : 0) + half * G::ROWP);
    }
    f32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    // B operands of step t of a chunk: channel t / S, kernel column t % S
    auto read_step = [&](int t, float (&b)[NT]) {
        const int c = t / S, s = t % S;
#pragma unroll
        for (int j = 0; j < NT; ++j) b[j] = bp[j][c * G::PLANE + (s % ST) * G::PW + s / ST];
    };

    __syncthreads();       // the input tile is complete
    float b_cur[NT];
    read_step(0, b_cur);
    for (int ch = 0; ch < G::NCH; ++ch) {
        const int ch1 = ch + 1 < G::NCH ? ch + 1 : G::NCH - 1;     // past the end: the last chunk again, never used
#pragma unroll
        for (int t = 0; t < JC; ++t) {
            float b_nxt[NT];
            if (t + 1 < JC) {
                read_step(t + 1, b_nxt);
            } else {
                // next pair of kernel rows; R odd: in the last chunk the high half has zero weights and reads the
                // tile's zero row (never 0 x data)
                const bool zero_row = (R & 1) && ch + 2 == G::NCH && half;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int i = j * 32 + l32;
                    bp[j] = zero_row ? (const lds_float*)(xl + (G::ROWS - 1) * G::ROWP + (i < G::NPIX ? i % G::WO : 0))
                                     : bp[j] + 2 * G::ROWP;
                }
                read_step(0, b_nxt);
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wcur[t], b_cur[j], acc[j], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 DS read
            }
            __builtin_amdgcn_sched_barrier(0);
            fetch_w(t, ch1, wcur);
#pragma unroll
            for (int j = 0; j < NT; ++j) b_cur[j] = b_nxt[j];
        }
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
    static std::atomic<unsigned long long> attr_done{0};     // one bit per device: the attribute is the device's
    {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_conv_c3_strided<G>), G::LDS_BYTES, "hipFuncSetAttribute(conv_c3_strided)");
        if (st_attr != CNN_OK) return st_attr;
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
