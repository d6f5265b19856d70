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



struct WgGeo {
    int N, C, K, HI, WI, HO, WO, pad;
    int TW, NBI, WLD;            // output columns per tile, images per step, staged input columns per row (TW+S-1)
    int XSTR, DSTR;              // odd LDS strides per input feature / output feature
    int col_tiles, rows_per_split, total_rows;
};

// TW_ / NBI_ != 0: the step geometry (output columns per tile, images per step) is a compile-time constant, C and K
// are multiples of the tile and every wave's feature rows lie inside it; the pixel-pair loop is then fully unrolled
// with immediate LDS offsets.  TW_ = 0: everything is a run-time value.
template <int R_, int S_, int KW_, int CW_, int RW_, int NSLOT_, int TW_ = 0, int NBI_ = 0>
struct WgCfg {
    static constexpr int R = R_, S = S_, KW = KW_, CW = CW_, RW = RW_, NSLOT = NSLOT_;
    static constexpr int TW_CT = TW_, NBI_CT = NBI_;
    static constexpr bool FIXED = TW_ != 0;
    // the waves share the tile's feature rows evenly: every wave stages whole rows at compile-time strides
    static constexpr bool EVEN = TW_ != 0 && (32 * CW_) % (KW_ * CW_ * RW_) == 0 && (32 * KW_) % (KW_ * CW_ * RW_) == 0;
    static constexpr int RS = R * S, RPW = R / RW;
    static constexpr int KB = 32 * KW, CBK = 32 * CW;
    static constexpr int T = 64 * KW * CW * RW;
    static constexpr int NWAVE = T / 64;
    static constexpr int XS = (CBK + NWAVE - 1) / NWAVE, DS = (KB + NWAVE - 1) / NWAVE;   // rows staged per wave per step
    // LDS strides per input / output feature: odd, so the 32 features of an operand read 32 different banks
    static constexpr int xstr(int tw, int nbi) { return (nbi * NSLOT * (tw + S - 1)) | 1; }
    static constexpr int dstr(int tw, int nbi) { return (nbi * tw) | 1; }
    static constexpr int QLOOP_CT = NBI_ == 1 ? TW_ / 2 : TW_;                 // columns per wave half and image
    static constexpr int NPAIRS_CT = (NBI_ == 1 ? 1 : NBI_ / 2) * ((QLOOP_CT + 1) / 2);
    static_assert(R % RW == 0 && NSLOT >= R + 1 && (NSLOT & (NSLOT - 1)) == 0, "ring geometry");
    static_assert(!FIXED || (QLOOP_CT % 2 == 0 && NBI_ * (TW_ + S - 1) <= 64),
                  "fixed geometry: even column share per wave half");
};

template <class G>
__global__ void __launch_bounds__(G::T)
k_wgrad(WgGeo g, const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ partial) {
    constexpr int R = G::R, S = G::S, NSLOT = G::NSLOT, T = G::T;
    const int N = g.N, C = g.C, K = g.K, HI = g.HI, WI = g.WI, HO = g.HO, WO = g.WO, PAD = g.pad;
    const int TW = G::FIXED ? G::TW_CT : g.TW, NBI = G::FIXED ? G::NBI_CT : g.NBI, WLD = TW + S - 1;
    const int XSTR = G::xstr(TW, NBI), DSTR = G::dstr(TW, NBI);
    extern __shared__ float lds[];
    float* xl = lds;                                  // [CBK][XSTR]
    float* dyl = lds + G::CBK * XSTR;                 // [2][KB][DSTR]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform
    const int half = lane >> 5, l32 = lane & 31;
    const int kw = wave % G::KW, cw = (wave / G::KW) % G::CW, rw = wave / (G::KW * G::CW);

    const int split = blockIdx.x / g.col_tiles, q0 = (blockIdx.x % g.col_tiles) * TW;
    const int c0 = blockIdx.y * G::CBK, k0 = blockIdx.z * G::KB;

    // output rows are numbered gr = group*HO + p over image groups of NBI images
    const int g_begin = split * g.rows_per_split;
    const int g_end = min(g_begin + g.rows_per_split, g.total_rows);
    const int V = HO + R - 1;                         // input rows of one image incl. the zero rows above/below

    // zero the whole ring once (slots never written are never read, but must not hold NaN patterns)
    for (int e = tid; e < G::CBK * XSTR; e += T) xl[e] = 0.f;

    // ---- staging: wave w moves feature rows w, w+NWAVE, ... (those past the tile repeat the tile's last row);
    //      lane = position in the row(s) of the NBI images (lanes past the row wrap around and repeat its first
    //      positions: same value to the same word, at most two lanes per word; more would be serialised).
    //      Loads are raw buffer loads: descriptor base + scalar offset (image group, feature, row) + per-lane byte
    //      offset; a lane whose position is outside the image, or whose image or row does not exist, carries an
    //      offset beyond the descriptor's range and the hardware returns 0.  Features past C / K read whatever
    //      follows (or 0 past the end of the tensor): their results are never stored.
    const int lx = lane % (NBI * WLD), ld = lane % (NBI * TW);
    const int xb = lx / WLD, db = ld / TW;
    int xvo, dvo;
    {
        const int w = q0 - PAD + lx % WLD;
        xvo = (w >= 0 && w < WI) ? (int)((xb * C * HI * WI + w) * sizeof(float)) : kOutOfRange;
        dvo = (int)((db * K * HO * WO + q0 + ld % TW) * sizeof(float));
    }
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, (int)((size_t)N * C * HI * WI * sizeof(float)), kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rs_dy =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(dy), 0, (int)((size_t)N * K * HO * WO * sizeof(float)), kRsrcWord3);
    // feature rows this wave stages: wave, wave + NWAVE, ... clamped to the tile's (and the tensor's) last row, as
    // scalar row indices relative to the tile's first row; the scalar part of a buffer address is not range-checked
    const int x_rows = min(G::CBK, C - c0), d_rows = min(G::KB, K - k0);
    // staging destinations of this wave's first feature row (fixed geometry) or of the tile's first row
    lds_float* const xw = (lds_float*)(xl + (G::EVEN ? wave * XSTR : 0) + xb * NSLOT * WLD + lx % WLD);   // + ring slot
    lds_float* const dw_ = (lds_float*)(dyl + (G::EVEN ? wave * DSTR : 0) + db * TW + ld % TW);           // + buffer

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
    const lds_float* const a_lane = (const lds_float*)(dyl + (kw * 32 + l32) * DSTR + half * a_delta);
    const lds_float* const b_lane = (const lds_float*)(xl + (cw * 32 + l32) * XSTR + half * b_delta);
    const int qh = (q_loop + 1) / 2, npairs = nb_loop * qh;                    // the pixels are taken two at a time

    float xr[G::XS], dr[G::DS];

    // step u (virtual input row): image group = u / V, row within the zero-extended image = u % V
    const int x_plane = HI * WI * (int)sizeof(float), d_plane = HO * WO * (int)sizeof(float);
    auto fetch = [&](int u) {
        const int grp = u / V, vr = u % V;
        const int h = vr - PAD, p = vr - (R - 1);
        const int nleft = N - grp * NBI;                 // images of this group that exist
        const int xo = (h >= 0 && h < HI && xb < nleft) ? xvo : kOutOfRange;
        const int so = (((grp * NBI * C + c0) * HI + min(max(h, 0), HI - 1)) * WI) * (int)sizeof(float);
        int sx = so + wave * x_plane;
#pragma unroll
        for (int i = 0; i < G::XS; ++i) {
            const int off = G::EVEN ? sx : so + min(wave + i * G::NWAVE, x_rows - 1) * x_plane;
            xr[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, xo, off, 0));
            sx += G::NWAVE * x_plane;
        }
        const int gr = grp * HO + p;
        const bool rowv = p >= 0 && gr >= g_begin && gr < g_end;
        const int dyo = (rowv && db < nleft) ? dvo : kOutOfRange;
        const int sd = (((grp * NBI * K + k0) * HO + min(max(p, 0), HO - 1)) * WO) * (int)sizeof(float);
        int sy = sd + wave * d_plane;
#pragma unroll
        for (int i = 0; i < G::DS; ++i) {
            const int off = G::EVEN ? sy : sd + min(wave + i * G::NWAVE, d_rows - 1) * d_plane;
            dr[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_dy, dyo, off, 0));
            sy += G::NWAVE * d_plane;
        }
    };
    // registers of step u -> ring slot u % NSLOT and dy buffer u % 2 (a wave past the tile's last feature row
    // repeats that row: same value to the same word)
    auto stage = [&](int u) {
        lds_float* xd = xw + (u & (NSLOT - 1)) * WLD;
#pragma unroll
        for (int i = 0; i < G::XS; ++i) xd[(G::EVEN ? i * G::NWAVE : min(wave + i * G::NWAVE, G::CBK - 1)) * XSTR] = xr[i];
        lds_float* dd = dw_ + (u & 1) * G::KB * DSTR;
#pragma unroll
        for (int i = 0; i < G::DS; ++i) dd[(G::EVEN ? i * G::NWAVE : min(wave + i * G::NWAVE, G::KB - 1)) * DSTR] = dr[i];
    };

    // operands of pixel pair (b, q) of step u: a[2], bv[r][S+1] (the two pixels' taps overlap in S-1 columns);
    // `two` is false for the single last pixel of an odd row
    auto load_pair = [&](const lds_float* ap, const lds_float* const (&bp)[G::RPW], bool two, float (&a)[2],
                         float (&bv)[G::RPW][S + 1]) {
        if (G::FIXED) two = true;
        a[0] = ap[0];
        a[1] = two ? ap[1] : 0.f;
#pragma unroll
        for (int r = 0; r < G::RPW; ++r) {
#pragma unroll
            for (int s2 = 0; s2 < S; ++s2) bv[r][s2] = bp[r][s2];
            bv[r][S] = two ? bp[r][S] : 0.f;
        }
    };
    // pointers to pair 0 of step u
    auto step_ptrs = [&](int u, const lds_float*& ap, const lds_float* (&bp)[G::RPW]) {
        ap = a_lane + (u & 1) * G::KB * DSTR;
#pragma unroll
        for (int r = 0; r < G::RPW; ++r) bp[r] = b_lane + ((u - (R - 1) + rw * G::RPW + r) & (NSLOT - 1)) * WLD;
    };

    if (g_begin < g_end) {
        const int u_begin = (g_begin / HO) * V + (g_begin % HO);
        const int u_last = ((g_end - 1) / HO) * V + ((g_end - 1) % HO) + R - 1;
        __syncthreads();   // ring zeroed
        fetch(u_begin);
        stage(u_begin);
        fetch(min(u_begin + 1, u_last));
        __syncthreads();
        // Step u first sends the registers holding step u+1 to the ring slot and dy buffer that step u does not read
        // (last read before the previous barrier) and requests step u+2 from HBM.  Then it multiplies the output
        // row that completes with input row u out of LDS, one pixel pair at a time, the next pair's operands being
        // read while the current pair's MFMAs run.  One barrier per step, placed before the last pair's MFMAs: the
        // first operands of step u+1 are read behind it while those MFMAs run.  Past the last step a clamped row
        // is staged and fetched again instead of branching (same values to the same words).
        const lds_float* ap;
        const lds_float* bp[G::RPW];
        float a_cur[2], b_cur[G::RPW][S + 1];
        step_ptrs(u_begin, ap, bp);
        load_pair(ap, bp, 1 < q_loop, a_cur, b_cur);
        const int wrap_a = TW - 2 * (qh - 1), wrap_b = NSLOT * WLD - 2 * (qh - 1);   // last pair of an image -> next image
        for (int u = u_begin; u <= u_last; ++u) {
            const int vr = u % V, p = vr - (R - 1);
            const int gr = (u / V) * HO + p;
            const int u1 = min(u + 1, u_last), u2 = min(u + 2, u_last);
            stage(u1);
            fetch(u2);
            // pairs of this step: none unless an output row completes (gr < g_end by construction)
            const int np = (p >= 0 && gr >= g_begin) ? npairs : 0;
            auto mfmas = [&]() {
#pragma unroll
                for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                    for (int s2 = 0; s2 < S; ++s2)
                        acc[r][s2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[0], b_cur[r][s2], acc[r][s2], 0, 0, 0);
#pragma unroll
                for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                    for (int s2 = 0; s2 < S; ++s2)
                        acc[r][s2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[1], b_cur[r][s2 + 1], acc[r][s2], 0, 0, 0);
            };
            auto rotate = [&](const float (&an)[2], const float (&bn)[G::RPW][S + 1]) {
                a_cur[0] = an[0]; a_cur[1] = an[1];
#pragma unroll
                for (int r = 0; r < G::RPW; ++r)
#pragma unroll
                    for (int s2 = 0; s2 <= S; ++s2) b_cur[r][s2] = bn[r][s2];
            };
            // one MFMA, then one of the next pair's LDS reads, and so on
            auto interleave = [&]() {
#pragma unroll
                for (int k = 0; k < 2 * G::RPW * S; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            // all pairs but the last
            if (np) {
                if constexpr (G::FIXED) {
                    // fully unrolled: pair i sits at compile-time offsets from the step's pointers
                    constexpr int QH = (G::QLOOP_CT + 1) / 2;
#pragma unroll
                    for (int i = 1; i < G::NPAIRS_CT; ++i) {
                        float a_nxt[2], b_nxt[G::RPW][S + 1];
                        const int b = i / QH, q = 2 * (i % QH);
                        const lds_float* bq[G::RPW];
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r) bq[r] = bp[r] + (b * NSLOT * WLD + q);
                        load_pair(ap + (b * TW + q), bq, true, a_nxt, b_nxt);
                        mfmas();
                        interleave();
                        rotate(a_nxt, b_nxt);
                    }
                } else {
                    int q = 0;
                    for (int i = 1; i < np; ++i) {
                        float a_nxt[2], b_nxt[G::RPW][S + 1];
                        int qn = q + 2, da = 2, db2 = 2;
                        if (qn >= q_loop) { qn = 0; da = wrap_a; db2 = wrap_b; }
                        q = qn;
                        ap += da;
#pragma unroll
                        for (int r = 0; r < G::RPW; ++r) bp[r] += db2;
                        load_pair(ap, bp, qn + 1 < q_loop, a_nxt, b_nxt);
                        mfmas();
                        rotate(a_nxt, b_nxt);
                    }
                }
            }
            // the last pair's MFMAs run behind the barrier, under the reads of the next step's first operands
            {
                float a_nxt[2], b_nxt[G::RPW][S + 1];
                __syncthreads();
                step_ptrs(u1, ap, bp);
                load_pair(ap, bp, 1 < q_loop, a_nxt, b_nxt);
                if (np) {
                    mfmas();
                    interleave();
                }
                rotate(a_nxt, b_nxt);
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

// element (k*C + c)*RS + tap of the gradient = sum over splits of partial[split][tap][k*C + c], added in split order;
// the sum goes to dw or into the SGD step (sink).  One workgroup owns 64 consecutive (k, c) pairs: thread = (pair,
// quarter of the taps) reads its taps' partials coalesced along the pairs, the sums turn through LDS, and the
// 64*RS finished elements, contiguous in the gradient, leave (or update w, v) coalesced.
template <int RS>
__global__ void __launch_bounds__(256) k_wgrad_reduce(int nsplit, int KC, const float* __restrict__ partial, GradSink sink) {
    __shared__ float turn[64 * RS];               // [64][RS]
    constexpr int NT = (RS + 3) / 4;              // taps per thread: part, part + 4, ...
    const size_t total = (size_t)RS * KC;
    const int kcl = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int kc0 = blockIdx.x * 64, kc = kc0 + kcl;
    if (kc < KC) {
        // the thread's taps side by side, eight splits per trip: 8 * NT independent loads in flight; per element the
        // even splits add up in one sum and the odd ones in another, each in split order
        float s0[NT], s1[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) s0[t] = s1[t] = 0.f;
        const float* src = partial + (size_t)part * KC + kc;
        int s = 0;
        for (; s + 7 < nsplit; s += 8) {
            float a[8][NT];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    a[u][t] = part + 4 * t < RS ? src[(size_t)(s + u) * total + (size_t)4 * t * KC] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; u += 2)
#pragma unroll
                for (int t = 0; t < NT; ++t) { s0[t] += a[u][t]; s1[t] += a[u + 1][t]; }
        }
        for (; s + 1 < nsplit; s += 2) {
            float a[NT], b[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const bool ok = part + 4 * t < RS;
                a[t] = ok ? src[(size_t)s * total + (size_t)4 * t * KC] : 0.f;
                b[t] = ok ? src[(size_t)(s + 1) * total + (size_t)4 * t * KC] : 0.f;
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) { s0[t] += a[t]; s1[t] += b[t]; }
        }
        if (s < nsplit) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (part + 4 * t < RS) s0[t] += src[(size_t)s * total + (size_t)4 * t * KC];
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
            if (part + 4 * t < RS) turn[kcl * RS + part + 4 * t] = s0[t] + s1[t];
    }
    __syncthreads();
    const int live = min(64, KC - kc0) * RS;
    if (sink.w) {
        // SGD form: all reads of w and v first (same arithmetic as sink_store)
        constexpr int IT = (64 * RS + 255) / 256;
        float wv[IT], vv[IT];
#pragma unroll
        for (int t = 0; t < IT; ++t) {
            const int j = threadIdx.x + 256 * t;
            const size_t e = (size_t)kc0 * RS + (j < live ? j : 0);
            wv[t] = sink.w[e];
            vv[t] = sink.v ? sink.v[e] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < IT; ++t) {
            const int j = threadIdx.x + 256 * t;
            if (j >= live) continue;
            const size_t e = (size_t)kc0 * RS + j;
            float vel = turn[j];
            if (sink.v) {
                vel = fmaf(sink.mu, vv[t], vel);
                sink.v[e] = vel;
            }
            const float nw = fmaf(-sink.lr, vel, wv[t]);
            sink.w[e] = nw;
            if (sink.wT) {      // the mirrored transpose-weights follow the update: wT[c][k][RS-1-t] = w[k][c][t]
                const int pair = kc0 + j / RS, tap = j % RS;
                const int k = pair / sink.wt_C, c = pair - k * sink.wt_C;
                sink.wT[((size_t)c * sink.wt_K + k) * RS + (RS - 1 - tap)] = nw;
            }
        }
        return;
    }
    for (int j = threadIdx.x; j < live; j += 256) sink.dw[(size_t)kc0 * RS + j] = turn[j];
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
    // byte offsets inside the kernel are 32-bit
    if ((size_t)s.N * s.C * s.H * s.W * sizeof(float) >= 0x7fffffffu) return false;
    if ((size_t)s.N * s.K * s.P * s.Q * sizeof(float) >= 0x7fffffffu) return false;
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
    // widths without a usable divisor (primes such as 37) would run a handful of pixels per 32-wide MFMA step over
    // dozens of column tiles, each with its own copy of dw: the implicit-GEMM weight gradient serves those
    if (best_nbi * best_tw < 16 && s.Q / best_tw > 4) return false;
    WgGeo& g = p->g;
    g.N = s.N; g.C = s.C; g.K = s.K; g.HI = s.H; g.WI = s.W; g.HO = s.P; g.WO = s.Q; g.pad = s.pad;
    g.TW = best_tw; g.NBI = best_nbi; g.WLD = best_tw + G::S - 1;
    g.XSTR = G::xstr(g.TW, g.NBI);
    g.DSTR = G::dstr(g.TW, g.NBI);
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
int launch(cnn_ctx* ctx, const Plan& p, const ConvShape& s, const float* x, const float* dy, const GradSink& sink) {
    if (ctx->ws_bytes < p.ws_bytes || !ctx->ws) return CNN_EWORKSPACE;
    static std::atomic<unsigned long long> attr_done{0};      // one bit per device: the attribute is the device's
    if (p.lds_bytes > (size_t)cnn::kMaxLdsBytes) return CNN_EUNSUPPORTED;
    {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_wgrad<G>), cnn::kMaxLdsBytes,
                                               "hipFuncSetAttribute(wgrad)");
        if (st_attr != CNN_OK) return st_attr;
    }
    float* partial = reinterpret_cast<float*>(ctx->ws);
    dim3 grid((unsigned)(p.nsplit * p.g.col_tiles), (unsigned)p.ctiles, (unsigned)p.ktiles);
    static const std::string name_s =
        G::FIXED ? strf("k_wgrad<%dx%d KW%d CW%d RW%d tw%dx%d>", G::R, G::S, G::KW, G::CW, G::RW, G::TW_CT, G::NBI_CT)
                 : strf("k_wgrad<%dx%d KW%d CW%d RW%d>", G::R, G::S, G::KW, G::CW, G::RW);
    const char* const name = name_s.c_str();
    {
        cnn::ProfScope ps(ctx, name, cnn::conv_flops(s));
        hipLaunchKernelGGL(k_wgrad<G>, grid, dim3(G::T), p.lds_bytes, ctx->stream, p.g, x, dy, partial);
    }
    int st = cnn::launch_check(ctx, "wgrad");
    if (st != CNN_OK) return st;
    const unsigned gsz = (unsigned)(((size_t)s.K * s.C + 63) / 64);
    {
        cnn::ProfScope ps(ctx, sink.w ? "k_wgrad_reduce<sgd>" : "k_wgrad_reduce", 0.0);
        hipLaunchKernelGGL(k_wgrad_reduce<G::RS>, dim3(gsz), dim3(256), 0, ctx->stream, p.nsplit * p.g.col_tiles,
                           s.K * s.C, partial, sink);
    }
    return cnn::launch_check(ctx, "wgrad_reduce");
}

// (R, S, KW, CW, RW, NSLOT): 3x3 -> 128 k x 64 c x 9 taps per workgroup (8 waves); 5x5 -> 64 k x 32 c, one kernel
// row per wave (10 waves)
using Wg3 = WgCfg<3, 3, 4, 2, 1, 4>;
using Wg5 = WgCfg<5, 5, 2, 1, 5, 8>;
// 7x7 -> 32 k x 32 c, one kernel row per wave (7 waves: 112 accumulator registers each leave no room for more
// waves per SIMD)
using Wg7 = WgCfg<7, 7, 1, 1, 7, 8>;
// 3x3 with whole tiles (C % 64 == 0, K % 128 == 0) and the step geometry (TW, NBI) of VGG-A's 112 / 56-pixel,
// 28-pixel and 14-pixel layers and of OverFeat-FAST's 12-pixel layers
using Wg3F56 = WgCfg<3, 3, 4, 2, 1, 4, 56, 1>;
using Wg3F28 = WgCfg<3, 3, 4, 2, 1, 4, 28, 2>;
using Wg3F14 = WgCfg<3, 3, 4, 2, 1, 4, 14, 4>;
using Wg3F12 = WgCfg<3, 3, 4, 2, 1, 4, 12, 4>;
// 5x5 with whole tiles and the step geometry of OverFeat-FAST's 24-pixel layer (two images per step)
using Wg5F24 = WgCfg<5, 5, 2, 1, 5, 8, 24, 2>;

}  // namespace

namespace cnn {

bool mfma_conv_bwd_weight_keeps_wt(const ConvShape& s) {
    Plan p;
    return make_plan<Wg3>(s, &p) || make_plan<Wg5>(s, &p) || make_plan<Wg7>(s, &p);    // all end in k_wgrad_reduce
}

size_t mfma_conv_bwd_weight_ws(const ConvShape& s) {
    Plan p;
    if (make_plan<Wg3>(s, &p) || make_plan<Wg5>(s, &p) || make_plan<Wg7>(s, &p)) return p.ws_bytes;
    return 0;
}

int mfma_conv_bwd_weight(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, const GradSink& dw) {
    Plan p;
    if (make_plan<Wg3>(s, &p)) {
        const int tw = p.g.TW, nbi = p.g.NBI;
        if (s.C % Wg3::CBK == 0 && s.K % Wg3::KB == 0) {
            if (tw == 56 && nbi == 1) return launch<Wg3F56>(ctx, p, s, x, dy, dw);
            if (tw == 28 && nbi == 2) return launch<Wg3F28>(ctx, p, s, x, dy, dw);
            if (tw == 14 && nbi == 4) return launch<Wg3F14>(ctx, p, s, x, dy, dw);
            if (tw == 12 && nbi == 4) return launch<Wg3F12>(ctx, p, s, x, dy, dw);
        }
        return launch<Wg3>(ctx, p, s, x, dy, dw);
    }
    if (make_plan<Wg5>(s, &p)) {
        if (s.C % Wg5::CBK == 0 && s.K % Wg5::KB == 0 && p.g.TW == 24 && p.g.NBI == 2) return launch<Wg5F24>(ctx, p, s, x, dy, dw);
        return launch<Wg5>(ctx, p, s, x, dy, dw);
    }
    if (make_plan<Wg7>(s, &p)) return launch<Wg7>(ctx, p, s, x, dy, dw);
    return CNN_EUNSUPPORTED;
}

}  // namespace cnn
