// Convolution as an implicit contraction over (channel, kernel row, kernel col) on the fp32 matrix cores of gfx950
// (v_mfma_f32_32x32x2_f32).  One kernel serves
//   forward propagation  (Section 2.1, Algorithm 1):  out = y,  in = x,  contraction over ifm (any stride)
//   backpropagation      (Section 2.1, stride 1):     out = dx, in = dy, contraction over ofm,
//                                                      kernel taps mirrored, pad' = R-1-pad
// which is the paper's remark that the passes share one loop nest and one blocking strategy.
//
// Tiling (per workgroup): MB = 32*WM output features x a pixel tile of TR full-width output rows (at most 32*NT*WN
// pixels; TR and all image sizes are run-time values).  Output rows are numbered through the whole minibatch
// (image n, row p -> n*HO + p) and a tile takes TR consecutive ones, so it continues into the next image instead of
// ending with the image: every tile but the last is full whatever the image height.  Each wave owns 32 output features x NT
// blocks of 32 pixels: NT accumulators of 16 VGPRs.  The contraction runs over chunks of CB channels:
//   LDS  wl[MB][CB*R*S + 1]      filter tile, row stride odd  -> the 32 lanes of an A operand (one output feature
//                                each) hit 32 different banks
//   LDS  xl[CB][rows][width]     input rows the tile needs, numbered through the zero-extended images (pad rows
//                                above and below each image, so consecutive output rows need consecutive staged
//                                rows also across an image boundary); zeros where the image ends; lanes of a B
//                                operand are consecutive pixels -> consecutive words.  The row stride is padded so
//                                that this also holds across the end of a row (stride 1).
// The two halves of the 64-lane wave feed k = 0 and k = 1 of the MFMA: the low half walks channels [0, CB/2) of the
// chunk and the high half [CB/2, CB), so both halves use the same offsets.
// Two LDS buffers: while chunk ch is multiplied, chunk ch+1 moves from registers into the other buffer and chunk
// ch+2 from HBM into those registers, a few staging items between the MFMA groups (no staging phase, one barrier
// per chunk).  Every instruction that is not an MFMA costs matrix-pipe time here (measured: about 1 % per dozen
// instructions in the chunk loop), so the loop is kept lean:
//  * staging loads are raw buffer loads: the address is (descriptor base) + (scalar channel offset) + (per-thread
//    byte offset computed once); positions outside the image carry an offset beyond the descriptor's range, for
//    which the hardware returns 0 - no bounds selects, no 64-bit address arithmetic;
//  * threads and filter rows beyond the tile wrap around and repeat another thread's work (same value to the same
//    LDS word, but distinct words within a wave: lanes storing to one word would be serialised);
//  * operands are read per segment of TG taps of one kernel row: the TG consecutive words of a lane come from one
//    base address (paired LDS reads), one segment ahead of the MFMAs that use them - also across the chunk barrier;
//  * the hot layer shapes get instantiations with compile-time LDS strides, so all operand offsets are immediates.
#include <stdio.h>
#include <stdlib.h>

#include "common.h"

namespace {


// epilogues: plain store; ReLU of the result; result where aux > 0 else 0 (ReLU derivative, aux = the ReLU's output);
// ReLU followed by 2x2 / stride-2 max-pooling: only the pooled result and the window position of each maximum are
// stored (the full-size activation is needed by nothing in the backward pass of conv -> ReLU -> pool)
// the reverse for backpropagation: the result is the gradient of a pooled activation (aux) whose window positions are
// known (arg): each value goes to its window's position in the full-size gradient, if the activation was > 0, and
// zeros to the window's other three positions (max-pool backward + ReLU derivative without the pooled-size round trip)
enum { EPI_NONE = 0, EPI_RELU = 1, EPI_MASK = 2, EPI_POOL = 3, EPI_UNPOOL = 4 };

// Run-time geometry of one launch (uniform across the grid).
struct ConvGeo {
    int N, J, M;                   // images, contraction channels, output features
    int HI, WI, HO, WO;            // input and output image sizes
    int pad, stride;               // padding on the input side, stride
    int TR, VH;                    // output rows per tile; rows of a zero-extended image: HI + 2*pad
    int THI, WLD;                  // staged input rows (the widest tile's) / columns: WI + 2*pad
    int WLDP, PLANEP;              // LDS row / channel strides
    int PLANE;                     // staged elements per channel: THI * WLD
    int NPIX;                      // TR * WO
    int ptiles, mtiles, per_xcd;
    // Per XCD, workgroups [0, full_per_xcd) run one (pixel tile, feature tile) unit over the whole contraction; the
    // remaining tail_per_xcd units are each cut into nsl slices of chunks_per_slice channel chunks, one workgroup per
    // slice, whose partial results go to a scratch buffer and are added up by k_tile_reduce.
    int full_per_xcd, tail_per_xcd, nsl, chunks_per_slice;
    // flat != 0 (a grid within one round whose pixel tiles do not divide evenly over the 8 XCDs): workgroup
    // blockIdx.x is slice blockIdx.x % nsl of unit blockIdx.x / nsl, units numbered (pixel tile, feature tile); the
    // hardware's round-robin then spreads them over all XCDs instead of leaving some without work.
    int flat;
    // sk_share != 0 (a grid within one round that uniform slices cannot spread evenly, e.g. 224 units on 256 compute
    // units): the chunks of all units, laid end to end, are dealt out in equal runs of sk_share chunks, one run per
    // workgroup.  A run may end one unit and begin the next; every piece goes to the scratch buffer (at most sk_pmax
    // pieces per unit, numbered by the workgroups that touch it) and k_tile_reduce adds them in that order.
    int sk_share, sk_pmax, sk_nchunks;
    int epi;
    int lds_buf;                   // elements of one (filter tile, input tile) buffer
};

// VEC = 4: filter rows are fetched as float4 (needs J % CB == 0 and 16-byte aligned rows); VEC = 1: element-wise
// fetch with the channels past J zero-filled (first layers: J = 3).  XP: input-tile positions per thread per channel.
// TG: taps per operand segment.  WLDP / PLANEP: compile-time LDS row / channel strides (0 = run-time values).
template <int R_, int S_, int CB_, int WM_, int WN_, int NT_, int VEC_, int XP_, int TG_, int WLDP_, int PLANEP_>
struct ConvCfg {
    static constexpr int R = R_, S = S_, CB = CB_, WM = WM_, WN = WN_, NT = NT_, VEC = VEC_, XP = XP_, TG = TG_;
    static constexpr int WLDP_CT = WLDP_, PLANEP_CT = PLANEP_;
    static constexpr int RS = R * S;
    static constexpr int MB = 32 * WM;
    static constexpr int NPIXB = WN * NT * 32;               // pixel capacity of a tile
    static constexpr int T = WM * WN * 64;
    static constexpr int KCH = CB * RS;                      // contraction length of one chunk
    static constexpr int WSTR = (KCH % 2 == 0) ? KCH + 1 : KCH;
    static constexpr int Q4 = KCH / VEC;                     // fetch units (float4 or float) per filter row
    static constexpr int RPP = T / Q4;                       // filter rows fetched per pass of the workgroup
    static constexpr int WSL = (MB + RPP - 1) / RPP;         // passes
    static constexpr int MAXPLANE = XP * T;                  // staged elements per channel the threads can cover
    static constexpr int SEG = (S + TG - 1) / TG;            // operand segments per kernel row
    static constexpr int NSEG = (CB / 2) * R * SEG;          // ... per chunk (each wave half walks CB/2 channels)
    static_assert(CB % 2 == 0, "the two wave halves split the chunk's channels");
    static_assert(KCH % VEC == 0 && (VEC == 1 || VEC == 4), "filter tile is fetched as float4 or float");
    static_assert(Q4 <= T, "one pass fetches at least one filter row");
};


template <class G, bool SK>
__global__ void __launch_bounds__(G::T, 2)
k_conv_tiled(ConvGeo g, const float* __restrict__ in, const float* __restrict__ wt, const float* __restrict__ aux,
             float* __restrict__ out_base, float* __restrict__ partial, unsigned char* arg_out) {
    constexpr int R = G::R, S = G::S, RS = G::RS, CB = G::CB, NT = G::NT, T = G::T, TG = G::TG;
    extern __shared__ float lds[];
    float* wl = lds;
    float* xl = lds + G::MB * G::WSTR;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm = wave % G::WM, wn = wave / G::WM;
    const int N = g.N, J = g.J, M = g.M;
    const int WLDP = G::WLDP_CT ? G::WLDP_CT : g.WLDP;
    const int PLANEP = G::PLANEP_CT ? G::PLANEP_CT : g.PLANEP;

    // Workgroups are handed to the 8 XCDs round-robin by linear id.  Give each XCD (its own L2) a contiguous range
    // of pixel tiles and run the output-feature tiles of one pixel tile back to back on it, so the input tile, and
    // the halo rows it shares with the next tile, come from HBM once instead of once per feature tile.
    // SK: this workgroup's run of chunks [sk_c0, sk_c1) of the end-to-end numbering, spanning `parts` units
    const int nchunks = (J + CB - 1) / CB;
    int sk_c0 = 0, sk_c1 = 0, sk_first = 0, parts = 1;
    if (SK) {
        const int total = g.ptiles * g.mtiles * nchunks;
        sk_c0 = blockIdx.x * g.sk_share;
        if (sk_c0 >= total) return;
        sk_c1 = min(sk_c0 + g.sk_share, total);
        sk_first = sk_c0 / nchunks;
        parts = (sk_c1 - 1) / nchunks - sk_first + 1;
    }
    for (int part = 0; part < parts; ++part) {
    int ptile, m0, slice = -1;
    size_t tix;                          // index of a sliced unit's partial tiles in the scratch buffer
    int ch_begin = 0, ch_end = nchunks;
    if (SK) {
        const int ul = sk_first + part;
        ptile = ul / g.mtiles;
        m0 = (ul % g.mtiles) * G::MB;
        tix = ul;
        ch_begin = part == 0 ? sk_c0 - ul * nchunks : 0;
        ch_end = min(sk_c1 - ul * nchunks, nchunks);
        slice = blockIdx.x - (ul * nchunks) / g.sk_share;      // this piece's number among the unit's pieces
        if (part) __syncthreads();                               // the previous unit's operands are no longer read
    } else if (g.flat) {
        const int ul = blockIdx.x / g.nsl;
        if (g.nsl > 1) slice = blockIdx.x % g.nsl;
        ptile = ul / g.mtiles;
        m0 = (ul % g.mtiles) * G::MB;
        tix = ul;
    } else {
        const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
        int unit = seq;
        if (seq >= g.full_per_xcd) {
            const int t = seq - g.full_per_xcd;
            unit = g.full_per_xcd + t / g.nsl;
            slice = t % g.nsl;
        }
        ptile = xcd * g.per_xcd + unit / g.mtiles;
        m0 = (unit % g.mtiles) * G::MB;
        tix = (size_t)xcd * g.tail_per_xcd + (unit - g.full_per_xcd);
    }
    if (ptile >= g.ptiles) return;   // whole workgroup leaves: no barrier is left behind
    const int row0 = ptile * g.TR, nrows = N * g.HO;      // first output row of the tile, rows of the minibatch
    const int n0 = row0 / g.HO;                           // image the tile starts in
    const int v0 = n0 * g.VH + (row0 % g.HO) * g.stride;  // its first staged row, numbered through the extended images

    const int plane_g = g.HI * g.WI;
    const size_t in_img = (size_t)J * plane_g;         // elements per image of `in`
    // descriptors: the input from the tile's first image to the end of the tensor, and the whole filter tensor
    // (the planner keeps every offset used below 2^31 bytes)
    const size_t in_left = (size_t)(N - n0) * in_img * sizeof(float);
    const __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(in + (size_t)n0 * in_img), 0, in_left > 0x7fffffffu ? 0x7fffffff : (int)in_left, kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(wt), 0, (int)((size_t)M * J * RS * sizeof(float)), kRsrcWord3);

    // ---- input tile staging: each thread owns XP positions of the (image, row, col) plane and fetches them for
    //      every channel of the chunk: byte offset within one channel (or kOutOfRange) and LDS position
    int xvo[G::XP], xpos[G::XP];
#pragma unroll
    for (int j = 0; j < G::XP; ++j) {
        const int e = (tid + j * T) % g.PLANE;     // positions past the plane wrap around: distinct words per lane
        const int row = e / g.WLD, col = e % g.WLD;
        const int va = v0 + row, nb = va / g.VH - n0;         // image relative to the tile's first
        const int h = va % g.VH - g.pad, w = col - g.pad;
        xpos[j] = row * WLDP + col;
        const bool ok = n0 + nb < N && h >= 0 && h < g.HI && w >= 0 && w < g.WI;
        xvo[j] = ok ? (int)((nb * (int)in_img + h * g.WI + w) * sizeof(float)) : kOutOfRange;
    }
    // ---- filter tile staging: thread = (row m_sub, fetch unit kq) of a pass over RPP rows
    const int wtid = tid % (G::RPP * G::Q4);
    const int w_msub = wtid / G::Q4, w_kq = wtid % G::Q4;
    int wvo[G::WSL], wpos[G::WSL];
#pragma unroll
    for (int i = 0; i < G::WSL; ++i) {
        const int m = (w_msub + i * G::RPP) % G::MB;
        const int mrow = min(m0 + m, M - 1);          // rows past M repeat the last one (their results are not stored)
        wvo[i] = (int)((mrow * J * RS + w_kq * G::VEC) * sizeof(float));
        if (G::VEC == 1 && w_kq >= J * RS) wvo[i] = kOutOfRange;     // J < CB: one chunk, its missing channels are zero
        wpos[i] = m * G::WSTR + w_kq * G::VEC;
    }

    // ---- per-lane LDS read bases
    const int a_base = (wm * 32 + l32) * G::WSTR + half * (CB / 2) * RS;
    int b_base[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = (wn * NT + j) * 32 + l32;
        int o = 0;
        const int orow = row0 + i / g.WO;
        if (i < g.NPIX && orow < nrows)
            o = ((orow / g.HO) * g.VH + (orow % g.HO) * g.stride - v0) * WLDP + (i % g.WO) * g.stride;
        b_base[j] = o + half * (CB / 2) * PLANEP;
    }

    f32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    float xr[CB][G::XP];
    float4 wr[G::WSL];

    // Staging is cut into items (one input-tile register or one filter-tile fetch unit each) so that it can be
    // spread over the MFMA groups of a chunk instead of forming a phase of its own.
    constexpr int NX = CB * G::XP, NITEMS = NX + G::WSL;
    auto fetch_item = [&](int it, int c0) {
        if (it < NX) {
            const int c = it / G::XP, j = it % G::XP;
            const int vo = (G::VEC == 4 || c0 + c < J) ? xvo[j] : kOutOfRange;     // channels past J are zero
            xr[c][j] = __builtin_bit_cast(
                float, __builtin_amdgcn_raw_buffer_load_b32(rs_in, vo, (c0 + c) * plane_g * (int)sizeof(float), 0));
        } else {
            // w[m][c0 .. c0+CB)[R][S]: CB*R*S contiguous floats per output feature
            const int i = it - NX;
            if (G::VEC == 4)
                wr[i] = __builtin_bit_cast(
                    float4, __builtin_amdgcn_raw_buffer_load_b128(rs_w, wvo[i], c0 * RS * (int)sizeof(float), 0));
            else
                wr[i].x = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_w, wvo[i], 0, 0));
        }
    };
    // LDS addresses are kept in registers as 32-bit pointers and moved to the other buffer once per chunk; everything
    // else is an immediate offset.  (Left to itself the compiler recomputes them for every segment.)
    lds_float* xw[G::XP];                       // staging destinations, channel 0 of the chunk
    lds_float* ww[G::WSL];
    const lds_float* bp[CB / 2][NT];            // B operand bases per channel of this wave half
    const lds_float* ap;                        // A operand base
#pragma unroll
    for (int j = 0; j < G::XP; ++j) xw[j] = (lds_float*)(xl + xpos[j]);
#pragma unroll
    for (int i = 0; i < G::WSL; ++i) ww[i] = (lds_float*)(wl + wpos[i]);
#pragma unroll
    for (int cc = 0; cc < CB / 2; ++cc)
#pragma unroll
        for (int j = 0; j < NT; ++j) bp[cc][j] = (const lds_float*)(xl + b_base[j] + cc * PLANEP);
    ap = (const lds_float*)(wl + a_base);
    // wdelta = +-(elements of one buffer): the staging pointers move by it, the operand pointers the other way
    auto flip = [&](int wdelta) {
#pragma unroll
        for (int j = 0; j < G::XP; ++j) { xw[j] += wdelta; asm volatile("" : "+v"(xw[j])); }
#pragma unroll
        for (int i = 0; i < G::WSL; ++i) { ww[i] += wdelta; asm volatile("" : "+v"(ww[i])); }
#pragma unroll
        for (int cc = 0; cc < CB / 2; ++cc)
#pragma unroll
            for (int j = 0; j < NT; ++j) { bp[cc][j] -= wdelta; asm volatile("" : "+v"(bp[cc][j])); }
        ap -= wdelta;
        asm volatile("" : "+v"(ap));
    };

    auto stage_item = [&](int it) {
        if (it < NX) {
            const int c = it / G::XP, j = it % G::XP;
            xw[j][c * PLANEP] = xr[c][j];
        } else {
            const int i = it - NX;
            ww[i][0] = wr[i].x;
            if (G::VEC == 4) { ww[i][1] = wr[i].y; ww[i][2] = wr[i].z; ww[i][3] = wr[i].w; }
        }
    };

    // Operands of segment `seg` of a chunk: TG (or fewer, at the end of a kernel row) taps of one (channel, kernel
    // row): a[t] for this lane's output feature, b[j][t] for its pixel of block j.
    auto read_seg = [&](int seg, float (&a)[TG], float (&b)[NT][TG]) {
        const int cc = seg / (R * G::SEG), r = (seg / G::SEG) % R, s0 = (seg % G::SEG) * TG;
        const int len = TG < S - s0 ? TG : S - s0;
#pragma unroll
        for (int t = 0; t < len; ++t) a[t] = ap[cc * RS + r * S + s0 + t];
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int t = 0; t < len; ++t) b[j][t] = bp[cc][j][r * WLDP + s0 + t];
    };

    // Two LDS buffers.  While chunk ch is multiplied out of buffer ch&1, chunk ch+1 goes from registers into the
    // other buffer and chunk ch+2 from HBM into those registers, item by item between the MFMA groups.  One barrier
    // per chunk, placed before the MFMAs of the chunk's last segment: the first operands of the next chunk are read
    // behind it while those MFMAs run.  The last iterations stage and fetch a clamped chunk again instead of
    // branching (harmless: that buffer is never read for results), which keeps the chunk body one basic block.
    // A tail workgroup (slice >= 0) covers only its slice of the contraction and writes a partial tile.
    if (!SK && slice >= 0) {
        ch_begin = slice * g.chunks_per_slice;
        ch_end = min(ch_begin + g.chunks_per_slice, nchunks);
    }
    const size_t out_plane = (size_t)g.HO * g.WO;
    constexpr int NSEG = G::NSEG, IPS = (NITEMS + NSEG - 1) / NSEG;
    // fewer channels than one chunk (VEC == 1: first layers): the whole contraction is this one chunk, nothing is
    // staged ahead
    constexpr bool SINGLE = G::VEC == 1;
#pragma unroll
    for (int it = 0; it < NITEMS; ++it) fetch_item(it, ch_begin * CB);
#pragma unroll
    for (int it = 0; it < NITEMS; ++it) stage_item(it);
    if (!SINGLE) {
        const int c1 = min(ch_begin + 1, ch_end - 1) * CB;
#pragma unroll
        for (int it = 0; it < NITEMS; ++it) fetch_item(it, c1);
    }
    __syncthreads();
    float a_cur[TG] = {}, b_cur[NT][TG] = {};
    read_seg(0, a_cur, b_cur);
    // from here on: reads from buffer (ch - ch_begin) & 1, staging writes to the other one
#pragma unroll
    for (int j = 0; j < G::XP; ++j) xw[j] += g.lds_buf;
#pragma unroll
    for (int i = 0; i < G::WSL; ++i) ww[i] += g.lds_buf;
    // A wave whose 32 output features all lie past M (the last feature tile of a ragged M) only takes part in the
    // staging and the barriers: its MFMAs would be discarded, and skipping them leaves the matrix pipe to the waves
    // that share its SIMD.
    const bool wave_live = __builtin_amdgcn_readfirstlane(m0 + wm * 32) < M;
    if (!wave_live) {
        for (int ch = ch_begin; ch < ch_end; ++ch) {
            const int c2 = min(ch + 2, ch_end - 1) * CB;
            const int wdelta = ((ch - ch_begin) & 1) ? g.lds_buf : -g.lds_buf;
            if (!SINGLE) {
#pragma unroll
                for (int it = 0; it < NITEMS; ++it) {
                    stage_item(it);
                    fetch_item(it, c2);
                }
                __syncthreads();
                flip(wdelta);
            }
        }
    }
    for (int ch = ch_begin; wave_live && ch < ch_end; ++ch) {
        const int c2 = min(ch + 2, ch_end - 1) * CB;      // the staging registers hold chunk min(ch + 1, ch_end - 1)
        const int wdelta = ((ch - ch_begin) & 1) ? g.lds_buf : -g.lds_buf;   // where the write pointers go next
#pragma unroll
        for (int seg = 0; seg < NSEG; ++seg) {
#pragma unroll
            for (int u = 0; u < IPS; ++u) {
                const int it = seg * IPS + u;
                if (it < NITEMS && !SINGLE) {
                    stage_item(it);
                    fetch_item(it, c2);
                }
            }
            float a_nxt[TG] = {}, b_nxt[NT][TG] = {};
            if (seg + 1 < NSEG) {
                read_seg(seg + 1, a_nxt, b_nxt);
            } else if (!SINGLE) {
                __syncthreads();
                flip(wdelta);
                read_seg(0, a_nxt, b_nxt);
            }
            const int s0 = (seg % G::SEG) * TG, len = TG < S - s0 ? TG : S - s0;
#pragma unroll
            for (int t = 0; t < len; ++t)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[t], b_cur[j][t], acc[j], 0, 0, 0);
            // issue order inside the segment: one MFMA, then one of the next segment's LDS reads, and so on, so the
            // reads complete under the remaining MFMAs instead of being exposed at the start of the next segment;
            // the scheduling barrier keeps the staging items from being regrouped across segments
#pragma unroll
            for (int k = 0; k < NT * len; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 DS read
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < TG; ++t) {
                a_cur[t] = a_nxt[t];
#pragma unroll
                for (int j = 0; j < NT; ++j) b_cur[j][t] = b_nxt[j][t];
            }
        }
    }

    // ---- epilogue: lane = pixel (coalesced along the row), register v = output feature
    if (SK || slice >= 0) {              // (SK: every piece is partial; the other epilogues are compiled out)
        // partial tile [MB][NPIXB] of tail unit (xcd, unit - full_per_xcd), slice `slice`; no guards: the scratch
        // buffer holds whole tiles and the reduction skips what lies outside the tensor
        float* po = partial + (tix * (SK ? g.sk_pmax : g.nsl) + slice) * (size_t)(G::MB * G::NPIXB);
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int i = (wn * NT + j) * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                po[(size_t)m * G::NPIXB + i] = acc[j][v];
            }
        }
        if (SK) continue;                // on to the piece of the next unit
        return;
    }
    if (g.epi == EPI_POOL) {
        // ReLU + 2x2 max-pool.  The tile holds whole row pairs (TR, HO, WO even).  Step 1, in registers: a lane and
        // its neighbour (pixels q, q+1 of one row) exchange values; the even lane keeps the larger one and which it
        // was, packed into the sign bit (the values are >= 0 after the ReLU).  Step 2: through LDS (free after the
        // chunk loop; `hl[feature][pixel pair]`), the row pair is combined and the pooled value and the window
        // position (row-major, first maximum wins) go to HBM.
        float* hl = lds;
        const int hw = g.NPIX / 2;
        __syncthreads();                       // every wave is done with the operand buffers
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int i = (wn * NT + j) * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float val = acc[j][v] > 0.f ? acc[j][v] : 0.f;
                const float other = __builtin_bit_cast(
                    float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, val), 0xB1, 0xF, 0xF, true));   // lane ^ 1
                const bool right = other > val;                               // even lane: `other` is the pixel to the right
                const float hmax = right ? other : val;
                acc[j][v] = __builtin_bit_cast(float, __builtin_bit_cast(unsigned, hmax) | (right ? 0x80000000u : 0u));
            }
            if ((lane & 1) == 0 && i < g.NPIX) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    hl[m * hw + i / 2] = acc[j][v];
                }
            }
        }
        __syncthreads();
        // pooled pixels of the tile, the same for every feature: (TR/2) x (WO/2), one or two per lane
        const int pw = g.WO / 2, per_m = (g.TR / 2) * pw, php = g.HO / 2;
        constexpr int PPL = (G::NPIXB / 4 + 63) / 64;
        int src[PPL];
        size_t dst[PPL];
        bool ok[PPL];
#pragma unroll
        for (int t = 0; t < PPL; ++t) {
            const int e = lane + 64 * t, pr = e / pw, pq = e % pw;
            const int orow = row0 + 2 * pr;
            ok[t] = e < per_m && orow < nrows;
            src[t] = 2 * pr * pw + pq;
            dst[t] = ((size_t)(orow / g.HO) * M * php + (orow % g.HO) / 2) * pw + pq;
        }
        for (int m = wave; m < G::MB && m0 + m < M; m += T / 64) {
#pragma unroll
            for (int t = 0; t < PPL; ++t) {
                if (!ok[t]) continue;
                const float top = hl[m * hw + src[t]], bot = hl[m * hw + src[t] + pw];
                const float vt = __builtin_fabsf(top), vb = __builtin_fabsf(bot);
                const bool lower = vb > vt;
                const unsigned bits = __builtin_bit_cast(unsigned, lower ? bot : top);
                const size_t o = dst[t] + (size_t)(m0 + m) * php * pw;
                out_base[o] = lower ? vb : vt;
                arg_out[o] = (unsigned char)((lower ? 2u : 0u) + (bits >> 31));
            }
        }
        return;
    }
    // The epilogues that read a second tensor issue all 16 reads of a 32x32 block before its first store, without
    // branches (lanes and features outside the tensor read a clamped, valid address): one trip to memory per block
    // instead of one per element.
    if (g.epi == EPI_UNPOOL) {
        // lane = pixel (p, q) of the pooled map: its 2x2 window of the full-size gradient is written as two float2,
        // consecutive lanes writing consecutive 8-byte pairs of rows 2p and 2p+1
        typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int i = (wn * NT + j) * 32 + l32;
            const int orow = row0 + i / g.WO;
            const bool ok = i < g.NPIX && orow < nrows;
            const int n = ok ? orow / g.HO : 0, p = ok ? orow % g.HO : 0, q = ok ? i % g.WO : 0;
            const size_t o0 = ((size_t)n * M) * out_plane + (size_t)p * g.WO + q;
            const size_t f0 = ((size_t)n * M) * 4 * out_plane + (size_t)(2 * p) * (2 * g.WO) + 2 * q;
            float act[16];
            int pos[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                const size_t o = o0 + (size_t)(m < M ? m : M - 1) * out_plane;
                act[v] = aux[o];
                pos[v] = arg_out[o];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (ok && m < M) {
                    const float r = act[v] > 0.f ? acc[j][v] : 0.f;
                    f32x2* d = reinterpret_cast<f32x2*>(out_base + f0 + (size_t)m * 4 * out_plane);
                    f32x2 top, bot;
                    top.x = pos[v] == 0 ? r : 0.f; top.y = pos[v] == 1 ? r : 0.f;
                    bot.x = pos[v] == 2 ? r : 0.f; bot.y = pos[v] == 3 ? r : 0.f;
                    d[0] = top;
                    d[g.WO] = bot;        // next row of the full-size map: 2*WO floats = WO pairs further
                }
            }
        }
        return;
    }
    if (g.epi == EPI_MASK) {
        // fused ReLU derivative: the gradient passes where the forward activation was positive
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int i = (wn * NT + j) * 32 + l32;
            const int orow = row0 + i / g.WO;
            const bool ok = i < g.NPIX && orow < nrows;
            const size_t o0 = ok ? ((size_t)(orow / g.HO) * M) * out_plane + (size_t)(orow % g.HO) * g.WO + i % g.WO : 0;
            float act[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                act[v] = aux[o0 + (size_t)(m < M ? m : M - 1) * out_plane];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (ok && m < M) out_base[o0 + (size_t)m * out_plane] = act[v] > 0.f ? acc[j][v] : 0.f;
            }
        }
        return;
    }
    float* out = out_base;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int i = (wn * NT + j) * 32 + l32;
        const int orow = row0 + i / g.WO;
        if (i >= g.NPIX || orow >= nrows) continue;
        const size_t o0 = ((size_t)(orow / g.HO) * M) * out_plane + (size_t)(orow % g.HO) * g.WO + i % g.WO;
        float* o = out + o0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = m0 + wm * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (m < M) {
                float r = acc[j][v];
                if (g.epi == EPI_RELU) r = r > 0.f ? r : 0.f;                                      // fused ReLU
                o[(size_t)m * out_plane] = r;
            }
        }
    }
    }   // pieces (one pass unless SK; an SK piece never gets here: it leaves through the partial-tile store)
}

// wT[c][k][r][s] = w[k][c][R-1-r][S-1-s]: the "transpose-weights" of Section 2.3 with the taps mirrored, so that
// backpropagation is a forward convolution of dy with wT.  One workgroup moves a tk(k) x 32(c) block through LDS;
// the reads (32*RS contiguous floats per k) are coalesced, the writes are runs of tk*RS floats per c.
__global__ void __launch_bounds__(256) k_transpose_flip(int K, int C, int RS, int tk, const float* __restrict__ w,
                                                       float* __restrict__ wT) {
    extern __shared__ float tl[];               // [tk][32*RS + 1]
    const int k0 = blockIdx.x * tk, c0 = blockIdx.y * 32;
    const int row = 32 * RS, str = row + 1;
    const int cn = min(32, C - c0), kn = min(tk, K - k0);
    for (int e = threadIdx.x; e < tk * row; e += 256) {
        const int k = e / row, o = e % row;
        if (k < kn && o < cn * RS) tl[k * str + o] = w[((size_t)(k0 + k) * C + c0) * RS + o];
    }
    __syncthreads();
    const int orow = tk * RS;
    for (int e = threadIdx.x; e < 32 * orow; e += 256) {
        const int c = e / orow, o = e % orow, k = o / RS, t = o % RS;
        if (c < cn && k < kn) wT[((size_t)(c0 + c) * K + k0) * RS + o] = tl[k * str + c * RS + (RS - 1 - t)];
    }
}
// features per block (measured on 512 x 512 x 3 x 3: 2 / 4 / 8 / 16 / 32 -> 12.5 / 11.7 / 12.9 / 17.7 / 31 us: small
// blocks, many workgroups)
inline int transpose_tk(int) { return 4; }

// Adds up the slices of every tail unit in slice order and stores the tile with the epilogue applied.
// grid = (tail units, MB / 8): one block owns 8 feature rows of one tile.
// sum over the slices' partial tiles of one element, in slice order; four reads in flight at a time
__device__ __forceinline__ float slice_sum(const float* __restrict__ p, size_t tile, int nsl) {
    float r = 0.f;
    int s = 0;
    for (; s + 3 < nsl; s += 4) {
        const float a0 = p[(size_t)s * tile], a1 = p[(size_t)(s + 1) * tile], a2 = p[(size_t)(s + 2) * tile],
                    a3 = p[(size_t)(s + 3) * tile];
        r = (((r + a0) + a1) + a2) + a3;
    }
    for (; s < nsl; ++s) r += p[(size_t)s * tile];
    return r;
}

__global__ void __launch_bounds__(256) k_tile_reduce(ConvGeo g, int MB, int cap, int kRedF, const float* __restrict__ partial,
                                                    const float* __restrict__ aux, float* __restrict__ out,
                                                    unsigned char* arg_out) {
    int ptile, m0;
    if (g.flat) {
        ptile = blockIdx.x / g.mtiles;
        m0 = (blockIdx.x % g.mtiles) * MB;
    } else {
        const int xcd = blockIdx.x / g.tail_per_xcd, unit = g.full_per_xcd + blockIdx.x % g.tail_per_xcd;
        ptile = xcd * g.per_xcd + unit / g.mtiles;
        m0 = (unit % g.mtiles) * MB;
    }
    if (ptile >= g.ptiles) return;
    const int row0 = ptile * g.TR, nrows = g.N * g.HO;
    const size_t out_plane = (size_t)g.HO * g.WO, tile = (size_t)MB * cap;
    const float* pt = partial + (size_t)blockIdx.x * g.nsl * tile;
    int nsl = g.nsl;
    if (g.sk_share) {
        // the pieces of unit blockIdx.x: one per workgroup whose run of chunks touches it
        const int u = blockIdx.x;
        nsl = ((u + 1) * g.sk_nchunks - 1) / g.sk_share - (u * g.sk_nchunks) / g.sk_share + 1;
        pt = partial + (size_t)u * g.sk_pmax * tile;
    }
    if (g.epi == EPI_POOL) {
        // ReLU + 2x2 max-pool of the summed tile: one thread per pooled element (window order: row-major, first
        // maximum wins, as in the stand-alone pooling kernel)
        const int pw = g.WO / 2, per_m = (g.TR / 2) * pw, php = g.HO / 2;
        for (int e = threadIdx.x; e < kRedF * per_m; e += 256) {
            const int ml = blockIdx.y * kRedF + e / per_m, rem = e % per_m, pr = rem / pw, pq = rem % pw;
            const int orow = row0 + 2 * pr;
            if (orow >= nrows || m0 + ml >= g.M) continue;
            float best = 0.f;
            int idx = 0;
            for (int w4 = 0; w4 < 4; ++w4) {
                const int i = (2 * pr + w4 / 2) * g.WO + 2 * pq + (w4 & 1);
                float r = slice_sum(pt + (size_t)ml * cap + i, tile, nsl);
                r = r > 0.f ? r : 0.f;
                if (w4 == 0 || r > best) { best = r; idx = w4; }
            }
            const size_t o = (((size_t)(orow / g.HO) * g.M + m0 + ml) * php + (orow % g.HO) / 2) * pw + pq;
            out[o] = best;
            arg_out[o] = (unsigned char)idx;
        }
        return;
    }
    if (out_plane % 4 == 0 && g.NPIX % 4 == 0 && (g.epi != EPI_UNPOOL || g.WO % 2 == 0)) {
        // four consecutive pixels of a tile are four consecutive, 16-byte aligned elements of one output plane
        // (tiles and images start at multiples of four pixels): everything moves as float4; same order of additions
        typedef float f4 __attribute__((ext_vector_type(4)));
        const int c4 = cap / 4;
        const size_t lin0 = (size_t)row0 * g.WO, lin_end = (size_t)nrows * g.WO;
        for (int e = threadIdx.x; e < kRedF * c4; e += 256) {
            const int ml = blockIdx.y * kRedF + e / c4, i = (e % c4) * 4;
            if (i >= g.NPIX || lin0 + i >= lin_end || m0 + ml >= g.M) continue;
            const float* ps = pt + (size_t)ml * cap + i;
            f4 r = *reinterpret_cast<const f4*>(ps);
            if (nsl == 2) {
                r += *reinterpret_cast<const f4*>(ps + tile);
            } else if (nsl == 3) {
                const f4 a1 = *reinterpret_cast<const f4*>(ps + tile), a2 = *reinterpret_cast<const f4*>(ps + 2 * tile);
                r = (r + a1) + a2;
            } else {
                for (int sl = 1; sl < nsl; ++sl) r += *reinterpret_cast<const f4*>(ps + (size_t)sl * tile);
            }
            const size_t lin = lin0 + i, plane = (lin / out_plane) * g.M + m0 + ml, rem = lin % out_plane;
            const size_t o = plane * out_plane + rem;
            if (g.epi == EPI_UNPOOL) {
                const f4 a = *reinterpret_cast<const f4*>(aux + o);
                const int ps4[4] = {arg_out[o], arg_out[o + 1], arg_out[o + 2], arg_out[o + 3]};
                // two pixel pairs, each inside one row (even width): a pair's two windows are eight consecutive
                // floats, four in each of two rows of the full-size gradient
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const size_t q = rem + 2 * h;
                    const float v0 = a[2 * h] > 0.f ? r[2 * h] : 0.f, v1 = a[2 * h + 1] > 0.f ? r[2 * h + 1] : 0.f;
                    const int p0 = ps4[2 * h], p1 = ps4[2 * h + 1];
                    float* d = out + plane * 4 * out_plane + (q / g.WO) * (size_t)(4 * g.WO) + 2 * (q % g.WO);
                    f4 top, bot;
                    top[0] = p0 == 0 ? v0 : 0.f; top[1] = p0 == 1 ? v0 : 0.f; top[2] = p1 == 0 ? v1 : 0.f; top[3] = p1 == 1 ? v1 : 0.f;
                    bot[0] = p0 == 2 ? v0 : 0.f; bot[1] = p0 == 3 ? v0 : 0.f; bot[2] = p1 == 2 ? v1 : 0.f; bot[3] = p1 == 3 ? v1 : 0.f;
                    *reinterpret_cast<f4*>(d) = top;
                    *reinterpret_cast<f4*>(d + 2 * g.WO) = bot;
                }
                continue;
            }
            if (g.epi == EPI_RELU) {
#pragma unroll
                for (int t = 0; t < 4; ++t) r[t] = r[t] > 0.f ? r[t] : 0.f;
            } else if (g.epi == EPI_MASK) {
                const f4 a = *reinterpret_cast<const f4*>(aux + o);
#pragma unroll
                for (int t = 0; t < 4; ++t) r[t] = a[t] > 0.f ? r[t] : 0.f;
            }
            *reinterpret_cast<f4*>(out + o) = r;
        }
        return;
    }
    for (int e = threadIdx.x; e < kRedF * cap; e += 256) {
        const int ml = blockIdx.y * kRedF + e / cap, i = e % cap;
        const int orow = row0 + i / g.WO;
        if (i >= g.NPIX || orow >= nrows || m0 + ml >= g.M) continue;
        float r = slice_sum(pt + (size_t)ml * cap + i, tile, nsl);
        if (g.epi == EPI_UNPOOL) {
            const size_t plane = (size_t)(orow / g.HO) * g.M + m0 + ml;
            const size_t o = plane * out_plane + (size_t)(orow % g.HO) * g.WO + i % g.WO;
            r = aux[o] > 0.f ? r : 0.f;
            const int pos = arg_out[o];
            float* d = out + plane * 4 * out_plane + (size_t)(2 * (orow % g.HO)) * (2 * g.WO) + 2 * (i % g.WO);
            d[0] = pos == 0 ? r : 0.f; d[1] = pos == 1 ? r : 0.f;
            d[2 * g.WO] = pos == 2 ? r : 0.f; d[2 * g.WO + 1] = pos == 3 ? r : 0.f;
            continue;
        }
        const size_t o = ((size_t)(orow / g.HO) * g.M + m0 + ml) * out_plane + (size_t)(orow % g.HO) * g.WO + i % g.WO;
        if (g.epi == EPI_RELU) r = r > 0.f ? r : 0.f;
        else if (g.epi == EPI_MASK) r = aux[o] > 0.f ? r : 0.f;
        out[o] = r;
    }
}

struct LaunchArgs {
    ConvGeo g;
    size_t lds_bytes;
    const float *in, *wt, *aux;
    float *out, *partial;
    unsigned char* arg;
};
typedef int (*LaunchFn)(cnn_ctx*, const LaunchArgs&);

template <class G>
int launch(cnn_ctx* ctx, const LaunchArgs& a) {
    constexpr bool kHasSK = G::R == 3 && G::VEC == 4 && G::WM == 4;      // instantiations the planner may run this way
    // the plans differ in their LDS need: the limit is raised to the whole LDS once per device
    static std::atomic<unsigned long long> attr_done{0}, attr_done_sk{0};
    if (a.lds_bytes > (size_t)cnn::kMaxLdsBytes) return CNN_EUNSUPPORTED;
    {
        int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_conv_tiled<G, false>), cnn::kMaxLdsBytes,
                                         "hipFuncSetAttribute(conv_tiled)");
        if (st_attr == CNN_OK && kHasSK)
            st_attr = cnn::lds_attr_once(ctx, attr_done_sk, reinterpret_cast<const void*>(&k_conv_tiled<G, kHasSK>), cnn::kMaxLdsBytes,
                                         "hipFuncSetAttribute(conv_tiled runs)");
        if (st_attr != CNN_OK) return st_attr;
    }
    dim3 grid((unsigned)(a.g.flat ? a.g.ptiles * a.g.mtiles * a.g.nsl : 8 * (a.g.full_per_xcd + a.g.tail_per_xcd * a.g.nsl)));
    if (a.g.sk_share) {
        if (!kHasSK) return CNN_EUNSUPPORTED;
        const long total = (long)a.g.ptiles * a.g.mtiles * a.g.sk_nchunks;
        grid = dim3((unsigned)((total + a.g.sk_share - 1) / a.g.sk_share));
    }
    static const std::string name_s =
        G::WLDP_CT ? strf("k_conv_tiled<%dx%d CB%d WM%d WN%d NT%d ld%d/%d>", G::R, G::S, G::CB, G::WM, G::WN, G::NT,
                          G::WLDP_CT, G::PLANEP_CT)
                   : strf("k_conv_tiled<%dx%d CB%d WM%d WN%d NT%d%s>", G::R, G::S, G::CB, G::WM, G::WN, G::NT,
                          G::VEC == 1 ? " v1" : "");
    static const std::string name_sk_s = name_s + " runs";
    const char* const name = name_s.c_str();
    const char* const name_sk = name_sk_s.c_str();
    {
        cnn::ProfScope ps(ctx, a.g.sk_share ? name_sk : name, 2.0 * a.g.N * a.g.J * a.g.M * G::RS * a.g.HO * a.g.WO);
        if (kHasSK && a.g.sk_share)
            hipLaunchKernelGGL((k_conv_tiled<G, kHasSK>), grid, dim3(G::T), a.lds_bytes, ctx->stream, a.g, a.in, a.wt, a.aux,
                               a.out, a.partial, a.arg);
        else
            hipLaunchKernelGGL((k_conv_tiled<G, false>), grid, dim3(G::T), a.lds_bytes, ctx->stream, a.g, a.in, a.wt, a.aux,
                               a.out, a.partial, a.arg);
    }
    return cnn::launch_check(ctx, "conv_tiled");
}

// Instantiations: one per (kernel size, tile shape, LDS strides).  `mb`, `wn`, `nt`: features per tile, wave columns,
// pixel blocks per wave; `maxplane`: staged input elements per channel the workgroup's threads can cover; `wldp`,
// `planep`: the LDS strides the instantiation is compiled for (0: any, taken from the launch geometry).
struct Variant {
    int R, S, CB, vec, mb, wn, nt, threads, maxplane, wstr, wldp, planep;
    LaunchFn fn;
};
#define V(R_, S_, CB_, WM_, WN_, NT_, VEC_, XP_, TG_, WLDP_, PLANEP_)                                              \
    {R_, S_, CB_, VEC_, 32 * WM_, WN_, NT_, 64 * WM_ * WN_,                                                        \
     ConvCfg<R_, S_, CB_, WM_, WN_, NT_, VEC_, XP_, TG_, WLDP_, PLANEP_>::MAXPLANE,                                \
     ConvCfg<R_, S_, CB_, WM_, WN_, NT_, VEC_, XP_, TG_, WLDP_, PLANEP_>::WSTR, WLDP_, PLANEP_,                    \
     launch<ConvCfg<R_, S_, CB_, WM_, WN_, NT_, VEC_, XP_, TG_, WLDP_, PLANEP_>>}
const Variant kVariants[] = {
    // 3x3, 128-feature tiles (4 waves), strides of the 3x3 / pad 1 layers of VGG-A at 112, 56, 28 and 14 pixels and
    // of OverFeat-FAST at 12 pixels (both passes share them: backpropagation has pad' = 1 too)
    V(3, 3, 4, 4, 1, 7, 4, 2, 3, 144, 576), V(3, 3, 4, 4, 1, 7, 4, 2, 3, 88, 528), V(3, 3, 4, 4, 1, 7, 4, 2, 3, 60, 720),
    V(3, 3, 4, 4, 1, 7, 4, 2, 3, 46, 920), V(3, 3, 4, 4, 1, 9, 4, 2, 1, 44, 1232),
    // ... and the 64-feature tile at 112 pixels (backpropagation into a 64-channel layer)
    V(3, 3, 4, 2, 1, 7, 4, 4, 3, 144, 576),
    // 3x3, any strides: 128-feature tiles (4 waves) and 64-feature tiles (2 waves), 7 / 8 / 9 pixel blocks per wave
    V(3, 3, 4, 4, 1, 7, 4, 2, 3, 0, 0), V(3, 3, 4, 4, 1, 8, 4, 2, 1, 0, 0), V(3, 3, 4, 4, 1, 9, 4, 2, 1, 0, 0),
    V(3, 3, 4, 2, 1, 7, 4, 4, 3, 0, 0), V(3, 3, 4, 2, 1, 8, 4, 4, 1, 0, 0),
    // 64 features x two wave columns: four waves for grids of at most one workgroup per compute unit, where a
    // two-wave workgroup leaves half the SIMDs idle (small minibatches)
    V(3, 3, 4, 2, 2, 4, 4, 4, 3, 0, 0),
    // 3x3 with fewer than 4 contraction channels (first layers)
    V(3, 3, 4, 2, 2, 7, 1, 4, 1, 0, 0),
    // 5x5: 64-feature tiles, two wave columns
    V(5, 5, 4, 2, 2, 3, 4, 4, 2, 0, 0), V(5, 5, 4, 2, 2, 4, 4, 4, 2, 0, 0), V(5, 5, 4, 2, 2, 7, 4, 4, 2, 0, 0),
    // 5x5: 32-feature tiles, four wave columns (feature counts that are odd multiples of 32: 96-feature backpropagation)
    V(5, 5, 4, 1, 4, 5, 4, 4, 2, 0, 0),
    // 7x7: 64-feature tiles, two wave columns; and with fewer than 4 contraction channels (strided first layers:
    // up to 12 staged positions per thread and channel for the tall input tile a stride-2 pixel tile needs)
    V(7, 7, 4, 2, 2, 3, 4, 4, 2, 0, 0), V(7, 7, 4, 2, 2, 4, 4, 4, 2, 0, 0),
    V(7, 7, 4, 2, 2, 7, 1, 12, 1, 0, 0),
};
#undef V

struct ConvPlan {
    const Variant* v;
    ConvGeo g;
    size_t lds_bytes, partial_bytes;
    int reduce_units;                  // units whose partial tiles k_tile_reduce adds up (0: none)
};


// Chooses, among the instantiations for this kernel size, the pixel tile (TR consecutive output rows of the whole
// minibatch) that wastes the fewest MFMA lanes, prefers the 128-feature tile unless the layer has at most 64 output
// features, and slices the contraction of the tail units (below).
// pool: the plan is for the ReLU + 2x2 max-pool epilogue (whole row pairs per tile, LDS room for the exchange).
bool make_plan(int R, int S, int pad, int stride, int N, int J, int M, int HI, int WI, ConvPlan* p, bool pool = false) {
    if (HI + 2 * pad < R || WI + 2 * pad < S) return false;
    // byte offsets inside the kernel are 32-bit: the filter tensor, and (below) the images one pixel tile touches
    if ((size_t)M * J * R * S * sizeof(float) >= 0x7fffffffu) return false;
    const int HO = (HI + 2 * pad - R) / stride + 1, WO = (WI + 2 * pad - S) / stride + 1;
    const int WLD = WI + 2 * pad, VH = HI + 2 * pad;
    const long nrows = (long)N * HO;
    if (pool && ((HO | WO) & 1)) return false;
    double best = 0.0;
    bool found = false;
    for (const Variant& v : kVariants) {
        if (v.R != R || v.S != S) continue;
        if (v.vec == 4 ? (J % v.CB != 0 || (J * R * S) % 4 != 0) : J >= 4) continue;
        if (v.vec == 4 && R == 3 && (M <= 64 ? v.mb != 64 : v.mb != 128)) continue;
        const int cap = v.nt * v.wn * 32;
        if (WO > cap) continue;
        const int tr_max = (long)(cap / WO) < nrows ? cap / WO : (int)nrows;
        for (int TR = tr_max; TR >= 1; --TR) {
            if (pool && (TR & 1)) continue;
            const int ptiles = (int)((nrows + TR - 1) / TR);
            // staged rows of the widest tile: from the first output row's first input row to the last one's last,
            // through the pad rows between images (the tile starts repeat with period HO)
            int THI = 0;
            for (int t = 0; t < ptiles && t <= HO; ++t) {
                const long r0 = (long)t * TR, r1 = (r0 + TR - 1 < nrows ? r0 + TR - 1 : nrows - 1);
                const long span = (r1 / HO) * VH + (r1 % HO) * stride + R - ((r0 / HO) * VH + (r0 % HO) * stride);
                if (span > THI) THI = (int)span;
            }
            if (THI * WLD > v.maxplane) continue;                    // the threads must cover the staged plane
            const int images = (THI + VH - 1) / VH + 1;              // images the staged rows of one tile can touch
            if ((size_t)images * J * HI * WI * sizeof(float) >= 0x7fffffffu) continue;
            // MFMA lanes doing useful work: pixels of the tiles, and features of the feature tiles
            const double eff = ((double)nrows * WO) / ((double)ptiles * cap) * ((double)M / ((M + v.mb - 1) / v.mb * v.mb));
            for (int padded = (stride == 1 ? 1 : 0); padded >= 0; --padded) {
                // LDS row stride: padded so consecutive pixels stay in consecutive banks across the end of a row
                const int WLDP = padded ? WO + 32 * ((WLD - WO + 31) / 32) : WLD;
                const int PLANEP = THI * WLDP;
                const int lds_buf = v.mb * v.wstr + v.CB * PLANEP;
                // two buffers; the single-chunk kernels (first layers) only ever use the first
                size_t lds_bytes = (size_t)lds_buf * (v.vec == 1 ? 1 : 2) * sizeof(float);
                if (pool && lds_bytes < (size_t)v.mb * (TR * WO / 2) * sizeof(float))
                    lds_bytes = (size_t)v.mb * (TR * WO / 2) * sizeof(float);   // the pooling exchange reuses them
                if (lds_bytes > 156 * 1024) continue;
                // an instantiation compiled for fixed LDS strides serves exactly those
                if (v.wldp && (v.wldp != WLDP || v.planep != PLANEP)) continue;
                // score: MFMA lanes doing useful work, x 0.9 if only one workgroup fits a compute unit, x 0.97 for
                // the conflicting LDS layout, and a penalty for the share of staged rows that are halo (short tiles
                // re-stage the same rows; measured on 14x14 and 24x24 layers)
                double score = eff * (lds_bytes <= 78 * 1024 ? 1.0 : 0.9) * (padded || stride != 1 ? 1.0 : 0.97);
                score *= 1.0 - 0.3 * (double)(THI - TR * stride) / THI;
                if (v.wldp) score *= 1.03;                          // operand offsets are immediates
                // a two-wave workgroup alone on its compute unit (grid within one round) uses two of the four SIMDs
                if (v.threads == 128 && (long)ptiles * ((M + v.mb - 1) / v.mb) <= 256) score *= 0.55;
                {
                    // a grid that cannot fill the chip even with every unit sliced as far as allowed takes as long
                    // as one of its workgroups: then the smaller pixel tile wins, not the better filled one
                    const int nch = (J + v.CB - 1) / v.CB, max_nsl = nch / 8 < 1 ? 1 : (nch / 8 > 16 ? 16 : nch / 8);
                    const long units = (long)ptiles * ((M + v.mb - 1) / v.mb);
                    if (units * max_nsl <= 256) score *= 7.0 / v.nt / eff;     // time of one workgroup ~ pixel blocks per wave
                }
                if (found && score <= best + 1e-9) continue;
                found = true;
                best = score;
                p->v = &v;
                ConvGeo& g = p->g;
                g.N = N; g.J = J; g.M = M; g.HI = HI; g.WI = WI; g.HO = HO; g.WO = WO; g.pad = pad; g.stride = stride;
                g.TR = TR; g.VH = VH; g.THI = THI; g.WLD = WLD; g.WLDP = WLDP; g.PLANEP = PLANEP;
                g.PLANE = THI * WLD; g.NPIX = TR * WO;
                g.ptiles = ptiles; g.mtiles = (M + v.mb - 1) / v.mb;
                g.per_xcd = (g.ptiles + 7) / 8;
                g.lds_buf = lds_buf;
                p->lds_bytes = lds_bytes;
            }
        }
    }
    if (!found) return false;
    const Variant& v = *p->v;
    ConvGeo& g = p->g;
    // Tail slicing.  Workgroups are handed to the 256 compute units as slots free up, so with `units` equal units
    // the busiest compute unit works through ceil(units / 256) of them while the others idle at the end.  The
    // units % 256 that overhang the last full round (all of them, when the grid is no larger than one round) are
    // therefore cut along the contraction into nsl shorter workgroups each, so that the final round is even too.
    // The price is the partial tiles, written and read once (8 bytes per element at ~4 TB/s, relative to the
    // tile's compute time).
    const int upx = g.per_xcd * g.mtiles;                          // units per XCD
    const long units = 8L * upx;
    const int nchunks = (J + v.CB - 1) / v.CB;
    const double ov_job = (8.0 / 4.0e12) / (2.0 * J * R * S / (0.85 * 157.3e12));
    const long slots = 256;            // workgroups per round: one per compute unit
    // units that exist (the XCD ranges are padded with empty ones when the pixel tiles do not divide by 8); if they
    // fit one round they are not padded at all (flat numbering, below)
    const long live = (long)g.ptiles * g.mtiles;
    const long rounds = live > slots ? units / slots : 0, tail = units - rounds * slots;
    int best_tail = 0, best_nsl = 1;
    if (rounds == 0) {
        // a grid within one round: slice every unit just far enough that (almost) every compute unit gets a
        // workgroup; finer slices only add partial-tile traffic (measured at minibatch 4)
        int nsl = 1;
        while (live * nsl < slots * 13 / 16 && nsl < 16 && nchunks / (nsl + 1) >= 8) ++nsl;
        best_nsl = nsl;
        if (nsl > 1) best_tail = (int)units;
    } else if (tail > 0) {
        double best_t = 0.0;
        for (int nsl = 1; nsl <= 16; ++nsl) {
            if (nsl > 1 && nchunks / nsl < 8) break;               // at least 8 chunks per slice
            const long k = (tail * nsl + slots - 1) / slots;       // slices on the busiest compute unit
            double t = (double)rounds + (double)k / nsl;
            if (nsl > 1) t += (double)(tail * nsl) / (double)slots * ov_job;
            if (nsl == 1 || t < best_t * 0.98) { best_t = t; best_nsl = nsl; }
        }
        if (best_nsl > 1) best_tail = (int)tail;
    }
    g.tail_per_xcd = best_tail / 8;
    g.full_per_xcd = upx - g.tail_per_xcd;
    g.nsl = best_tail ? best_nsl : 1;
    g.chunks_per_slice = (nchunks + g.nsl - 1) / g.nsl;
    g.flat = rounds == 0 && g.ptiles % 8 != 0;
    long sliced_units = g.flat ? (g.nsl > 1 ? (long)g.ptiles * g.mtiles : 0) : best_tail;
    int pieces = g.nsl;
    // Equal runs of chunks instead of equal slices of units, where that spreads a one-round grid better: the busiest
    // compute unit works through share / nchunks of a unit instead of 1 / nsl.  The pieces cost a partial tile each
    // (two or three per unit) and the reduction pass, so the saving must be worth tens of microseconds when the
    // uniform plan needs no reduction at all.
    g.sk_share = g.sk_pmax = 0;
    g.sk_nchunks = nchunks;
    if (rounds == 0 && v.vec == 4 && R == 3 && v.mb == 128) {
        const long total = live * nchunks;
        const int share = (int)((total + slots - 1) / slots);
        const double unit_us = 2.0 * J * R * S * v.mb * (v.nt * v.wn * 32) / 0.55e12 * 1e6;     // one unit on one compute unit
        const double saving_us = unit_us * (1.0 / g.nsl - (double)share / nchunks);
        if (share >= 8 && share < nchunks && saving_us > (g.nsl > 1 ? 5.0 : 40.0)) {
            g.sk_share = share;
            g.sk_pmax = (nchunks + share - 1) / share + 1;
            g.flat = 1;
            sliced_units = live;
            pieces = g.sk_pmax;
        }
    }
    p->partial_bytes = (size_t)sliced_units * pieces * v.mb * (v.nt * v.wn * 32) * sizeof(float);
    p->reduce_units = (int)sliced_units;
    return true;
}

// ws: scratch for the partial tiles (only touched when the plan has tail units)
int run_plan(cnn_ctx* ctx, ConvPlan& p, const float* in, const float* wt, float* out, float* ws, int epi,
             const float* aux, unsigned char* arg = nullptr) {
    p.g.epi = epi;
    LaunchArgs a{p.g, p.lds_bytes, in, wt, aux, out, ws, arg};
    int st = p.v->fn(ctx, a);
    if (st != CNN_OK || p.reduce_units == 0) return st;
    {
        cnn::ProfScope ps(ctx, "k_tile_reduce", 0.0);
        // features of a tile per reduction workgroup: 16 where that still leaves thousands of workgroups, else 8
        const int fpb = (long)p.reduce_units * (p.v->mb / 16) >= 2048 ? 16 : 8;
        hipLaunchKernelGGL(k_tile_reduce, dim3((unsigned)p.reduce_units, (unsigned)(p.v->mb / fpb)), dim3(256), 0,
                           ctx->stream, p.g, p.v->mb, p.v->nt * p.v->wn * 32, fpb, ws, aux, out, arg);
    }
    return cnn::launch_check(ctx, "tile_reduce");
}

}  // namespace

namespace cnn {

size_t mfma_conv_fwd_ws(const ConvShape& s) {
    ConvPlan p;
    if (!make_plan(s.R, s.S, s.pad, s.stride, s.N, s.C, s.K, s.H, s.W, &p)) return 0;
    return p.partial_bytes;
}

int mfma_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* y, int relu) {
    ConvPlan p;
    if (!make_plan(s.R, s.S, s.pad, s.stride, s.N, s.C, s.K, s.H, s.W, &p)) return CNN_EUNSUPPORTED;
    if (p.partial_bytes && (!ctx->ws || ctx->ws_bytes < p.partial_bytes)) return CNN_EWORKSPACE;
    return run_plan(ctx, p, x, w, y, reinterpret_cast<float*>(ctx->ws), relu ? EPI_RELU : EPI_NONE, nullptr);
}

size_t mfma_conv_fwd_pool_ws(const ConvShape& s) {
    ConvPlan p;
    if (!make_plan(s.R, s.S, s.pad, s.stride, s.N, s.C, s.K, s.H, s.W, &p, true)) return 0;
    return p.partial_bytes;
}

// a = maxpool2(max(conv_fwd(x, w), 0)) and the window position of each maximum; the full-size result is not stored.
int mfma_conv_fwd_pool(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* a, unsigned char* arg) {
    ConvPlan p;
    if (!make_plan(s.R, s.S, s.pad, s.stride, s.N, s.C, s.K, s.H, s.W, &p, true)) return CNN_EUNSUPPORTED;
    if (p.partial_bytes && (!ctx->ws || ctx->ws_bytes < p.partial_bytes)) return CNN_EWORKSPACE;
    return run_plan(ctx, p, x, w, a, reinterpret_cast<float*>(ctx->ws), EPI_POOL, nullptr, arg);
}

// Backpropagation with stride 1 is a forward convolution of dy (P x Q, K channels) with the mirrored
// transpose-weights and pad' = R-1-pad.
static bool bwd_plan(const ConvShape& s, ConvPlan* p) {
    if (s.stride != 1 || s.R - 1 - s.pad < 0 || s.S - 1 - s.pad < 0 || s.R != s.S) return false;
    if (!make_plan(s.R, s.S, s.R - 1 - s.pad, 1, s.N, s.K, s.C, s.P, s.Q, p)) return false;
    return p->g.HO == s.H && p->g.WO == s.W;
}

// The planner's tile for one pass, for reporting (see cnn_conv_tile_info).
bool mfma_conv_tile_info(const ConvShape& s, int op, int32_t tile[8]) {
    ConvPlan p;
    bool ok = false;
    if (op == CNN_OP_CONV_FWD) ok = make_plan(s.R, s.S, s.pad, s.stride, s.N, s.C, s.K, s.H, s.W, &p);
    else if (op == CNN_OP_CONV_FWD_RELU_POOL) ok = make_plan(s.R, s.S, s.pad, s.stride, s.N, s.C, s.K, s.H, s.W, &p, true);
    else if (op == CNN_OP_CONV_BWD_DATA) ok = bwd_plan(s, &p);
    if (!ok) return false;
    tile[0] = p.v->mb;
    tile[1] = p.g.TR;
    tile[2] = p.g.WO;
    tile[3] = p.v->CB;
    tile[4] = p.g.sk_share ? -p.g.sk_pmax : (p.g.nsl > 0 ? p.g.nsl : 1);
    tile[5] = (int32_t)p.lds_bytes;
    tile[6] = p.g.sk_share ? (int32_t)(((long)p.g.ptiles * p.g.mtiles * p.g.sk_nchunks + p.g.sk_share - 1) / p.g.sk_share)
                           : p.g.ptiles * p.g.mtiles;
    tile[7] = p.v->wn * p.v->nt * 32;
    return true;
}

static size_t wt_bytes(const ConvShape& s) {   // mirrored transpose of the weights, rounded up to 256 bytes
    return ((size_t)s.K * s.C * s.R * s.S * sizeof(float) + 255) / 256 * 256;
}

size_t mfma_conv_bwd_data_ws(const ConvShape& s) {
    ConvPlan p;
    if (!bwd_plan(s, &p)) return 0;
    return wt_bytes(s) + p.partial_bytes;
}

// act != NULL: dx is zeroed where act <= 0 (act = the ReLU output that was this layer's forward input).
// arg != NULL as well: act is a pooled ReLU output with window positions arg, and dx is the full-size (2H x 2W)
// gradient in front of that ReLU + pool.
int mfma_conv_transpose_weights(cnn_ctx* ctx, int K, int C, int RS, const float* w, float* wT) {
    const int tk = transpose_tk(RS);
    dim3 grid((unsigned)((K + tk - 1) / tk), (unsigned)((C + 31) / 32));
    const size_t tl_bytes = ((size_t)tk * (32 * RS + 1)) * sizeof(float);
    if (tl_bytes > 48 * 1024) return CNN_EUNSUPPORTED;
    {
        ProfScope ps(ctx, "k_transpose_flip", 0.0);
        hipLaunchKernelGGL(k_transpose_flip, grid, dim3(256), tl_bytes, ctx->stream, K, C, RS, tk, w, wT);
    }
    return launch_check(ctx, "transpose_flip");
}

int mfma_conv_bwd_data(cnn_ctx* ctx, const ConvShape& s, const float* dy, const float* w, float* dx, const float* act,
                       const unsigned char* arg) {
    ConvPlan p;
    if (!bwd_plan(s, &p)) return CNN_EUNSUPPORTED;      // decided before the workspace is touched
    if (!ctx->ws || ctx->ws_bytes < wt_bytes(s) + p.partial_bytes) return CNN_EWORKSPACE;
    float* wT = reinterpret_cast<float*>(ctx->ws);
    float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(ctx->ws) + wt_bytes(s));
    const int st = mfma_conv_transpose_weights(ctx, s.K, s.C, s.R * s.S, w, wT);
    if (st != CNN_OK) return st;
    return run_plan(ctx, p, dy, wT, dx, partial, arg ? EPI_UNPOOL : (act ? EPI_MASK : EPI_NONE), act,
                    const_cast<unsigned char*>(arg));
}

int mfma_conv_bwd_data_wt(cnn_ctx* ctx, const ConvShape& s, const float* dy, const float* wT, float* dx, const float* act,
                          const unsigned char* arg) {
    ConvPlan p;
    if (!bwd_plan(s, &p)) return CNN_EUNSUPPORTED;
    // the partial tiles sit where the plain call puts them (behind the room of its own transposed copy)
    if (p.partial_bytes && (!ctx->ws || ctx->ws_bytes < wt_bytes(s) + p.partial_bytes)) return CNN_EWORKSPACE;
    float* partial = p.partial_bytes ? reinterpret_cast<float*>(reinterpret_cast<char*>(ctx->ws) + wt_bytes(s)) : nullptr;
    return run_plan(ctx, p, dy, wT, dx, partial, arg ? EPI_UNPOOL : (act ? EPI_MASK : EPI_NONE), act,
                    const_cast<unsigned char*>(arg));
}

}  // namespace cnn
