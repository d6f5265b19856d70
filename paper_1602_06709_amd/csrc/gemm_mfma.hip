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
//
// The chunk loop follows the convolution kernel's recipe (every non-MFMA instruction costs matrix-pipe time):
// two LDS buffers with one barrier per chunk, placed before the chunk's last MFMA group so that the next chunk's
// first operands are read behind it; staging by raw buffer loads whose per-thread byte offsets are computed once
// (rows past the matrix carry an out-of-range offset and read 0), one staging item between MFMA groups; operands
// read one group (two k-steps) ahead through persistent 32-bit LDS pointers with immediate offsets.
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

constexpr int KCP = 32;   // planning unit of the contraction: every chunk size is a multiple of it

// KS: wave groups that share a tile and split every chunk's contraction steps between them (their accumulators are
// added through LDS at the end).  With one workgroup per compute unit it doubles the waves per SIMD, which is what
// hides the LDS and barrier latencies when the grid is a single round.
template <int MT_, int NT_, int WGM_, int WGN_, bool AKM_, bool BKM_, int KS_, int KC_ = 32>
struct GemmCfg {
    static constexpr int MT = MT_, NT = NT_, WGM = WGM_, WGN = WGN_, KS = KS_;
    static constexpr int KC = KC_;      // contraction elements per LDS chunk
    static constexpr bool AKM = AKM_, BKM = BKM_;
    static constexpr int TM = 32 * MT * WGM, TN = 32 * NT * WGN, T = 64 * WGM * WGN * KS;
    static constexpr int A_LDS = AKM ? KC * TM : TM * (KC + 1);
    static constexpr int B_LDS = BKM ? KC * TN : TN * (KC + 1);
    static constexpr int BUF = (A_LDS + B_LDS + 3) / 4 * 4;          // one (A tile, B tile) buffer, 16-byte multiple
    static constexpr int A4 = TM * KC / 4, B4 = TN * KC / 4;
    static constexpr int AS = (A4 + T - 1) / T, BS = (B4 + T - 1) / T;
    static_assert(A4 % T == 0 && B4 % T == 0, "every thread stages whole float4 slots");
    static_assert(KS == 1 || KS == 2, "one or two wave groups");
    static_assert(KS == 1 || WGM * WGN * MT * NT * 1024 <= 2 * BUF, "the accumulator exchange fits the operand buffers");
};

// One operand tile of ROWS x KC elements: per-thread staging slots (float4 each).
//   KM == false: src[row][Kd], float4 along k;  LDS [row][KC+1]
//   KM == true:  src[Kd][rows_total], float4 along the row index;  LDS [k][ROWS]
template <bool KM, int ROWS, int T, int SLOTS, int KC>
struct Stager {
    int vo[SLOTS];         // byte offset of the slot's float4 within chunk 0 of the split (or kOutOfRange)
    int kofs[SLOTS];       // first contraction index of the slot within the chunk
    lds_float* dst[SLOTS]; // where it goes in LDS buffer 0
    f32x4 reg[SLOTS];

    __device__ void init(int rows_total, int Kd, int row0, int tid, float* l) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int f = tid + i * T;
            if (!KM) {
                const int r = f / (KC / 4), kq = f % (KC / 4);
                vo[i] = row0 + r < rows_total ? (int)(((size_t)(row0 + r) * Kd + kq * 4) * sizeof(float)) : kOutOfRange;
                kofs[i] = kq * 4;
                dst[i] = (lds_float*)(l + r * (KC + 1) + kq * 4);
            } else {
                const int k = f / (ROWS / 4), rq = f % (ROWS / 4);
                vo[i] = row0 + rq * 4 < rows_total ? (int)(((size_t)k * rows_total + row0 + rq * 4) * sizeof(float)) : kOutOfRange;
                kofs[i] = k;
                dst[i] = (lds_float*)(l + k * ROWS + rq * 4);
            }
        }
    }
    // chunk starting at contraction index k0; `whole`: the chunk lies entirely below k_end
    __device__ void fetch(int i, __amdgpu_buffer_rsrc_t rs, int rows_total, int k0, int k_end, bool whole) {
        const int so = (KM ? k0 * rows_total : k0) * (int)sizeof(float);
        const int v = (whole || k0 + kofs[i] < k_end) ? vo[i] : kOutOfRange;
        reg[i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, v, so, 0));
    }
    // dst moves between the two LDS buffers once per chunk (kept in registers; recomputing it costs more)
    __device__ void flip(int delta) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) { dst[i] += delta; asm volatile("" : "+v"(dst[i])); }
    }
    __device__ void stage(int i) {
        lds_float* d = dst[i];
        if (!KM) {
            d[0] = reg[i].x; d[1] = reg[i].y; d[2] = reg[i].z; d[3] = reg[i].w;
        } else {
            *(lds_f32x4*)d = reg[i];
        }
    }
};

// Tail slicing: when the tiles fill the chip's workgroup slots one or more times over and leave a short last round,
// the tiles of that round are cut along the contraction into nsl workgroups each (dispatched after all whole tiles),
// which store partial tiles [tail tile][slice][TM][TN]; k_gemm_tail_reduce adds them in slice order.  584 tiles of
// 128 x 128 on 512 slots: 512 whole tiles, then 72 x 7 slices instead of 72 lone workgroups on 72 compute units.
struct GemmTail {
    int flat;               // 1: one-dimensional grid of whole tiles followed by tail slices (one contraction split)
    int tiles_n;            // tiles along Nn
    int whole_tiles;        // tiles [0, whole_tiles) are computed by one workgroup each
    int nsl, k_per_slice;   // slices per tail tile, contraction elements per slice (a multiple of KC)
    float* partial;
};

template <class G>
__global__ void __launch_bounds__(G::T, G::KS == 1 ? 2 : 1)
k_gemm(int M, int Nn, int Kd, int k_per_split, const float* __restrict__ A, const float* __restrict__ B,
       GradSink sink_in, GemmTail tail) {
    constexpr int MT = G::MT, NT = G::NT, T = G::T, KC = G::KC;
    extern __shared__ __attribute__((aligned(16))) float lds[];      // two (A tile, B tile) buffers
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int kg = wave / (G::WGM * G::WGN), wt = wave % (G::WGM * G::WGN);     // wave group, wave within the tile
    const int wm = wt % G::WGM, wn = wt / G::WGM;
    int n0, m0, k_begin, k_end;
    // where the tile goes: element (m, n) at out0 + (m - om0) * ldc + (n - on0) of sink.dw / sink.w / sink.v
    size_t out0 = 0;
    int ldc = Nn, om0 = 0, on0 = 0;
    GradSink sink = sink_in;
    if (tail.flat) {
        int t = blockIdx.x;
        k_begin = 0;
        k_end = Kd;
        const bool slice = t >= tail.whole_tiles;
        if (slice) {
            const int r = t - tail.whole_tiles, sl = r % tail.nsl;
            t = tail.whole_tiles + r / tail.nsl;
            k_begin = sl * tail.k_per_slice;
            k_end = min(k_begin + tail.k_per_slice, Kd);
            sink = GradSink{tail.partial + (size_t)r * G::TM * G::TN, nullptr, nullptr, 0.f, 0.f, ACT_NONE, nullptr, nullptr, 0, 0};     // a partial tile, stored [TM][TN]
            ldc = G::TN;
        }
        n0 = (t % tail.tiles_n) * G::TN;
        m0 = (t / tail.tiles_n) * G::TM;
        if (slice) { om0 = m0; on0 = n0; }
    } else {
        n0 = blockIdx.x * G::TN;
        m0 = blockIdx.y * G::TM;
        k_begin = blockIdx.z * k_per_split;
        k_end = min(k_begin + k_per_split, Kd);
        // sink.dw = C, or the split's private copy [blockIdx.z][M][Nn]; sink.w is only set when there is one split
        out0 = (size_t)blockIdx.z * M * Nn;
    }

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (k_begin < k_end) {
        const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(A), 0, (int)((size_t)M * Kd * sizeof(float)), kRsrcWord3);
        const __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(B), 0, (int)((size_t)Nn * Kd * sizeof(float)), kRsrcWord3);
        Stager<G::AKM, G::TM, T, G::AS, G::KC> sa;
        Stager<G::BKM, G::TN, T, G::BS, G::KC> sb;
        sa.init(M, Kd, m0, tid, lds);
        sb.init(Nn, Kd, n0, tid, lds + G::A_LDS);
        constexpr int NITEMS = G::AS + G::BS;
        auto fetch_item = [&](int it, int k0, bool whole) {
            if (it < G::AS) sa.fetch(it, rs_a, M, k0, k_end, whole);
            else sb.fetch(it - G::AS, rs_b, Nn, k0, k_end, whole);
        };
        auto stage_item = [&](int it) {
            if (it < G::AS) sa.stage(it);
            else sb.stage(it - G::AS);
        };

        // LDS read pointers: element (row, k) at row*sr + k*sk; the high wave half starts KC/2 further along k
        constexpr int a_sr = G::AKM ? 1 : KC + 1, a_sk = G::AKM ? G::TM : 1;
        constexpr int b_sr = G::BKM ? 1 : KC + 1, b_sk = G::BKM ? G::TN : 1;
        // operands of group g: two k-steps (kk = 2g, 2g+1) for every row / column block of the wave; wave group kg
        // takes the chunk's groups [kg * NG, (kg + 1) * NG)
        constexpr int NG = KC / 4 / G::KS;
        const lds_float* ap = (const lds_float*)(lds + (wm * MT * 32 + l32) * a_sr + (half * (KC / 2) + kg * 2 * NG) * a_sk);
        const lds_float* bp = (const lds_float*)(lds + G::A_LDS + (wn * NT * 32 + l32) * b_sr +
                                                 (half * (KC / 2) + kg * 2 * NG) * b_sk);
        auto read_group = [&](int g, float (&a)[MT][2], float (&b)[NT][2]) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int t = 0; t < 2; ++t) a[i][t] = ap[i * 32 * a_sr + (2 * g + t) * a_sk];
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int t = 0; t < 2; ++t) b[j][t] = bp[j * 32 * b_sr + (2 * g + t) * b_sk];
        };

        const int nchunks = (k_end - k_begin + KC - 1) / KC;
        auto chunk_k = [&](int c) { return k_begin + (c < nchunks - 1 ? c : nchunks - 1) * KC; };   // clamped
        auto chunk_whole = [&](int c) { return c < nchunks - 1 || k_begin + nchunks * KC <= k_end; };
#pragma unroll
        for (int it = 0; it < NITEMS; ++it) fetch_item(it, chunk_k(0), chunk_whole(0));
#pragma unroll
        for (int it = 0; it < NITEMS; ++it) stage_item(it);
#pragma unroll
        for (int it = 0; it < NITEMS; ++it) fetch_item(it, chunk_k(1), chunk_whole(1));
        __syncthreads();
        float a_cur[MT][2], b_cur[NT][2];
        read_group(0, a_cur, b_cur);
        int wr_off = G::BUF;                      // staging writes go to the buffer that is not being read
        sa.flip(wr_off);
        sb.flip(wr_off);
        for (int c = 0; c < nchunks; ++c) {
            const int k2 = chunk_k(c + 2);
            const bool whole2 = chunk_whole(c + 2);
            constexpr int IPG = (NITEMS + NG - 1) / NG;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int u = 0; u < IPG; ++u) {
                    const int it = g * IPG + u;
                    if (it < NITEMS) {
                        stage_item(it);
                        fetch_item(it, k2, whole2);
                    }
                }
                float a_nxt[MT][2], b_nxt[NT][2];
                if (g + 1 < NG) {
                    read_group(g + 1, a_nxt, b_nxt);
                } else {
                    __syncthreads();
                    // swap the roles of the two buffers
                    ap += wr_off; bp += wr_off;
                    asm volatile("" : "+v"(ap)); asm volatile("" : "+v"(bp));
                    sa.flip(-wr_off);
                    sb.flip(-wr_off);
                    wr_off = -wr_off;
                    read_group(0, a_nxt, b_nxt);
                }
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < NT; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[i][t], b_cur[j][t], acc[i][j], 0, 0, 0);
#pragma unroll
                for (int k = 0; k < 2 * MT * NT; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 DS read
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
#pragma unroll
                    for (int i = 0; i < MT; ++i) a_cur[i][t] = a_nxt[i][t];
#pragma unroll
                    for (int j = 0; j < NT; ++j) b_cur[j][t] = b_nxt[j][t];
                }
            }
        }
    }

    if (G::KS > 1) {
        // the second wave group hands its accumulators to the first through LDS (free now): [wave][block][v][lane]
        __syncthreads();
        float* ex = lds + (size_t)wt * MT * NT * 1024 + lane;
        if (kg == 1) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) ex[((i * NT + j) * 16 + v) * 64] = acc[i][j][v];
        }
        __syncthreads();
        if (kg == 0) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] += ex[((i * NT + j) * 16 + v) * 64];
        }
    }

    if ((Nn & 3) == 0) {
        // Rows of C are 16-byte aligned: the tile turns through LDS ([TM][TN], lane = column: conflict-free) and
        // leaves as float4, 512 contiguous bytes per tile row, with every thread of the workgroup taking part; the
        // SGD form reads w and v the same way, four float4 pairs in flight per thread.
        constexpr int TM = G::TM, TN = G::TN;
        __syncthreads();                     // operand buffers and exchange slots are no longer read
        if (kg == 0) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        lds[((wm * MT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4)) * TN + (wn * NT + j) * 32 + l32] = acc[i][j][v];
        }
        __syncthreads();
        constexpr int ITER = TM * TN / 4 / T;      // float4 per thread: 4 to 16
        static_assert(TM * TN <= 2 * G::BUF, "the output tile fits the operand buffers");
        auto where = [&](int it, size_t* e) {
            const int idx = tid + it * T, row = idx / (TN / 4), c4 = idx % (TN / 4);
            const int m = m0 + row, n = n0 + 4 * c4;
            const bool ok = m < M && n < Nn;
            *e = ok ? (size_t)(m - om0) * ldc + (n - on0) : 0;
            return ok;
        };
        if (sink.w) {
            // the accumulators are in LDS, their registers are free: every read of w and v the thread needs is issued
            // before the first update (up to 32 float4 in flight per thread; the update is latency-bound otherwise)
            f32x4 wq[ITER], vq[ITER];
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                size_t e;
                where(it, &e);
                // streamed once: non-temporal like the stores (4-6 % on the 25088->4096 and 36864->3072 updates)
                wq[it] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(sink.w + e));
                if (sink.v) vq[it] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(sink.v + e));
            }
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                size_t e;
                if (!where(it, &e)) continue;
                const int idx = tid + it * T;
                const f32x4 gq = *(const lds_f32x4*)(lds + (idx / (TN / 4)) * TN + 4 * (idx % (TN / 4)));
                f32x4 vel = gq, o;
                if (sink.v) {
                    vel.x = fmaf(sink.mu, vq[it].x, gq.x); vel.y = fmaf(sink.mu, vq[it].y, gq.y);
                    vel.z = fmaf(sink.mu, vq[it].z, gq.z); vel.w = fmaf(sink.mu, vq[it].w, gq.w);
                    __builtin_nontemporal_store(vel, reinterpret_cast<f32x4*>(sink.v + e));
                }
                o.x = fmaf(-sink.lr, vel.x, wq[it].x); o.y = fmaf(-sink.lr, vel.y, wq[it].y);
                o.z = fmaf(-sink.lr, vel.z, wq[it].z); o.w = fmaf(-sink.lr, vel.w, wq[it].w);
                __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(sink.w + e));
            }
        } else {
            float* dst = sink.dw + out0;
            if (sink.act != ACT_NONE) {
                // activation folded into the store (never together with contraction splits: out0 == 0)
                const bool masked = sink.act >= ACT_RELU_BWD;
                f32x4 ax[ITER];
#pragma unroll
                for (int it = 0; it < ITER; ++it) {
                    size_t e;
                    where(it, &e);
                    ax[it] = masked ? *reinterpret_cast<const f32x4*>(sink.aux + e) : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int it = 0; it < ITER; ++it) {
                    size_t e;
                    if (!where(it, &e)) continue;
                    const int idx = tid + it * T;
                    f32x4 c = *(const lds_f32x4*)(lds + (idx / (TN / 4)) * TN + 4 * (idx % (TN / 4)));
                    c.x = act_apply(sink.act, c.x, ax[it].x); c.y = act_apply(sink.act, c.y, ax[it].y);
                    c.z = act_apply(sink.act, c.z, ax[it].z); c.w = act_apply(sink.act, c.w, ax[it].w);
                    *reinterpret_cast<f32x4*>(dst + e) = c;
                }
                return;
            }
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                size_t e;
                if (!where(it, &e)) continue;
                const int idx = tid + it * T;
                *reinterpret_cast<f32x4*>(dst + e) = *(const lds_f32x4*)(lds + (idx / (TN / 4)) * TN + 4 * (idx % (TN / 4)));
            }
        }
        return;
    }
    if (kg == 1) return;

    if (sink.w) {
        // SGD step on the tile's elements: all of a 32x32 block's reads are issued before its first write (the
        // update is bound by memory latency otherwise); same arithmetic as sink_store
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int n = n0 + (wn * NT + j) * 32 + l32;
                if (n >= Nn) continue;
                float wv[16], vv[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + (wm * MT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    const size_t e = (size_t)((m < M ? m : M - 1) - om0) * ldc + (n - on0);
                    wv[v] = sink.w[e];
                    vv[v] = sink.v ? sink.v[e] : 0.f;
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + (wm * MT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    if (m >= M) continue;
                    const size_t e = (size_t)(m - om0) * ldc + (n - on0);
                    float vel = acc[i][j][v];
                    if (sink.v) {
                        vel = fmaf(sink.mu, vv[v], vel);
                        __builtin_nontemporal_store(vel, &sink.v[e]);
                    }
                    __builtin_nontemporal_store(fmaf(-sink.lr, vel, wv[v]), &sink.w[e]);
                }
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int n = n0 + (wn * NT + j) * 32 + l32;
            if (n >= Nn) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * MT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (m < M) {
                    const size_t e = out0 + (size_t)(m - om0) * ldc + (n - on0);
                    sink.dw[e] = sink.act == ACT_NONE ? acc[i][j][v]
                                                      : act_apply(sink.act, acc[i][j][v], sink.act >= ACT_RELU_BWD ? sink.aux[e] : 0.f);
                }
            }
        }
}

// C[i] (or the SGD step, sink) = sum over splits of partial[split][i], in split order.
__global__ void __launch_bounds__(256) k_splitk_reduce(int nsplit, size_t MN, const float* __restrict__ partial,
                                                      GradSink sink) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < MN; i += (size_t)gridDim.x * 256) {
        float s0 = 0.f, s1 = 0.f;
        int s = 0;
        for (; s + 1 < nsplit; s += 2) {
            s0 += partial[(size_t)s * MN + i];
            s1 += partial[(size_t)(s + 1) * MN + i];
        }
        if (s < nsplit) s0 += partial[(size_t)s * MN + i];
        sink_store(sink, i, s0 + s1);
    }
}

// C (or the SGD step, sink) of the tail tiles = sum over their slices' partial tiles, in slice order.  One thread per
// element; grid = (TM * TN / 256, tail tiles).
__global__ void __launch_bounds__(256) k_gemm_tail_reduce(int M, int Nn, int TM, int TN, GemmTail tail, GradSink sink) {
    const int t = tail.whole_tiles + blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;                    // element of the tile, row-major [TM][TN]
    const int m = (t / tail.tiles_n) * TM + e / TN, n = (t % tail.tiles_n) * TN + e % TN;
    if (m >= M || n >= Nn) return;
    const size_t tile = (size_t)TM * TN;
    const float* src = tail.partial + (size_t)blockIdx.y * tail.nsl * tile + e;
    float s0 = 0.f, s1 = 0.f;
    int sl = 0;
    for (; sl + 1 < tail.nsl; sl += 2) {
        s0 += src[(size_t)sl * tile];
        s1 += src[(size_t)(sl + 1) * tile];
    }
    if (sl < tail.nsl) s0 += src[(size_t)sl * tile];
    sink_store(sink, (size_t)m * Nn + n, s0 + s1);
}

struct GemmPlan {
    int tm, tn, ks, nsplit, k_per_split;
    int tail_tiles, tail_nsl, tail_k;     // tail slicing (tail_nsl >= 2) of the last tail_tiles tiles
    size_t ws_bytes;
};

GemmPlan plan_gemm(int M, int Nn, int Kd) {
    GemmPlan p;
    p.tm = M <= 32 ? 32 : M <= 64 ? 64 : 128;      // a minibatch of 32 or fewer rows: half the padded MFMA work of a 64-row tile
    // too few 128-row tiles to fill the chip and a short contraction: 64-row tiles (twice as many workgroups) beat
    // splitting the contraction, which needs the partial products written, read back and added
    if (p.tm == 128 && (long)((M + 127) / 128) * ((Nn + 127) / 128) < 256 && Kd <= 4096) p.tm = 64;
    // a few rounds of 128-row tiles whose last round is mostly empty: the busiest compute unit works through
    // ceil(tiles / 256) tiles, and 64-row tiles cut that in finer steps (where the tail of the 128-row tiles is
    // not sliced, below)
    if (p.tm == 128) {
        const long t128 = (long)((M + 127) / 128) * ((Nn + 127) / 128), t64 = (long)((M + 63) / 64) * ((Nn + 127) / 128);
        if (t128 > 256 && t128 < 2 * 256 && ((t64 + 255) / 256) * 64 * 10 < ((t128 + 255) / 256) * 128 * 9) p.tm = 64;
    }
    p.tn = 128;
    const long tiles = (long)((M + p.tm - 1) / p.tm) * ((Nn + p.tn - 1) / p.tn);
    const int chunks = (Kd + KCP - 1) / KCP;
    int max_split = chunks / 8;            // at least 8 chunks (256 contraction elements) per split
    if (max_split < 1) max_split = 1;
    if (max_split > 32) max_split = 32;
    // Splits of the contraction: the busiest compute unit works through ceil(tiles * splits / 256) workgroups of
    // 1 / splits of a tile each (a lone workgroup per compute unit, although it runs two wave groups, below, reaches
    // about 0.9 of the rate of two), and the partial products are written, read back and added (about 4 TB/s, plus
    // the second launch).
    // 288 tiles are two rounds unsplit and nine eighths of one in eight splits.
    int want = 1;
    const long tail_slots = p.tm == 128 ? 512 : 768;      // resident workgroups of the one-wave-group kernels (below)
    const bool sliceable = p.tm >= 64 && tiles > tail_slots && tiles % tail_slots > 0 && tiles % tail_slots <= tail_slots / 2 &&
                           tail_slots / (tiles % tail_slots) >= 2 && chunks >= 16;
    if (!sliceable) {
        const double unit_us = 2.0 * p.tm * p.tn * (double)Kd / 0.55e6;
        double best_t = 0.0;
        for (int ns = 1; ns <= max_split; ++ns) {
            const int c = (chunks + ns - 1) / ns, real = (chunks + c - 1) / c;
            if (real != ns) continue;
            const long k = (tiles * ns + 255) / 256;
            double t = (double)k * c / chunks * unit_us / (k >= 2 ? 1.0 : 0.9);
            if (ns > 1) t += (double)(ns + 1) * M * Nn * 4.0 / 4.0e6 + 6.0;
            if (ns == 1 || t < best_t * 0.97) { best_t = t; want = ns; }
        }
    }
    const int cps = (chunks + want - 1) / want;
    p.k_per_split = cps * KCP;
    p.nsplit = (Kd + p.k_per_split - 1) / p.k_per_split;
    p.ws_bytes = p.nsplit > 1 ? (size_t)p.nsplit * M * Nn * sizeof(float) : 0;
    // a grid of at most one workgroup per compute unit: two wave groups per tile
    p.ks = tiles * p.nsplit <= 256 && p.tm != 32 ? 2 : 1;      // (the 32-row tile has too few staging slots for 512 threads)
    // Tail slicing.  Two workgroups of 128 x 128 are resident per compute unit (registers and LDS), three of
    // 64 x 128 (LDS): 512 or 768 slots.  Tiles beyond the last full round of slots would run one or two to a
    // compute unit on a mostly idle chip; cut along the contraction (at least 8 chunks per slice) they fill one
    // more, shorter, round.
    p.tail_tiles = p.tail_nsl = p.tail_k = 0;
    if (p.nsplit == 1 && p.ks == 1 && p.tm >= 64) {
        const long slots = tail_slots, tail = tiles % slots;
        if (tiles > slots && tail > 0 && tail <= slots / 2) {
            long nsl = slots / tail;
            if (nsl > chunks / 8) nsl = chunks / 8;
            if (nsl > 16) nsl = 16;
            if (nsl >= 2) {
                const int cps2 = (int)((chunks + nsl - 1) / nsl);
                p.tail_k = cps2 * KCP;
                p.tail_nsl = (Kd + p.tail_k - 1) / p.tail_k;
                p.tail_tiles = (int)tail;
                if (p.tail_nsl < 2) p.tail_tiles = p.tail_nsl = p.tail_k = 0;
                else p.ws_bytes = (size_t)p.tail_tiles * p.tail_nsl * p.tm * p.tn * sizeof(float);
            }
        }
    }
    return p;
}

template <class G>
int launch(cnn_ctx* ctx, const GemmPlan& p, int M, int Nn, int Kd, const float* A, const float* B, const GradSink& sink) {
    const GradSink first = p.nsplit > 1 ? sink_dw(reinterpret_cast<float*>(ctx->ws)) : sink;
    constexpr int lds_bytes = 2 * G::BUF * (int)sizeof(float);
    static std::atomic<unsigned long long> attr_done{0};     // one bit per device: the attribute is the device's
    if (lds_bytes > 48 * 1024) {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_gemm<G>), lds_bytes, "hipFuncSetAttribute(gemm)");
        if (st_attr != CNN_OK) return st_attr;
    }
    const int tiles_n = (Nn + G::TN - 1) / G::TN, tiles_m = (M + G::TM - 1) / G::TM;
    dim3 grid((unsigned)tiles_n, (unsigned)tiles_m, (unsigned)p.nsplit);
    GemmTail tail{0, tiles_n, tiles_n * tiles_m, 1, 0, nullptr};
    if (p.tail_nsl >= 2) {
        tail = GemmTail{1, tiles_n, tiles_n * tiles_m - p.tail_tiles, p.tail_nsl, p.tail_k, reinterpret_cast<float*>(ctx->ws)};
        grid = dim3((unsigned)(tail.whole_tiles + p.tail_tiles * p.tail_nsl));
    }
    static const std::string name_s = strf("k_gemm<%dx%d %s%s%s>", G::TM, G::TN, G::AKM ? "At" : "A", G::BKM ? "B" : "Bt",
                                           G::KS == 2 ? " x2" : "");   // (the chunk size is not part of the name)
    static const std::string name_sgd_s = name_s + "+sgd";
    const char* const name = name_s.c_str();
    const char* const name_sgd = name_sgd_s.c_str();
    {
        cnn::ProfScope ps(ctx, first.w ? name_sgd : name, 2.0 * M * Nn * Kd);
        hipLaunchKernelGGL(k_gemm<G>, grid, dim3(G::T), lds_bytes, ctx->stream, M, Nn, Kd, p.k_per_split, A, B, first, tail);
    }
    int st = cnn::launch_check(ctx, "gemm");
    if (st != CNN_OK) return st;
    if (p.tail_nsl >= 2) {
        cnn::ProfScope ps(ctx, sink.w ? "k_gemm_tail_reduce<sgd>" : "k_gemm_tail_reduce", 0.0);
        hipLaunchKernelGGL(k_gemm_tail_reduce, dim3((unsigned)(G::TM * G::TN / 256), (unsigned)p.tail_tiles), dim3(256), 0,
                           ctx->stream, M, Nn, G::TM, G::TN, tail, sink);
        return cnn::launch_check(ctx, "gemm_tail_reduce");
    }
    if (p.nsplit == 1) return st;
    const size_t MN = (size_t)M * Nn;
    size_t g = (MN + 255) / 256;
    if (g > 4096) g = 4096;
    {
        cnn::ProfScope ps(ctx, sink.w ? "k_splitk_reduce<sgd>" : "k_splitk_reduce", 0.0);
        hipLaunchKernelGGL(k_splitk_reduce, dim3((unsigned)g), dim3(256), 0, ctx->stream, p.nsplit, MN, first.dw, sink);
    }
    return cnn::launch_check(ctx, "splitk_reduce");
}

}  // namespace

namespace cnn {

size_t mfma_gemm_ws(int M, int Nn, int Kd) {
    if (M <= 0 || Nn <= 0 || Kd <= 0) return 0;
    return plan_gemm(M, Nn, Kd).ws_bytes;
}

bool mfma_gemm_serves(int M, int Nn, int Kd, int akm, int bkm) {
    // float4 fetches along the contiguous index of each operand
    if ((akm ? M : Kd) % 4 != 0 || (bkm ? Nn : Kd) % 4 != 0) return false;
    // byte offsets inside the kernel are 32-bit
    return (size_t)M * Kd * sizeof(float) < 0x7fffffffu && (size_t)Nn * Kd * sizeof(float) < 0x7fffffffu;
}

int mfma_gemm(cnn_ctx* ctx, int M, int Nn, int Kd, const float* A, int akm, const float* B, int bkm, float* Cp,
              const GradSink* sink) {
    if (!mfma_gemm_serves(M, Nn, Kd, akm, bkm)) return CNN_EUNSUPPORTED;
    const GradSink C = sink ? *sink : sink_dw(Cp);
    const GemmPlan p = plan_gemm(M, Nn, Kd);
    if (p.ws_bytes && (!ctx->ws || ctx->ws_bytes < p.ws_bytes)) return CNN_EWORKSPACE;
#define GO(MT, NT, WGM, WGN, KS, KCH)                                                                               \
    do {                                                                                                            \
        if (!akm && !bkm) return launch<GemmCfg<MT, NT, WGM, WGN, false, false, KS, KCH>>(ctx, p, M, Nn, Kd, A, B, C); \
        if (!akm && bkm) return launch<GemmCfg<MT, NT, WGM, WGN, false, true, KS, KCH>>(ctx, p, M, Nn, Kd, A, B, C);   \
        if (akm && bkm) return launch<GemmCfg<MT, NT, WGM, WGN, true, true, KS, KCH>>(ctx, p, M, Nn, Kd, A, B, C);     \
        return launch<GemmCfg<MT, NT, WGM, WGN, true, false, KS, KCH>>(ctx, p, M, Nn, Kd, A, B, C);                    \
    } while (0)
#ifndef GEMM_KC_A
#define GEMM_KC_A 32
#endif
#ifndef GEMM_KC_B
#define GEMM_KC_B 32
#endif
    if (p.tm == 32) GO(1, 1, 1, 4, 1, 32);
    if (p.tm == 64 && p.ks == 2) GO(2, 1, 1, 4, 2, GEMM_KC_A);
    if (p.tm == 64) GO(2, 1, 1, 4, 1, 32);
    if (p.ks == 2) GO(2, 2, 2, 2, 2, GEMM_KC_B);
    GO(2, 2, 2, 2, 1, 32);
#undef GO
}

}  // namespace cnn
