// Convolution as an implicit GEMM on the gfx950 matrix cores, for every shape the specialised kernels do not cover
// (kernel sizes other than 3x3 / 5x5 / 7x7, rectangular kernels, strided backpropagation and strided weight
// gradients with many input features).  The three loop nests of Section 3.1 are one contraction each:
//   forward          y [k][(n,p,q)]   = sum over (c,r,s)  w[k][(c,r,s)]   * x [n][c][p*st-pad+r][q*st-pad+s]
//   backpropagation  dx[c][(n,h,w)]   = sum over (k,r,s)  w[k][c][r][s]   * dy[n][k][(h+pad-r)/st][(w+pad-s)/st]
//   weight gradient  dw[k][(c,r,s)]   = sum over (n,p,q)  dy[n][k][p][q]  * x [n][c][p*st-pad+r][q*st-pad+s]
// (an element outside its tensor contributes 0).  Strided backpropagation runs once per phase
// ((h + pad) mod st, (w + pad) mod st): the input elements of one phase see only the kernel taps r = phase + st r',
// so each phase is a dense contraction over its own taps and no product is spent on positions the stride skips.
// Nothing is copied or unfolded in memory: the second operand is gathered element by element on its way into LDS.
// An element's address is the sum of a part that depends on its position along the contraction and a part that
// depends on its output column; the part that is fixed for a thread sits in registers, the part that varies comes
// from a small table in LDS (per chunk of the contraction: built three chunks ahead by one thread in eight; per
// output column: built once).
//
// Workgroup: 2 x 2 waves, each WMT x WNT blocks of 32 x 32 (v_mfma_f32_32x32x2_f32); chunks of 32 contraction
// elements in two LDS buffers, one barrier per chunk.  The chunk loop is one straight-line block of eight MFMA groups:
// between the groups, the registers holding chunk c + 1 go to the other LDS buffer one element at a time and each is
// refilled at once with its element of chunk c + 2, so every load has a whole chunk to arrive; operands are read one
// group ahead.  Tensors below 2 GiB are fetched by raw buffer loads (32-bit byte offsets, the hardware returns 0 for
// an element marked as outside), larger ones through 64-bit addresses.  The weight gradient splits the contraction
// over one resident round of workgroups and adds the partial products in a fixed order (Section 3.1: the sum over
// the minibatch).
#include <stdio.h>

#include "common.h"

namespace {


constexpr int KC = 32;
constexpr int kFar = 1 << 24;     // a coordinate no image reaches: marks table entries and columns past the end
enum { FWD = 0, BWD = 1, WGR = 2 };

struct IgArgs {
    int N, C, H, W, K, R, S, st, pad, P, Q;
    int M, Nn, Kd;             // the GEMM's sizes: rows, columns, contraction
    int k_per_split;
    int relu;
    unsigned a_bytes, b_bytes, o_bytes;   // sizes of the operand and output tensors, for their buffer descriptors (below 2 GiB)
};

// Backpropagation, one phase (a, b) of the stride: input rows h0 + st i (i < Hn) see kernel rows a + st r' (r' < Rn)
// at output row hb + i - r'; columns alike.
struct Phase {
    int a, b, h0, w0, Hn, Wn, Rn, Sn, hb, wb;
};
__device__ __forceinline__ Phase make_phase(const IgArgs& g, int z) {
    Phase f;
    f.a = z / g.st; f.b = z - f.a * g.st;
    f.h0 = ((f.a - g.pad) % g.st + g.st) % g.st;
    f.w0 = ((f.b - g.pad) % g.st + g.st) % g.st;
    f.Hn = f.h0 < g.H ? (g.H - f.h0 + g.st - 1) / g.st : 0;
    f.Wn = f.w0 < g.W ? (g.W - f.w0 + g.st - 1) / g.st : 0;
    f.Rn = f.a < g.R ? (g.R - f.a + g.st - 1) / g.st : 0;
    f.Sn = f.b < g.S ? (g.S - f.b + g.st - 1) / g.st : 0;
    f.hb = (f.h0 + g.pad - f.a) / g.st;
    f.wb = (f.w0 + g.pad - f.b) / g.st;
    return f;
}

struct Part {                  // one of the two parts of a gathered element's position
    int off, a, b;
};

// Position along (c, r, s) or (k, r, s): its share of the element offset, and the kernel tap (r, s).
template <int MODE>
__device__ __forceinline__ Part tap_part(const IgArgs& g, const Phase& ph, int idx, int limit) {
    Part t;
    if (idx >= limit) {
        t.off = 0; t.a = MODE == BWD ? kFar : -kFar; t.b = 0;
        return t;
    }
    const int Sn = MODE == BWD ? ph.Sn : g.S;
    const int RS = MODE == BWD ? ph.Rn * ph.Sn : g.R * g.S;
    const int f = idx / RS, rs = idx - f * RS;
    t.a = rs / Sn;
    t.b = rs - t.a * Sn;
    t.off = MODE == BWD ? f * g.P * g.Q : (f * g.H + t.a) * g.W + t.b;
    return t;
}

// Position along (n, p, q) (forward, weight gradient: top-left input element of the window) or (n, h, w)
// (backpropagation: the input element itself, shifted by the padding).
template <int MODE>
__device__ __forceinline__ Part pix_part(const IgArgs& g, const Phase& ph, int idx, int limit) {
    Part t;
    if (idx >= limit) {
        t.off = 0; t.a = -kFar; t.b = 0;
        return t;
    }
    if (MODE == BWD) {
        const int HW = ph.Hn * ph.Wn;
        const int n = idx / HW, hw = idx - n * HW;
        const int i = hw / ph.Wn;
        t.a = ph.hb + i;
        t.b = ph.wb + (hw - i * ph.Wn);
        t.off = n * g.K * g.P * g.Q;
    } else {
        const int PQ = g.P * g.Q;
        const int n = idx / PQ, pq = idx - n * PQ;
        const int p = pq / g.Q;
        t.a = p * g.st - g.pad;
        t.b = (pq - p * g.Q) * g.st - g.pad;
        t.off = (n * g.C * g.H + t.a) * g.W + t.b;
    }
    return t;
}

// Offset of the gathered element, or -1 where it contributes 0.
template <int MODE>
__device__ __forceinline__ int gather_offset(const IgArgs& g, const Part& pix, const Part& tap) {
    if (MODE == BWD) {
        const int oh = pix.a - tap.a, ow = pix.b - tap.b;
        const bool ok = ((unsigned)oh < (unsigned)g.P) & ((unsigned)ow < (unsigned)g.Q);
        return ok ? pix.off + tap.off + oh * g.Q + ow : -1;
    }
    const int h = pix.a + tap.a, w = pix.b + tap.b;
    const bool ok = ((unsigned)h < (unsigned)g.H) & ((unsigned)w < (unsigned)g.W);
    return ok ? pix.off + tap.off : -1;
}

// First operand, element (row m, contraction index kk): offset = m * row_stride + k_part(kk).
template <int MODE>
__device__ __forceinline__ int a_row_stride(const IgArgs& g) {
    return MODE == FWD ? g.Kd : MODE == BWD ? g.R * g.S : g.P * g.Q;
}
template <int MODE>
__device__ __forceinline__ int a_k_part(const IgArgs& g, const Phase& ph, int kk) {
    if (MODE == FWD) return kk;
    if (MODE == BWD) {
        const int RS = ph.Rn * ph.Sn, k = kk / RS, rs = kk - k * RS;
        const int r = rs / ph.Sn, s = rs - r * ph.Sn;
        return (k * g.C * g.R + ph.a + g.st * r) * g.S + ph.b + g.st * s;
    }
    const int PQ = g.P * g.Q, n = kk / PQ;
    return n * g.K * PQ + (kk - n * PQ);
}

// One table entry per contraction index of a chunk: the gathered operand's part that depends on that index (kernel
// tap for forward / backpropagation, pixel for the weight gradient) and the first operand's offset along the
// contraction (-1 past the end of the contraction: such an element is fetched as 0 on both sides).
// NOCHECK (see the kernel): x is a byte offset, beyond every descriptor past the end of the contraction.
template <int MODE, bool NOCHECK>
__device__ __forceinline__ int4 chunk_entry(const IgArgs& g, const Phase& ph, int kk, int k_end) {
    const Part t = MODE == WGR ? pix_part<MODE>(g, ph, kk, k_end) : tap_part<MODE>(g, ph, kk, k_end);
    const bool in = kk < k_end;
    return make_int4(NOCHECK ? (in ? t.off * 4 : kOutOfRange) : t.off, t.a, t.b, in ? a_k_part<MODE>(g, ph, kk) : -1);
}

// WIDE = false: both operands are below 2 GiB and are fetched by raw buffer loads with 32-bit byte offsets (an
// element that contributes 0 gets an offset beyond the descriptor and the hardware returns 0); WIDE = true: 64-bit
// addresses, a clamped offset and a bit per element that decides at the LDS store whether it counts.
// NOCHECK (never with WIDE): every window element of an existing output position exists - forward and weight
// gradient without padding, backpropagation of 1x1 kernels without padding - so a gathered element's byte offset is
// one addition of the two parts, with no coordinates to compare (1x1 layers, the commonest shape that comes here).
template <int MODE, int WMT, int WNT, bool WIDE, bool NOCHECK>
__global__ void __launch_bounds__(256, 2)
k_conv_igemm(IgArgs g, const float* __restrict__ Asrc, const float* __restrict__ Bsrc, const float* __restrict__ act,
             GradSink sink) {
    constexpr int TM = 64 * WMT, TN = 64 * WNT;
    constexpr bool BKM = MODE != WGR;                       // second operand in LDS as [k][TN] (else [TN][KC+1])
    constexpr int A_LDS = TM * (KC + 1);
    constexpr int B_LDS = BKM ? KC * TN : TN * (KC + 1);
    constexpr int BUF = A_LDS + B_LDS;
    constexpr int NA = TM * KC / 256, NB = TN * KC / 256;   // elements per thread and chunk
    constexpr int NITEMS = NA + NB;
    constexpr int NG = KC / 4;                              // MFMA groups per chunk: two contraction steps each
    constexpr int IPG = (NITEMS + NG - 1) / NG;             // staging items per group
    constexpr int SC = WIDE ? 1 : 4;                        // offsets in elements (64-bit addressing) or bytes
    extern __shared__ __attribute__((aligned(16))) float lds[];     // two operand buffers, then the tables
    int4* const ktab = reinterpret_cast<int4*>(lds + 2 * BUF);      // [2][KC]: chunk tables, built three chunks ahead
    int4* const ctab = ktab + 2 * KC;                               // [TN]: per output column (weight gradient only)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wm = wave & 1, wn = wave >> 1;
    const int n0 = blockIdx.x * TN, m0 = blockIdx.y * TM;
    // backpropagation: blockIdx.z is the stride phase, with its own column and contraction counts
    Phase ph = {};
    int Nn = g.Nn, k_begin = 0, k_end = g.Kd;
    if (MODE == BWD) {
        ph = make_phase(g, blockIdx.z);
        Nn = g.N * ph.Hn * ph.Wn;
        k_end = g.K * ph.Rn * ph.Sn;
        if (n0 >= Nn) return;                               // the whole workgroup: no barrier has been reached
    } else {
        k_begin = blockIdx.z * g.k_per_split;
        k_end = min(k_begin + g.k_per_split, g.Kd);
    }
    const int nchunks = (k_end - k_begin + KC - 1) / KC;

    f32x16 acc[WMT][WNT];
#pragma unroll
    for (int i = 0; i < WMT; ++i)
#pragma unroll
        for (int j = 0; j < WNT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (nchunks > 0) {
        // ---- staging: who fetches what.  Operands stored [row][KC+1]: a thread has a fixed contraction index kq
        // and rows rbase + RSTEP i; the [k][TN] operand: a fixed column bn and contraction indices bk + BSTEP i.
        constexpr int RSTEP = 256 / KC, BSTEP = 256 / TN;
        const int kq = tid % KC, rbase = tid / KC;
        const int bn = tid % TN, bk = tid / TN;
        const int a_rs = a_row_stride<MODE>(g);
        const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(Asrc), 0, (int)g.a_bytes, kRsrcWord3);
        const __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(Bsrc), 0, (int)g.b_bytes, kRsrcWord3);
        // rows past the last one repeat it: their products land in output rows that are never stored
        int a_ro[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) a_ro[i] = min(m0 + rbase + RSTEP * i, g.M - 1) * a_rs * SC;
        Part fix = {};                                      // the thread's fixed part of the second operand
        if (BKM) fix = pix_part<MODE>(g, ph, n0 + bn, Nn);
        if (BKM && NOCHECK)                                 // as a byte offset; a column past the end reads element 0
            fix.off = n0 + bn < Nn ? (fix.off + (MODE == BWD ? fix.a * g.Q + fix.b : 0)) * 4 : 0;

        auto build_ktab = [&](int c) {
            if (tid < KC) ktab[(c & 1) * KC + tid] = chunk_entry<MODE, NOCHECK>(g, ph, k_begin + c * KC + tid, k_end);
        };
        build_ktab(0);
        build_ktab(1);
        if (!BKM && tid < TN) {
            const Part t = tap_part<MODE>(g, ph, n0 + tid, Nn);
            ctab[tid] = make_int4(NOCHECK ? t.off * 4 : t.off, t.a, t.b, 0);
        }
        __syncthreads();

        float ra[NA], rb[NB];
        unsigned oka = 0, okb = 0;                          // WIDE: one bit per fetched element, set if it counts
        int a_kv = 0;                                       // the chunk's first-operand offset along the contraction
        Part px = {};                                       // weight gradient: the chunk's pixel for this thread
        lds_float* a_dst = (lds_float*)(lds + rbase * (KC + 1) + kq);
        lds_float* b_dst = (lds_float*)(lds + A_LDS + (BKM ? bk * TN + bn : rbase * (KC + 1) + kq));
        auto begin_chunk = [&](int c) {                     // this thread's entry of chunk c's table
            const int4 e = ktab[(c & 1) * KC + kq];
            a_kv = WIDE ? e.w : (e.w >= 0 ? e.w * 4 : kOutOfRange);
            px.off = e.x; px.a = e.y; px.b = e.z;
        };
        auto table_entry = [&](int c, int j) {              // what B element j of chunk c combines with the thread's part
            return BKM ? ktab[(c & 1) * KC + bk + BSTEP * j] : ctab[rbase + RSTEP * j];
        };
        auto fetch_a = [&](int i) {
            if (WIDE) {
                const bool ok = a_kv >= 0;
                ra[i] = Asrc[ok ? (size_t)(a_ro[i] + a_kv) : 0];
                oka = (oka & ~(1u << i)) | ((unsigned)ok << i);
            } else {
                ra[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_a, a_ro[i] + a_kv, 0, 0));
            }
        };
        auto fetch_b = [&](int j, const int4& e) {
            if (NOCHECK) {
                rb[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_b, (BKM ? fix.off : px.off) + e.x, 0, 0));
                return;
            }
            Part t;
            t.off = e.x; t.a = e.y; t.b = e.z;
            const int o = gather_offset<MODE>(g, BKM ? fix : px, t);
            if (WIDE) {
                rb[j] = Bsrc[o >= 0 ? (size_t)o : 0];
                okb = (okb & ~(1u << j)) | ((unsigned)(o >= 0) << j);
            } else {
                rb[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_b, o >= 0 ? o * 4 : kOutOfRange, 0, 0));
            }
        };
        auto stage_a = [&](int i) { a_dst[i * RSTEP * (KC + 1)] = (!WIDE || ((oka >> i) & 1)) ? ra[i] : 0.f; };
        auto stage_b = [&](int j) {
            b_dst[BKM ? j * BSTEP * TN : j * RSTEP * (KC + 1)] = (!WIDE || ((okb >> j) & 1)) ? rb[j] : 0.f;
        };
        auto fetch_all = [&](int c) {
            begin_chunk(c);
#pragma unroll
            for (int i = 0; i < NA; ++i) fetch_a(i);
#pragma unroll
            for (int j0 = 0; j0 < NB; j0 += 4) {
                int4 e[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) e[u] = table_entry(c, j0 + u);
#pragma unroll
                for (int u = 0; u < 4; ++u) fetch_b(j0 + u, e[u]);
            }
        };

        // chunk 0 to LDS buffer 0, chunk 1 to the registers, then the table of chunk 2 over that of chunk 0
        fetch_all(0);
#pragma unroll
        for (int i = 0; i < NA; ++i) stage_a(i);
#pragma unroll
        for (int j = 0; j < NB; ++j) stage_b(j);
        fetch_all(1);
        __syncthreads();
        build_ktab(2);
        __syncthreads();

        // LDS read pointers of the wave's blocks; the high wave half starts KC/2 further along the contraction
        constexpr int b_sr = BKM ? 1 : KC + 1, b_sk = BKM ? TN : 1;
        const lds_float* ap = (const lds_float*)(lds + (wm * WMT * 32 + l32) * (KC + 1) + half * (KC / 2));
        const lds_float* bp = (const lds_float*)(lds + A_LDS + (wn * WNT * 32 + l32) * b_sr + half * (KC / 2) * b_sk);
        auto read_group = [&](int gq, float (&a)[WMT][2], float (&b)[WNT][2]) {
#pragma unroll
            for (int i = 0; i < WMT; ++i)
#pragma unroll
                for (int t = 0; t < 2; ++t) a[i][t] = ap[i * 32 * (KC + 1) + 2 * gq + t];
#pragma unroll
            for (int j = 0; j < WNT; ++j)
#pragma unroll
                for (int t = 0; t < 2; ++t) b[j][t] = bp[j * 32 * b_sr + (2 * gq + t) * b_sk];
        };
        // the table entries of a group's B items are read one group ahead
        auto read_entries = [&](int c, int gq, int4 (&e)[IPG]) {
#pragma unroll
            for (int u = 0; u < IPG; ++u) {
                const int it = gq * IPG + u;
                if (it >= NA && it < NITEMS) e[u] = table_entry(c, it - NA);
            }
        };

        float a_cur[WMT][2], b_cur[WNT][2];
        read_group(0, a_cur, b_cur);
        int wr_off = BUF;                         // staging writes go to the buffer that is not being read
        a_dst += wr_off;
        b_dst += wr_off;
        int4 e_cur[IPG] = {};
        begin_chunk(2);
        read_entries(2, 0, e_cur);
        // Chunk c: its MFMAs, group by group; between them the registers' elements (chunk c + 1) go to the other LDS
        // buffer one by one, each register being refilled at once with its element of chunk c + 2; one thread in
        // eight also builds the table of chunk c + 3.  Everything past the end of the contraction is fetched as 0.
        for (int c = 0; c < nchunks; ++c) {
            build_ktab(c + 3);
#pragma unroll
            for (int gq = 0; gq < NG; ++gq) {
                int4 e_nxt[IPG] = {};
                float a_nxt[WMT][2], b_nxt[WNT][2];
                if (gq + 1 < NG) read_entries(c + 2, gq + 1, e_nxt);
#pragma unroll
                for (int u = 0; u < IPG; ++u) {
                    const int it = gq * IPG + u;
                    if (it < NA) {
                        stage_a(it);
                        fetch_a(it);
                    } else if (it < NITEMS) {
                        stage_b(it - NA);
                        fetch_b(it - NA, e_cur[u]);
                    }
                }
                if (gq + 1 < NG) {
                    read_group(gq + 1, a_nxt, b_nxt);
                } else {
                    __syncthreads();
                    // swap the roles of the two buffers; the next chunk's table has just become visible
                    ap += wr_off; bp += wr_off;
                    a_dst -= wr_off; b_dst -= wr_off;
                    asm volatile("" : "+v"(ap)); asm volatile("" : "+v"(bp));
                    asm volatile("" : "+v"(a_dst)); asm volatile("" : "+v"(b_dst));
                    wr_off = -wr_off;
                    read_group(0, a_nxt, b_nxt);
                    begin_chunk(c + 3);
                    read_entries(c + 3, 0, e_nxt);
                }
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < WMT; ++i)
#pragma unroll
                        for (int j = 0; j < WNT; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[i][t], b_cur[j][t], acc[i][j], 0, 0, 0);
#pragma unroll
                for (int k = 0; k < 2 * WMT * WNT; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 DS read
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
#pragma unroll
                    for (int i = 0; i < WMT; ++i) a_cur[i][t] = a_nxt[i][t];
#pragma unroll
                    for (int j = 0; j < WNT; ++j) b_cur[j][t] = b_nxt[j][t];
                }
#pragma unroll
                for (int u = 0; u < IPG; ++u) e_cur[u] = e_nxt[u];
            }
        }
    }

    // ---- epilogue: lane = output column (contiguous in memory for all three passes)
#pragma unroll
    for (int j = 0; j < WNT; ++j) {
        const int n = n0 + (wn * WNT + j) * 32 + l32;
        const bool nok = n < Nn;
        int col, rs_out;
        if (MODE == WGR) {
            col = n; rs_out = g.Nn;
        } else if (MODE == FWD) {
            const int plane = g.P * g.Q;
            const int img = (nok ? n : 0) / plane;
            col = img * g.M * plane + ((nok ? n : 0) - img * plane);
            rs_out = plane;
        } else {
            const int plane = ph.Hn * ph.Wn;                // > 0: the workgroup has columns
            const int img = (nok ? n : 0) / plane, hw = (nok ? n : 0) - img * plane;
            const int i = hw / ph.Wn;
            rs_out = g.H * g.W;
            col = img * g.M * rs_out + (ph.h0 + g.st * i) * g.W + ph.w0 + g.st * (hw - i * ph.Wn);
        }
        if (MODE != WGR && !WIDE) {
            // Forward and backpropagation below 2 GiB: buffer stores (and mask loads) whose per-lane offset is fixed for
            // the column and whose row goes into the scalar offset; a column or row outside the tensor gets an offset
            // beyond the descriptor, which the hardware drops.
            const __amdgpu_buffer_rsrc_t rs_o = __builtin_amdgcn_make_buffer_rsrc(sink.dw, 0, (int)g.o_bytes, kRsrcWord3);
            const __amdgpu_buffer_rsrc_t rs_m = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(act ? act : sink.dw), 0,
                                                                                 (int)g.o_bytes, kRsrcWord3);
            const int mlane = m0 + wm * WMT * 32 + 4 * half;
            const int vo = nok ? (col + mlane * rs_out) * 4 : kOutOfRange;
            const bool full = m0 + TM <= g.M;                // every row of the tile exists (uniform)
#pragma unroll
            for (int i = 0; i < WMT; ++i) {
                float mask[16];
                if (MODE == BWD && act) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int mr = i * 32 + 8 * (v / 4) + (v % 4);
                        const int vv = full || mlane + mr < g.M ? vo : kOutOfRange;
                        mask[v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_m, vv, mr * rs_out * 4, 0));
                    }
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int mr = i * 32 + 8 * (v / 4) + (v % 4);
                    const int vv = full || mlane + mr < g.M ? vo : kOutOfRange;
                    float r = acc[i][j][v];
                    if (MODE == FWD && g.relu) r = fmaxf(r, 0.f);
                    if (MODE == BWD && act) r = mask[v] > 0.f ? r : 0.f;
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, r), rs_o, vv, mr * rs_out * 4, 0);
                }
            }
            continue;
        }
#pragma unroll
        for (int i = 0; i < WMT; ++i) {
            float mask[16];
            if (MODE == BWD && act) {      // ReLU derivative of the layer below: all reads before the first store
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + (wm * WMT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    mask[v] = act[(nok && m < g.M) ? (size_t)(col + m * rs_out) : 0];
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * WMT + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (!nok || m >= g.M) continue;
                float r = acc[i][j][v];
                if (MODE == FWD && g.relu) r = fmaxf(r, 0.f);
                if (MODE == BWD && act) r = mask[v] > 0.f ? r : 0.f;
                const size_t e = (size_t)(col + m * rs_out);
                if (MODE == WGR) sink_store(sink, (size_t)blockIdx.z * g.M * g.Nn + e, r);
                else sink.dw[e] = r;
            }
        }
    }
}

// out (or the SGD step, sink) = sum over splits of partial[split][i], in split order
__global__ void __launch_bounds__(256) k_igemm_reduce(int nsplit, size_t MN, const float* __restrict__ partial, GradSink sink) {
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

struct IgPlan {
    bool ok;
    IgArgs a;
    int tm, nsplit;
    size_t ws_bytes;
};

IgPlan plan(int mode, const ConvShape& s) {
    IgPlan p{};
    p.ok = false;
    const size_t lim = 0x7fff0000u;        // element offsets and column indices are 32-bit
    const size_t nx = (size_t)s.N * s.C * s.H * s.W, ny = (size_t)s.N * s.K * s.P * s.Q, nw = (size_t)s.K * s.C * s.R * s.S;
    if (nx == 0 || ny == 0 || nw == 0 || nx >= lim || ny >= lim || nw >= lim) return p;
    // coordinates stay far below the marker for "outside"; one grid layer per stride phase
    if (s.H + s.pad + s.R >= 65536 || s.W + s.pad + s.S >= 65536 || s.stride > 128) return p;
    if ((size_t)s.P * s.stride + s.R >= 65536 || (size_t)s.Q * s.stride + s.S >= 65536) return p;
    IgArgs& a = p.a;
    a.N = s.N; a.C = s.C; a.H = s.H; a.W = s.W; a.K = s.K; a.R = s.R; a.S = s.S; a.st = s.stride; a.pad = s.pad;
    a.P = s.P; a.Q = s.Q;
    a.relu = 0;
    size_t M, Nn, Kd;
    if (mode == FWD) { M = s.K; Nn = (size_t)s.N * s.P * s.Q; Kd = (size_t)s.C * s.R * s.S; }
    else if (mode == BWD) { M = s.C; Nn = (size_t)s.N * s.H * s.W; Kd = (size_t)s.K * s.R * s.S; }
    else { M = s.K; Nn = (size_t)s.C * s.R * s.S; Kd = (size_t)s.N * s.P * s.Q; }
    a.M = (int)M; a.Nn = (int)Nn; a.Kd = (int)Kd;
    p.tm = M <= 64 ? 64 : 128;
    const size_t tiles = ((M + p.tm - 1) / p.tm) * ((Nn + 127) / 128);
    if ((Nn + 127) / 128 > 0x7fffffffu / 2) return p;
    int want = 1;
    if (mode == WGR && tiles < 256) want = (int)(512 / tiles);    // one resident round of workgroups (two per compute unit)
    const int chunks = (int)((Kd + KC - 1) / KC);
    int max_split = chunks / 4;
    if (max_split < 1) max_split = 1;
    if (want > max_split) want = max_split;
    const int cps = (chunks + want - 1) / want;
    a.k_per_split = cps * KC;
    p.nsplit = (int)((Kd + a.k_per_split - 1) / a.k_per_split);
    p.ws_bytes = p.nsplit > 1 ? (size_t)p.nsplit * M * Nn * sizeof(float) : 0;
    p.ok = true;
    return p;
}

template <int MODE, int WMT, bool WIDE, bool NOCHECK>
int launch_as(cnn_ctx* ctx, const IgPlan& p, const ConvShape& s, const float* A, const float* B, const float* act,
              const GradSink& sink) {
    constexpr int TM = 64 * WMT, TN = 128;
    const IgArgs& a = p.a;
    const GradSink first = p.nsplit > 1 ? sink_dw(reinterpret_cast<float*>(ctx->ws)) : sink;
    // backpropagation: a layer of the grid per stride phase, each with at most ceil(H / st) x ceil(W / st) columns per image
    const int hn = (s.H + s.stride - 1) / s.stride, wn = (s.W + s.stride - 1) / s.stride;
    const size_t cols = MODE == BWD ? (size_t)s.N * hn * wn : (size_t)a.Nn;
    dim3 grid((unsigned)((cols + TN - 1) / TN), (unsigned)((a.M + TM - 1) / TM),
              (unsigned)(MODE == BWD ? s.stride * s.stride : p.nsplit));
    constexpr int lds_bytes = (2 * (TM * (KC + 1) + (MODE != WGR ? KC * TN : TN * (KC + 1))) + 4 * (2 * KC + (MODE == WGR ? TN : 0))) *
                              (int)sizeof(float);
    static std::atomic<unsigned long long> attr_done{0};     // one bit per device: the attribute is the device's
    if (lds_bytes > 48 * 1024) {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_conv_igemm<MODE, WMT, 2, WIDE, NOCHECK>), lds_bytes, "hipFuncSetAttribute(conv_igemm)");
        if (st_attr != CNN_OK) return st_attr;
    }
    static const std::string name_s = strf("k_conv_igemm<%s %dx%d%s>", MODE == FWD ? "fwd" : MODE == BWD ? "bwd" : "wgrad", TM, TN,
                                           WIDE ? " wide" : NOCHECK ? " unpadded" : "");
    const char* const name = name_s.c_str();
    {
        cnn::ProfScope ps(ctx, name, cnn::conv_flops(s));
        hipLaunchKernelGGL((k_conv_igemm<MODE, WMT, 2, WIDE, NOCHECK>), grid, dim3(256), lds_bytes, ctx->stream, a, A, B, act, first);
    }
    int st = cnn::launch_check(ctx, "conv_igemm");
    if (st != CNN_OK || p.nsplit == 1) return st;
    const size_t MN = (size_t)a.M * a.Nn;
    size_t gsz = (MN + 255) / 256;
    if (gsz > 4096) gsz = 4096;
    {
        cnn::ProfScope ps(ctx, sink.w ? "k_igemm_reduce<sgd>" : "k_igemm_reduce", 0.0);
        hipLaunchKernelGGL(k_igemm_reduce, dim3((unsigned)gsz), dim3(256), 0, ctx->stream, p.nsplit, MN, first.dw, sink);
    }
    return cnn::launch_check(ctx, "igemm_reduce");
}

// A = the first operand's tensor (weights, or dy for the weight gradient), B = the gathered one
template <int MODE, int WMT>
int launch(cnn_ctx* ctx, IgPlan& p, const ConvShape& s, const float* A, const float* B, const float* act, const GradSink& sink) {
    const size_t nx = (size_t)s.N * s.C * s.H * s.W, ny = (size_t)s.N * s.K * s.P * s.Q, nw = (size_t)s.K * s.C * s.R * s.S;
    const size_t na = MODE == WGR ? ny : nw, nb = MODE == BWD ? ny : nx, no = MODE == FWD ? ny : MODE == BWD ? nx : 0;
    const size_t two_gib = (size_t)1 << 31;
    if (na * sizeof(float) < two_gib && nb * sizeof(float) < two_gib && no * sizeof(float) < two_gib) {
        p.a.a_bytes = (unsigned)(na * sizeof(float));
        p.a.b_bytes = (unsigned)(nb * sizeof(float));
        p.a.o_bytes = (unsigned)(no * sizeof(float));
        // no coordinate can leave its tensor: see NOCHECK at the kernel
        if (s.pad == 0 && (MODE != BWD || (s.R == 1 && s.S == 1)))
            return launch_as<MODE, WMT, false, true>(ctx, p, s, A, B, act, sink);
        return launch_as<MODE, WMT, false, false>(ctx, p, s, A, B, act, sink);
    }
    p.a.a_bytes = p.a.b_bytes = p.a.o_bytes = 0;
    return launch_as<MODE, WMT, true, false>(ctx, p, s, A, B, act, sink);
}

}  // namespace

namespace cnn {

int igemm_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* y, int relu) {
    IgPlan p = plan(FWD, s);
    if (!p.ok) return CNN_EUNSUPPORTED;
    p.a.relu = relu;
    if (p.tm == 64) return launch<FWD, 1>(ctx, p, s, w, x, nullptr, sink_dw(y));
    return launch<FWD, 2>(ctx, p, s, w, x, nullptr, sink_dw(y));
}

int igemm_conv_bwd_data(cnn_ctx* ctx, const ConvShape& s, const float* dy, const float* w, float* dx, const float* act) {
    IgPlan p = plan(BWD, s);
    if (!p.ok) return CNN_EUNSUPPORTED;
    if (p.tm == 64) return launch<BWD, 1>(ctx, p, s, w, dy, act, sink_dw(dx));
    return launch<BWD, 2>(ctx, p, s, w, dy, act, sink_dw(dx));
}

size_t igemm_conv_bwd_weight_ws(const ConvShape& s) {
    const IgPlan p = plan(WGR, s);
    return p.ok ? p.ws_bytes : 0;
}

int igemm_conv_bwd_weight(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* dy, const GradSink& sink) {
    IgPlan p = plan(WGR, s);
    if (!p.ok) return CNN_EUNSUPPORTED;
    if (p.ws_bytes && (!ctx->ws || ctx->ws_bytes < p.ws_bytes)) return CNN_EWORKSPACE;
    if (p.tm == 64) return launch<WGR, 1>(ctx, p, s, dy, x, nullptr, sink);
    return launch<WGR, 2>(ctx, p, s, dy, x, nullptr, sink);
}

}  // namespace cnn
