// Forward propagation (Section 2.1, Algorithm 1) of a first layer with three input feature maps under a 3x3 kernel
// (stride 1, pad 1, 224 columns, 64 output features: VGG-A's first layer), with the ReLU and the 2x2 max-pool that
// follow it taken in the epilogue.  The layer is bound by memory and latency, not by the matrix cores (13 FLOP per
// byte), and its contraction is a single chunk (27 taps), so the generic tiled kernel spends most of its time in
// load -> barrier -> multiply -> pool phases that do not overlap.  Here a workgroup takes a band of 14 output rows
// of one image: the 16 input rows x 3 channels go to LDS once, the 27 filter taps of every output feature stay in
// registers for the whole band (an A operand is one element per lane), and the band is walked in row pairs with no
// barrier after the load.
//
// Pixel mapping: the 32 pixel lanes of a B operand are 2 rows x 16 columns, so a 2x2 pooling window lies inside one
// wave: the horizontal neighbour is lane ^ 1 (DPP), the vertical one lane ^ 16 (swizzle); no LDS, no barrier.
// Contraction: the 27 taps are paired into 14 MFMA steps (k = 0 on the low wave half, k = 1 on the high half) such
// that the two taps of a pair differ by a constant LDS offset, which is folded into the lane's base address; every
// other offset is an immediate:
//   9 steps  (c, r, 0) | (c, r, 1)            halves differ by one column
//   3 steps  (c, 0, 2) | (c, 1, 2)            ... by one row
//   1 step   (0, 2, 2) | (1, 2, 2)            ... by one channel
//   1 step   (2, 2, 2) | nothing (A = 0)
#include <stdio.h>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;


constexpr int kW = 224, kK = 64;               // columns, output features
constexpr int kBR = 14;                        // output rows per band
constexpr int kRows = kBR + 2;                 // input rows of a band
constexpr int kWP = 240;                       // LDS row stride: 240 % 32 == 16, the two pixel rows hit different banks
constexpr int kCol0 = 4;                       // LDS column of input column 0 (16-byte aligned rows, left pad at 3)
constexpr int kPlane = kRows * kWP;            // LDS channel stride
constexpr int kNTB = kW / 16 / 2;              // 16-column blocks per wave: 7
constexpr int kSteps = 14;
constexpr int kLdsBytes = 3 * kPlane * 4;      // 46080
constexpr int kStageU = (3 * kRows * (kW / 4) + 255) / 256;   // float4 per thread to stage a band: 11

// tap (c*9 + r*3 + s) of the low / high wave half in MFMA step st; -1: none
__host__ __device__ constexpr int tap_lo(int st) {
    return st < 9 ? (st / 3) * 9 + (st % 3) * 3 : st < 12 ? (st - 9) * 9 + 2 : st == 12 ? 8 : 26;
}
__host__ __device__ constexpr int tap_hi(int st) {
    return st < 9 ? tap_lo(st) + 1 : st < 12 ? tap_lo(st) + 3 : st == 12 ? 17 : -1;
}
// LDS offset (floats) of the low half's tap relative to the lane's base
__host__ __device__ constexpr int tap_off(int st) {
    return (tap_lo(st) / 9) * kPlane + ((tap_lo(st) % 9) / 3) * kWP + tap_lo(st) % 3;
}

__global__ void __launch_bounds__(256, 2)
k_conv_c3_pool(int N, int H, int bands, const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ out,
               unsigned char* __restrict__ arg) {
    extern __shared__ __attribute__((aligned(16))) float xl[];    // [3][kRows][kWP]; row i = input row p0 - 1 + i
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int fb = wave & 1, pw = wave >> 1;          // feature block, half of the row's pixel blocks
    const int rr = l32 >> 4, cc = l32 & 15;           // pixel lane = (row of the pair, column in the block)
    const int n = blockIdx.x / bands, p0 = (blockIdx.x % bands) * kBR;

    // ---- the band's input rows: float4 loads (rows outside the image read 0), all issued before the first LDS write
    {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(x), 0, (int)((size_t)N * 3 * H * kW * sizeof(float)), kRsrcWord3);
        constexpr int W4 = kW / 4, total = 3 * kRows * W4;
        f32x4 v[kStageU];
#pragma unroll
        for (int t = 0; t < kStageU; ++t) {
            const int u = tid + 256 * t;
            const int c = u / (kRows * W4), i = (u / W4) % kRows, q4 = u % W4;
            const int h = p0 - 1 + i;
            const bool ok = u < total && h >= 0 && h < H;
            const int vo = ok ? (int)(((((size_t)n * 3 + c) * H + h) * kW + 4 * q4) * sizeof(float)) : kOutOfRange;
            v[t] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, vo, 0, 0));
        }
        // zero columns left and right of every row
        for (int idx = tid; idx < 3 * kRows * 2; idx += 256) xl[(idx >> 1) * kWP + ((idx & 1) ? kCol0 + kW : kCol0 - 1)] = 0.f;
#pragma unroll
        for (int t = 0; t < kStageU; ++t) {
            const int u = tid + 256 * t;
            const int c = u / (kRows * W4), i = (u / W4) % kRows, q4 = u % W4;
            if (u < total) *(lds_f32x4*)(xl + (c * kRows + i) * kWP + kCol0 + 4 * q4) = v[t];
        }
    }

    // ---- this lane's filter taps: feature fb*32 + l32, one element per MFMA step
    float a_reg[kSteps];
    {
        const float* wk = w + (size_t)(fb * 32 + l32) * 27;
#pragma unroll
        for (int st = 0; st < kSteps; ++st) {
            const int tap = half ? tap_hi(st) : tap_lo(st);
            a_reg[st] = tap >= 0 ? wk[tap] : 0.f;
        }
    }
    __syncthreads();

    // per-lane LDS bases for the four kinds of tap pair; input column of output column q and tap column s is
    // q + s - 1, i.e. LDS column q + s + kCol0 - 1
    const int lane0 = rr * kWP + cc + kCol0 - 1 + pw * kNTB * 16;
    const lds_float* b_col = (const lds_float*)(xl + lane0 + half);            // halves one column apart
    const lds_float* b_row = (const lds_float*)(xl + lane0 + half * kWP);      // ... one row apart
    const lds_float* b_chn = (const lds_float*)(xl + lane0 + half * kPlane);   // ... one channel apart
    const lds_float* b_one = (const lds_float*)(xl + lane0);                   // single tap

    // Output addressing: raw buffer stores with a 32-bit per-lane element offset (feature t of group 0, this lane's
    // pooled column in block 0, pooled row 0 of the band), the block as an immediate, the feature group and the row
    // pair as scalar offsets.
    const int HP = H / 2, WPo = kW / 2;
    const __amdgpu_buffer_rsrc_t rs_out = __builtin_amdgcn_make_buffer_rsrc(out, 0, (int)((size_t)N * kK * HP * WPo * sizeof(float)), kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rs_arg = __builtin_amdgcn_make_buffer_rsrc(arg, 0, (int)((size_t)N * kK * HP * WPo), kRsrcWord3);
    const int lane_out = (((n * kK + fb * 32 + 4 * half + 2 * rr + (cc & 1)) * HP + p0 / 2) * WPo) + (pw * kNTB * 16 + cc) / 2;
    const int group_stride = 8 * HP * WPo;            // elements between feature groups (8 features)
    const int rows_here = min(kBR, H - p0);
    const bool odd = cc & 1, low = rr != 0;
    auto pick = [&](float a0, float a1, float a2, float a3) {       // element t = 2*rr + (cc & 1) of (a0, a1, a2, a3)
        const float lo = odd ? a1 : a0, hi = odd ? a3 : a2;
        return low ? hi : lo;
    };
    auto relu = [](float f) { return f > 0.f ? f : 0.f; };

    for (int pl = 0; pl < rows_here; pl += 2) {
        f32x16 acc[kNTB];
        float b_cur[kSteps], b_nxt[kSteps];
        // the 14 B operands of pixel block j (one per MFMA step)
        auto read_block = [&](int j, float (&b)[kSteps]) {
#pragma unroll
            for (int st = 0; st < kSteps; ++st) {
                const lds_float* base = st < 9 ? b_col : st < 12 ? b_row : st == 12 ? b_chn : b_one;
                b[st] = base[pl * kWP + tap_off(st) + 16 * j];
            }
        };
        auto mfma_block = [&](int j, const float (&b)[kSteps]) {
            f32x16 zero;
#pragma unroll
            for (int v = 0; v < 16; ++v) zero[v] = 0.f;
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_reg[0], b[0], zero, 0, 0, 0);
#pragma unroll
            for (int st = 1; st < kSteps; ++st) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_reg[st], b[st], acc[j], 0, 0, 0);
        };
        // ReLU + 2x2 max-pool of block j in registers.  Of every group of four features (registers v = 4g .. 4g+3)
        // lane t = 2*row + column parity of a window keeps feature 4g + t: it picks that feature's value from its
        // own registers and receives it from the three other lanes of the window (each lane sends the register its
        // partner needs), so a group costs three lane exchanges and every lane of a store is active.  First maximum
        // in row-major window order: a column or row wins only if strictly larger.
        auto pool_block = [&](int j) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float r0 = acc[j][4 * g4], r1 = acc[j][4 * g4 + 1], r2 = acc[j][4 * g4 + 2], r3 = acc[j][4 * g4 + 3];
                const float own = relu(pick(r0, r1, r2, r3));
                const float s1 = pick(r1, r0, r3, r2), s2 = pick(r2, r3, r0, r1), s3 = pick(r3, r2, r1, r0);   // for t^1, t^2, t^3
                const float h = relu(__builtin_bit_cast(
                    float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s1), 0xB1, 0xF, 0xF, true)));          // lane ^ 1
                const float vv = relu(__builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, s2), 0x401F)));  // ^ 16
                const float dd = relu(__builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, s3), 0x441F)));  // ^ 17
                const float m_r = own > h ? own : h, m_o = vv > dd ? vv : dd;            // my row, the other row
                const bool right_r = odd ? own > h : h > own, right_o = odd ? vv > dd : dd > vv;
                const bool lower = low ? m_r > m_o : m_o > m_r;
                const bool right = lower == low ? right_r : right_o;
                const int so = g4 * group_stride + (pl / 2) * WPo;      // wave-uniform
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, m_r > m_o ? m_r : m_o), rs_out,
                                                      (lane_out + 8 * j) * 4, so * 4, 0);
                __builtin_amdgcn_raw_buffer_store_b8((unsigned char)((lower ? 2 : 0) + (right ? 1 : 0)), rs_arg,
                                                     lane_out + 8 * j, so, 0);
            }
        };
        // Block j's MFMAs are issued between the pooling instructions of block j - 1 (a wave issues in order, and
        // the two workgroups of a compute unit run in step, so without this the matrix cores idle while every
        // resident wave pools, and the vector ALUs idle while every wave multiplies).
        read_block(0, b_cur);
        read_block(1, b_nxt);
        mfma_block(0, b_cur);
#pragma unroll
        for (int j = 1; j < kNTB; ++j) {
#pragma unroll
            for (int st = 0; st < kSteps; ++st) b_cur[st] = b_nxt[st];
            if (j + 1 < kNTB) read_block(j + 1, b_nxt);
            mfma_block(j, b_cur);
            pool_block(j - 1);
#pragma unroll
            for (int i = 0; i < kSteps; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x080, 1, 0);    // 1 LDS instruction (operand read or lane exchange)
                __builtin_amdgcn_sched_group_barrier(0x002, 11, 0);   // 11 vector ALU instructions
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        pool_block(kNTB - 1);
    }
}

}  // namespace

namespace cnn {

// served: C = 3, 3x3, stride 1, pad 1, 224 columns, 64 output features, an even number of rows, and enough bands to
// fill the chip (a small minibatch is better off with the tiled kernel's finer units)
bool c3_pool_serves(const ConvShape& s) {
    if (s.C != 3 || s.R != 3 || s.S != 3 || s.stride != 1 || s.pad != 1 || s.W != kW || s.K != kK || (s.H & 1)) return false;
    if ((size_t)s.N * 3 * s.H * s.W * sizeof(float) >= 0x7fffffffu) return false;
    const long groups = (long)s.N * ((s.H + kBR - 1) / kBR);
    return groups >= 224;      // measured: 59 against 79 us at 256 bands, 56 against 48 us at 128
}

int c3_pool_conv_fwd(cnn_ctx* ctx, const ConvShape& s, const float* x, const float* w, float* a, unsigned char* arg) {
    if (!c3_pool_serves(s)) return CNN_EUNSUPPORTED;
    static std::atomic<unsigned long long> attr_done{0};     // one bit per device: the attribute is the device's
    {
        const int st_attr = cnn::lds_attr_once(ctx, attr_done, reinterpret_cast<const void*>(&k_conv_c3_pool), kLdsBytes, "hipFuncSetAttribute(conv_c3_pool)");
        if (st_attr != CNN_OK) return st_attr;
    }
    const int bands = (s.H + kBR - 1) / kBR;
    {
        ProfScope ps(ctx, "k_conv_c3_pool<3x3 W224 K64>", conv_flops(s));
        hipLaunchKernelGGL(k_conv_c3_pool, dim3((unsigned)(s.N * bands)), dim3(256), kLdsBytes, ctx->stream, s.N, s.H, bands,
                           x, w, a, arg);
    }
    return launch_check(ctx, "conv_c3_pool");
}

}  // namespace cnn
