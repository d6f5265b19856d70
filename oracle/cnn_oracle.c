/*
 * CPU oracle for the convolution / fully-connected / SGD training path of
 * "Distributed Deep Learning Using Synchronous Stochastic Gradient Descent"
 * (arxiv 1602.06709).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * obviously-correct loop-nest implementation, written straight from the
 * paper's definitions (Section 2.1: Algorithm 1 "Forward Propagation", the
 * "Backpropagation" and "Weight-gradient Update" statements, and the remark
 * that a fully-connected layer is the same nest with k_h = k_w = out_h =
 * out_w = 1).  Inputs are fp32 values; every product and every sum is taken
 * in fp64.  There is no blocking, no fusion, no reordering beyond choosing
 * which loop is outermost (so OpenMP can split it without two threads ever
 * writing one output element).  It shares no code with the GPU library and
 * may only be used by tests, the smoke check and the CPU-baseline leg of the
 * benchmark.
 *
 * Conventions (all arrays dense, row-major, caller-owned):
 *   activations  x[N][C][H][W], y[N][K][P][Q]       (minibatch, feature, h, w)
 *   weights      w[K][C][R][S]  -- the paper's wts[ifm][ofm][kh][kw] with
 *                                  the first two axes swapped
 *   P = floor((H + 2*pad - R)/stride) + 1, Q likewise.
 *   The paper hard-codes "-1" in the input index (pad 1 of its 3x3 examples);
 *   here it is "-pad".  Out-of-range input positions contribute 0.
 *   Cross-correlation: the kernel is not flipped (index is "+ i5", "+ i6").
 *   No bias anywhere (the paper's loops have none).
 *
 * Every contraction can also return S = sum |a*b| over the same terms; the
 * parity bound for the GPU is |diff| <= 1e-4 * S per element.
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC -o liboracle.so cnn_oracle.c -lm
 */
#include <math.h>
#include <omp.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static int out_dim(int in, int k, int stride, int pad) {
    int span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

int oracle_out_dim(int in, int k, int stride, int pad) { return out_dim(in, k, stride, pad); }
int oracle_num_threads(void) { return omp_get_max_threads(); }

/* ------------------------------------------------------------------ */
/* Section 2.1, Algorithm 1: forward propagation.                      */
/* output[n,k,p,q] += input[n,c,p*s+r-pad,q*s+t-pad] * wts[k,c,r,t]    */
/* (the listing's output index "i1" is read as the ofm index i2, as    */
/* the backpropagation statement has it).                              */
/* ------------------------------------------------------------------ */
void oracle_conv_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     const float* x, const float* w, double* y, double* sabs /* may be NULL */) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    const size_t ysz = (size_t)N * K * P * Q;
    memset(y, 0, ysz * sizeof(double));
    if (sabs) memset(sabs, 0, ysz * sizeof(double));
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < C; ++c)
                for (int r = 0; r < R; ++r)
                    for (int t = 0; t < S; ++t) {
                        const double wv = (double)w[(((size_t)k * C + c) * R + r) * S + t];
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            const float* xrow = x + (((size_t)n * C + c) * H + h) * W;
                            double* yrow = y + (((size_t)n * K + k) * P + p) * Q;
                            double* srow = sabs ? sabs + (((size_t)n * K + k) * P + p) * Q : 0;
                            for (int q = 0; q < Q; ++q) {
                                const int ww = q * stride + t - pad;
                                if (ww < 0 || ww >= W) continue;
                                const double prod = (double)xrow[ww] * wv;
                                yrow[q] += prod;
                                if (srow) srow[q] += fabs(prod);
                            }
                        }
                    }
}

/* ------------------------------------------------------------------ */
/* Section 2.1, "Backpropagation" (scatter form, as printed):          */
/* grad_input[n,c,p*s+r-pad,q*s+t-pad] += grad_output[n,k,p,q]*wts[..] */
/* ------------------------------------------------------------------ */
void oracle_conv_bwd_data(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          const float* dy, const float* w, double* dx, double* sabs) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    const size_t xsz = (size_t)N * C * H * W;
    memset(dx, 0, xsz * sizeof(double));
    if (sabs) memset(sabs, 0, xsz * sizeof(double));
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int k = 0; k < K; ++k)
                for (int r = 0; r < R; ++r)
                    for (int t = 0; t < S; ++t) {
                        const double wv = (double)w[(((size_t)k * C + c) * R + r) * S + t];
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            const float* grow = dy + (((size_t)n * K + k) * P + p) * Q;
                            double* drow = dx + (((size_t)n * C + c) * H + h) * W;
                            double* srow = sabs ? sabs + (((size_t)n * C + c) * H + h) * W : 0;
                            for (int q = 0; q < Q; ++q) {
                                const int ww = q * stride + t - pad;
                                if (ww < 0 || ww >= W) continue;
                                const double prod = (double)grow[q] * wv;
                                drow[ww] += prod;
                                if (srow) srow[ww] += fabs(prod);
                            }
                        }
                    }
}

/* ------------------------------------------------------------------ */
/* Section 2.1, "Weight-gradient Update":                              */
/* grad_wts[k,c,r,t] += input[n,c,p*s+r-pad,q*s+t-pad]*grad_out[n,k,p,q]*/
/* a plain sum over the minibatch (no 1/N).  The ofm loop is outermost  */
/* so that threads own disjoint outputs.                               */
/* ------------------------------------------------------------------ */
void oracle_conv_bwd_weight(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            const float* x, const float* dy, double* dw, double* sabs) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t) {
                    double acc = 0.0, sa = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            const float* xrow = x + (((size_t)n * C + c) * H + h) * W;
                            const float* grow = dy + (((size_t)n * K + k) * P + p) * Q;
                            for (int q = 0; q < Q; ++q) {
                                const int ww = q * stride + t - pad;
                                if (ww < 0 || ww >= W) continue;
                                const double prod = (double)xrow[ww] * (double)grow[q];
                                acc += prod;
                                sa += fabs(prod);
                            }
                        }
                    const size_t o = (((size_t)k * C + c) * R + r) * S + t;
                    dw[o] = acc;
                    if (sabs) sabs[o] = sa;
                }
}

/* ------------------------------------------------------------------ */
/* Element-wise ("sampled") forms: the same sums, evaluated only at a   */
/* caller-chosen list of flat output indices.  Each output element of   */
/* every pass is an independent dot product, so large layers can be     */
/* checked on a sample.  bwd-data is written here in gather form (all   */
/* (k,r,t,p,q) whose scatter target is the requested element); a CPU    */
/* test checks it against the printed scatter form above.               */
/* ------------------------------------------------------------------ */
void oracle_conv_fwd_at(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                        const float* x, const float* w, size_t nidx, const int64_t* idx,
                        double* out, double* sabs) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    (void)N;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < nidx; ++i) {
        int64_t f = idx[i];
        const int q = (int)(f % Q); f /= Q;
        const int p = (int)(f % P); f /= P;
        const int k = (int)(f % K); f /= K;
        const int n = (int)f;
        double acc = 0.0, sa = 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t) {
                    const int h = p * stride + r - pad, ww = q * stride + t - pad;
                    if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                    const double prod = (double)x[(((size_t)n * C + c) * H + h) * W + ww] *
                                        (double)w[(((size_t)k * C + c) * R + r) * S + t];
                    acc += prod;
                    sa += fabs(prod);
                }
        out[i] = acc;
        if (sabs) sabs[i] = sa;
    }
}

void oracle_conv_bwd_data_at(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             const float* dy, const float* w, size_t nidx, const int64_t* idx,
                             double* out, double* sabs) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    (void)N;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < nidx; ++i) {
        int64_t f = idx[i];
        const int ww = (int)(f % W); f /= W;
        const int h = (int)(f % H); f /= H;
        const int c = (int)(f % C); f /= C;
        const int n = (int)f;
        double acc = 0.0, sa = 0.0;
        for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t) {
                    const int hn = h + pad - r, wn = ww + pad - t;
                    if (hn < 0 || wn < 0 || hn % stride || wn % stride) continue;
                    const int p = hn / stride, q = wn / stride;
                    if (p >= P || q >= Q) continue;
                    const double prod = (double)dy[(((size_t)n * K + k) * P + p) * Q + q] *
                                        (double)w[(((size_t)k * C + c) * R + r) * S + t];
                    acc += prod;
                    sa += fabs(prod);
                }
        out[i] = acc;
        if (sabs) sabs[i] = sa;
    }
}

void oracle_conv_bwd_weight_at(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dy, size_t nidx, const int64_t* idx,
                               double* out, double* sabs) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for schedule(dynamic, 4)
    for (size_t i = 0; i < nidx; ++i) {
        int64_t f = idx[i];
        const int t = (int)(f % S); f /= S;
        const int r = (int)(f % R); f /= R;
        const int c = (int)(f % C); f /= C;
        const int k = (int)f;
        double acc = 0.0, sa = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p) {
                const int h = p * stride + r - pad;
                if (h < 0 || h >= H) continue;
                for (int q = 0; q < Q; ++q) {
                    const int ww = q * stride + t - pad;
                    if (ww < 0 || ww >= W) continue;
                    const double prod = (double)x[(((size_t)n * C + c) * H + h) * W + ww] *
                                        (double)dy[(((size_t)n * K + k) * P + p) * Q + q];
                    acc += prod;
                    sa += fabs(prod);
                }
            }
        out[i] = acc;
        if (sabs) sabs[i] = sa;
    }
}

/* ------------------------------------------------------------------ */
/* Fully-connected layer: Section 2.1, the 7-loop with                  */
/* k_h = k_w = out_h = out_w = 1.   x[N][I], w[O][I], y[N][O].          */
/* ------------------------------------------------------------------ */
void oracle_fc_fwd(int N, int I, int O, const float* x, const float* w, double* y, double* sabs) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o) {
            double acc = 0.0, sa = 0.0;
            for (int i = 0; i < I; ++i) {
                const double prod = (double)x[(size_t)n * I + i] * (double)w[(size_t)o * I + i];
                acc += prod;
                sa += fabs(prod);
            }
            y[(size_t)n * O + o] = acc;
            if (sabs) sabs[(size_t)n * O + o] = sa;
        }
}

/* dx[n,i] = sum_o dy[n,o] w[o,i] */
void oracle_fc_bwd_data(int N, int I, int O, const float* dy, const float* w, double* dx, double* sabs) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < I; ++i) {
            double acc = 0.0, sa = 0.0;
            for (int o = 0; o < O; ++o) {
                const double prod = (double)dy[(size_t)n * O + o] * (double)w[(size_t)o * I + i];
                acc += prod;
                sa += fabs(prod);
            }
            dx[(size_t)n * I + i] = acc;
            if (sabs) sabs[(size_t)n * I + i] = sa;
        }
}

/* dw[o,i] = sum_n dy[n,o] x[n,i]  (sum over the minibatch, no 1/N) */
void oracle_fc_bwd_weight(int N, int I, int O, const float* x, const float* dy, double* dw, double* sabs) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < O; ++o)
        for (int i = 0; i < I; ++i) {
            double acc = 0.0, sa = 0.0;
            for (int n = 0; n < N; ++n) {
                const double prod = (double)dy[(size_t)n * O + o] * (double)x[(size_t)n * I + i];
                acc += prod;
                sa += fabs(prod);
            }
            dw[(size_t)o * I + i] = acc;
            if (sabs) sabs[(size_t)o * I + i] = sa;
        }
}

/* Sampled FC forms (flat indices into y[N][O], dx[N][I], dw[O][I]). */
void oracle_fc_fwd_at(int N, int I, int O, const float* x, const float* w, size_t nidx,
                      const int64_t* idx, double* out, double* sabs) {
    (void)N;
#pragma omp parallel for schedule(static)
    for (size_t j = 0; j < nidx; ++j) {
        const int o = (int)(idx[j] % O), n = (int)(idx[j] / O);
        double acc = 0.0, sa = 0.0;
        for (int i = 0; i < I; ++i) {
            const double prod = (double)x[(size_t)n * I + i] * (double)w[(size_t)o * I + i];
            acc += prod; sa += fabs(prod);
        }
        out[j] = acc;
        if (sabs) sabs[j] = sa;
    }
}
void oracle_fc_bwd_data_at(int N, int I, int O, const float* dy, const float* w, size_t nidx,
                           const int64_t* idx, double* out, double* sabs) {
    (void)N;
#pragma omp parallel for schedule(static)
    for (size_t j = 0; j < nidx; ++j) {
        const int i = (int)(idx[j] % I), n = (int)(idx[j] / I);
        double acc = 0.0, sa = 0.0;
        for (int o = 0; o < O; ++o) {
            const double prod = (double)dy[(size_t)n * O + o] * (double)w[(size_t)o * I + i];
            acc += prod; sa += fabs(prod);
        }
        out[j] = acc;
        if (sabs) sabs[j] = sa;
    }
}
void oracle_fc_bwd_weight_at(int N, int I, int O, const float* x, const float* dy, size_t nidx,
                             const int64_t* idx, double* out, double* sabs) {
#pragma omp parallel for schedule(static)
    for (size_t j = 0; j < nidx; ++j) {
        const int i = (int)(idx[j] % I), o = (int)(idx[j] / I);
        double acc = 0.0, sa = 0.0;
        for (int n = 0; n < N; ++n) {
            const double prod = (double)dy[(size_t)n * O + o] * (double)x[(size_t)n * I + i];
            acc += prod; sa += fabs(prod);
        }
        out[j] = acc;
        if (sabs) sabs[j] = sa;
    }
}

/* ------------------------------------------------------------------ */
/* SGD.  The paper says only "vanilla SGD" with unaltered hyper-         */
/* parameters (Section 1) and places the update between the gradient     */
/* reduction and the weight broadcast (Section 3.4).  Reading taken:     */
/*     v <- mu*v + g ;  w <- w - lr*v     (mu = 0: w <- w - lr*g)         */
/* no weight decay, no Nesterov.  fp64 from fp32-valued inputs.          */
/* v == NULL means no momentum buffer (mu treated as 0).                 */
/* ------------------------------------------------------------------ */
void oracle_sgd_update(size_t n, const float* w, const float* g, const float* v, double lr, double mu,
                       double* w_out, double* v_out /* NULL iff v NULL */) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        double vel = (double)g[i];
        if (v) { vel = mu * (double)v[i] + (double)g[i]; v_out[i] = vel; }
        w_out[i] = (double)w[i] - lr * vel;
    }
}

/* ------------------------------------------------------------------ */
/* Section 2.3 data layouts (pure permutations, bit-exact):              */
/*  activations N x C x H x W  ->  N x ceil(C/SW) x H x W x SW           */
/*  weights (paper's IFM x OFM x KH x KW -> IFM x (OFM/SW) x KH x KW x SW;*/
/*  from canonical KCRS that is packed[c][k/SW][r][s][k%SW])             */
/*  transpose-weights OFM x (IFM/SW) x KH x KW x SW:                     */
/*  packed[k][c/SW][r][s][c%SW].   Lanes past C (or K) are zero.         */
/* ------------------------------------------------------------------ */
void oracle_pack_act(int N, int C, int H, int W, int SW, const float* nchw, float* packed) {
    const int CB = (C + SW - 1) / SW;
    for (int n = 0; n < N; ++n)
        for (int cb = 0; cb < CB; ++cb)
            for (int h = 0; h < H; ++h)
                for (int ww = 0; ww < W; ++ww)
                    for (int l = 0; l < SW; ++l) {
                        const int c = cb * SW + l;
                        packed[((((size_t)n * CB + cb) * H + h) * W + ww) * SW + l] =
                            c < C ? nchw[(((size_t)n * C + c) * H + h) * W + ww] : 0.0f;
                    }
}
void oracle_unpack_act(int N, int C, int H, int W, int SW, const float* packed, float* nchw) {
    const int CB = (C + SW - 1) / SW;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int ww = 0; ww < W; ++ww)
                    nchw[(((size_t)n * C + c) * H + h) * W + ww] =
                        packed[((((size_t)n * CB + c / SW) * H + h) * W + ww) * SW + c % SW];
}
void oracle_pack_wt(int K, int C, int R, int S, int SW, int transpose, const float* kcrs, float* packed) {
    if (!transpose) {
        const int KB = (K + SW - 1) / SW;
        for (int c = 0; c < C; ++c)
            for (int kb = 0; kb < KB; ++kb)
                for (int r = 0; r < R; ++r)
                    for (int t = 0; t < S; ++t)
                        for (int l = 0; l < SW; ++l) {
                            const int k = kb * SW + l;
                            packed[((((size_t)c * KB + kb) * R + r) * S + t) * SW + l] =
                                k < K ? kcrs[(((size_t)k * C + c) * R + r) * S + t] : 0.0f;
                        }
    } else {
        const int CB = (C + SW - 1) / SW;
        for (int k = 0; k < K; ++k)
            for (int cb = 0; cb < CB; ++cb)
                for (int r = 0; r < R; ++r)
                    for (int t = 0; t < S; ++t)
                        for (int l = 0; l < SW; ++l) {
                            const int c = cb * SW + l;
                            packed[((((size_t)k * CB + cb) * R + r) * S + t) * SW + l] =
                                c < C ? kcrs[(((size_t)k * C + c) * R + r) * S + t] : 0.0f;
                        }
    }
}
void oracle_unpack_wt(int K, int C, int R, int S, int SW, int transpose, const float* packed, float* kcrs) {
    const int KB = (K + SW - 1) / SW, CB = (C + SW - 1) / SW;
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t)
                    kcrs[(((size_t)k * C + c) * R + r) * S + t] =
                        !transpose ? packed[((((size_t)c * KB + k / SW) * R + r) * S + t) * SW + k % SW]
                                   : packed[((((size_t)k * CB + c / SW) * R + r) * S + t) * SW + c % SW];
}

/* ------------------------------------------------------------------ */
/* Glue between layers.  The paper does not describe these; the network  */
/* workloads need them.  Readings: ReLU'(0) = 0; 2x2 stride-2 max-pool,   */
/* gradient to the first maximum in row-major window order; logistic      */
/* sigmoid; loss = mean over the minibatch of -log softmax(z)[label],     */
/* dz = (softmax(z) - onehot)/N.                                          */
/* ------------------------------------------------------------------ */
void oracle_relu_fwd(size_t n, const float* z, double* a) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) a[i] = z[i] > 0.0f ? (double)z[i] : 0.0;
}
/* da -> dz using the forward INPUT z (mask z > 0) */
void oracle_relu_bwd(size_t n, const float* z, const float* da, double* dz) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) dz[i] = z[i] > 0.0f ? (double)da[i] : 0.0;
}
/* planes = N*C; H, W even.  arg[.] in 0..3 = first max in window row-major order */
void oracle_maxpool2_fwd(size_t planes, int H, int W, const float* x, double* y, int32_t* arg) {
    const int P = H / 2, Q = W / 2;
#pragma omp parallel for schedule(static)
    for (size_t pl = 0; pl < planes; ++pl)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                const float* base = x + (pl * H + 2 * p) * W + 2 * q;
                float best = base[0]; int a = 0;
                if (base[1] > best) { best = base[1]; a = 1; }
                if (base[W] > best) { best = base[W]; a = 2; }
                if (base[W + 1] > best) { best = base[W + 1]; a = 3; }
                y[(pl * P + p) * Q + q] = (double)best;
                if (arg) arg[(pl * P + p) * Q + q] = a;
            }
}
void oracle_maxpool2_bwd(size_t planes, int H, int W, const float* dy, const int32_t* arg, double* dx) {
    const int P = H / 2, Q = W / 2;
    memset(dx, 0, planes * H * W * sizeof(double));
#pragma omp parallel for schedule(static)
    for (size_t pl = 0; pl < planes; ++pl)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                const int a = arg[(pl * P + p) * Q + q];
                dx[(pl * H + 2 * p + a / 2) * W + 2 * q + a % 2] = (double)dy[(pl * P + p) * Q + q];
            }
}
void oracle_sigmoid_fwd(size_t n, const float* z, double* a) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) a[i] = 1.0 / (1.0 + exp(-(double)z[i]));
}
/* da -> dz using the forward OUTPUT a */
void oracle_sigmoid_bwd(size_t n, const float* a, const float* da, double* dz) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) dz[i] = (double)da[i] * (double)a[i] * (1.0 - (double)a[i]);
}
/* z[N][O], label[N]; returns the mean loss; dz[N][O] (may be NULL) */
double oracle_softmax_xent(int N, int O, const float* z, const int32_t* label, double* dz) {
    double loss = 0.0;
    for (int n = 0; n < N; ++n) {
        const float* zr = z + (size_t)n * O;
        double m = (double)zr[0];
        for (int o = 1; o < O; ++o) if ((double)zr[o] > m) m = (double)zr[o];
        double sum = 0.0;
        for (int o = 0; o < O; ++o) sum += exp((double)zr[o] - m);
        loss += -(((double)zr[label[n]] - m) - log(sum));
        if (dz)
            for (int o = 0; o < O; ++o)
                dz[(size_t)n * O + o] = (exp((double)zr[o] - m) / sum - (o == label[n] ? 1.0 : 0.0)) / N;
    }
    return loss / N;
}

/* ------------------------------------------------------------------ */
/* FLOP count, Section 3.1:                                             */
/* per pass 2 * MB * ifm * ofm * k_w * k_h * out_w * out_h.             */
/* ------------------------------------------------------------------ */
double oracle_conv_flops_per_pass(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    return 2.0 * N * C * K * R * S * P * Q;
}
