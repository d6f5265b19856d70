/*
 * libcnn -- one GPU's share of a synchronous-SGD training step for CNNs/DNNs,
 * native to AMD MI355X (gfx950): direct convolution forward, backward-data and
 * backward-weights (with the weight-gradient sum over the per-GPU minibatch),
 * the fully-connected GEMMs and the SGD weight update, all in fp32.
 * The operations are those of arxiv 1602.06709, Section 2.1.
 *
 * General rules for every entry point
 *   - Returns an int status: CNN_OK (0) or a negative CNN_E* code.  Never throws,
 *     aborts or prints.  cnn_strerror() maps a code to a static string and
 *     cnn_last_error() returns the last HIP error text recorded in the context.
 *   - Every tensor pointer is DEVICE memory owned by the caller, at least 16-byte
 *     aligned, dense row-major fp32.  The library allocates and frees no device
 *     memory, keeps no pointer after a call returns, and never synchronises:
 *     work is enqueued on the context's stream (borrowed from the caller).
 *   - Scratch memory is a caller-owned device buffer attached with
 *     cnn_set_workspace(); cnn_workspace_bytes() says how much a call needs.
 *     Calls sharing one context must not overlap in time (they share the scratch).
 *   - Outputs are overwritten (the paper's "+=" starts from zero).  Inputs and
 *     outputs must not alias, except w and v in cnn_sgd_update (in place).
 *   - Arguments are validated before anything is launched: a failed call leaves
 *     device memory untouched.
 *
 * Layouts (canonical on this boundary)
 *   activations and their gradients:   [N][C][H][W]   (minibatch, feature map, row, col)
 *   weights and their gradients:       [K][C][R][S]   (output feature, input feature, kernel row, col);
 *       the paper writes wts[ifm][ofm][kh][kw] -- the same tensor with its first two axes swapped.
 *   fully connected:                   x[N][I], w[O][I], y[N][O]
 *   P = floor((H + 2*pad - R)/stride) + 1 output rows, Q likewise columns.
 *   The paper's channel-blocked layouts (Section 2.3) are available through
 *   cnn_pack_* / cnn_unpack_* for callers that hold data in that form.
 */
#ifndef CNN_H
#define CNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CNN_OK = 0,
    CNN_EINVAL = -1,       /* null pointer, non-positive dimension, stride < 1, pad < 0, empty output, misaligned pointer */
    CNN_EUNSUPPORTED = -2, /* shape outside what any kernel covers (e.g. a tensor of 2^31 or more elements)               */
    CNN_EWORKSPACE = -3,   /* attached workspace smaller than cnn_workspace_bytes() for this call                        */
    CNN_EHIP = -4          /* a HIP call failed; text via cnn_last_error()                                              */
};

/* op codes for cnn_workspace_bytes() */
enum {
    CNN_OP_CONV_FWD = 0,
    CNN_OP_CONV_BWD_DATA = 1,
    CNN_OP_CONV_BWD_WEIGHT = 2,
    CNN_OP_FC_FWD = 3,     /* N, I = C, O = K; H = W = R = S = 1 */
    CNN_OP_FC_BWD = 4,
    CNN_OP_CONV_FWD_RELU_POOL = 5,
    CNN_OP_BLOCK_SEARCH = 6, /* cnn_block_search / cnn_block_search_traversal; the dimensions are ignored */
    CNN_OP_CONV_BWD_WEIGHT_UNPOOL = 7   /* 0 where cnn_conv_bwd_weight_unpool does not serve the shape */
};

/* options for cnn_set_option() */
enum {
    CNN_OPT_FORCE_DIRECT = 0, /* value != 0: route conv / fc calls to the plain one-thread-per-output kernels
                                 (any shape, slow; otherwise only reached by tensors the matrix-core kernels cannot
                                 index); default 0 */
    CNN_OPT_PROFILE = 1       /* value != 0: bracket every kernel the library launches with a pair of HIP events
                                 on the context's stream (host-side objects only); read back with cnn_profile_*.
                                 Recording stops silently after 16384 entries until cnn_profile_reset(). default 0 */
};

typedef struct cnn_ctx cnn_ctx; /* opaque; owns nothing on the device */

/* Context.  hip_stream is a hipStream_t passed as void* (NULL = the default stream); it is borrowed. */
int cnn_create(cnn_ctx** out, void* hip_stream);
int cnn_destroy(cnn_ctx* ctx);
int cnn_set_stream(cnn_ctx* ctx, void* hip_stream);
int cnn_set_workspace(cnn_ctx* ctx, void* dev_ptr, size_t bytes); /* caller-owned; may be NULL/0 to detach */
int cnn_set_option(cnn_ctx* ctx, int option, int value);
/* Scratch bytes the given call needs (0 if none).  For FC ops pass C = I, K = O, H = W = R = S = 1, stride 1, pad 0. */
size_t cnn_workspace_bytes(int op, int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
const char* cnn_strerror(int status);
const char* cnn_last_error(const cnn_ctx* ctx);

/* Per-kernel timing (measurement aid, see CNN_OPT_PROFILE).  cnn_profile_get waits for entry `index` to finish
 * and returns the kernel's name (static string naming the kernel and its tile geometry), the algorithmic FLOPs
 * of that launch (Section 3.1 count; 0 for non-contraction kernels) and its duration in milliseconds. */
int cnn_profile_count(const cnn_ctx* ctx);
int cnn_profile_get(cnn_ctx* ctx, int index, const char** kernel_name, double* flops, float* ms);
int cnn_profile_reset(cnn_ctx* ctx);

/* ---- What this GPU sustains on the two resources the kernels are bound by (measurement aids; results are read
 *   through CNN_OPT_PROFILE timings or events of the caller's own around the call).
 *   cnn_probe_mfma: 512 workgroups of four waves issue iters * 8 register-only fp32 matrix-core instructions
 *     (v_mfma_f32_32x32x2_f32, the one every contraction kernel here is built on) per wave; *flops (host, may be
 *     NULL) receives the FLOPs of the launch.  sink: device memory, CNN_PROBE_SINK_FLOATS floats, overwritten.
 *   cnn_probe_stream: one pass over n floats (n a multiple of 4) in the launch shape of cnn_sgd_update:
 *     CNN_STREAM_READ reads src (dst needs one float and is not written), CNN_STREAM_WRITE fills dst (src may be
 *     NULL), CNN_STREAM_COPY dst <- src.  4*n bytes read and / or written. */
enum { CNN_STREAM_READ = 0, CNN_STREAM_WRITE = 1, CNN_STREAM_COPY = 2 };
#define CNN_PROBE_SINK_FLOATS (512 * 256)
int cnn_probe_mfma(cnn_ctx* ctx, int iters, float* sink, double* flops);
int cnn_probe_stream(cnn_ctx* ctx, int mode, size_t n, const float* src, float* dst);

/* ---- Section 2.1, Algorithm 1 "Forward Propagation":
 *   y[n][k][p][q] = sum_{c,r,s} x[n][c][p*stride + r - pad][q*stride + s - pad] * w[k][c][r][s]
 *   (cross-correlation; positions outside the input contribute 0).
 *   x: N*C*H*W in, w: K*C*R*S in, y: N*K*P*Q out. */
int cnn_conv_fwd(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                 const float* x, const float* w, float* y);

/* ---- Section 2.1 "Backpropagation":
 *   dx[n][c][p*stride + r - pad][q*stride + s - pad] += dy[n][k][p][q] * w[k][c][r][s]   (from dx = 0)
 *   dy: N*K*P*Q in, w in, dx: N*C*H*W out (input positions no tap reaches get 0). */
int cnn_conv_bwd_data(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float* dy, const float* w, float* dx);

/* ---- The same two passes with the neighbouring ReLU folded into the store (saves one pass over the tensor each):
 *   cnn_conv_fwd_relu:       a = max(conv_fwd(x, w), 0)
 *   cnn_conv_bwd_data_relu:  dz = conv_bwd_data(dy, w) where x_act > 0, else 0.  x_act (N*C*H*W) is this layer's
 *                            forward input when that input is a ReLU output, so dz is the gradient in front of
 *                            that ReLU (ReLU'(0) = 0).  Same workspace needs as the plain calls. */
int cnn_conv_fwd_relu(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      const float* x, const float* w, float* a);
int cnn_conv_bwd_data_relu(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const float* dy, const float* w, const float* x_act, float* dz);

/* ---- Forward propagation with the following ReLU AND 2x2 / stride-2 max-pooling folded into the store:
 *   a[n][k][i][j] = max over the window (2i + di, 2j + dj), di, dj in {0, 1}, of max(conv_fwd(x, w), 0)
 *   arg[n][k][i][j] = 2*di + dj of that maximum (the first one in row-major window order on ties), as
 *   cnn_maxpool2_fwd writes it.  a: N*K*(P/2)*(Q/2) floats out, arg: as many bytes out (both device memory).
 *   The full-size activation is never written: in a conv -> ReLU -> pool chain nothing in the backward pass needs
 *   it (cnn_maxpool2_relu_bwd works from a and arg).  Results equal cnn_maxpool2_fwd(cnn_conv_fwd_relu(x, w)) up
 *   to the rounding of the convolution's summation order (pooling wants tiles of whole row pairs, so the two calls
 *   may cut the contraction differently; where they are tiled alike the results are the same bit for bit), and
 *   the window positions agree except at such near-ties.  P and Q must be even.  Returns CNN_EUNSUPPORTED (nothing launched, outputs untouched) for shapes the
 *   tiled kernel does not serve: call the two unfused entry points then.  Workspace: cnn_workspace_bytes with
 *   CNN_OP_CONV_FWD_RELU_POOL. */
int cnn_conv_fwd_relu_pool(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           const float* x, const float* w, float* a, uint8_t* arg);

/* ---- Backpropagation through a layer whose forward input x (N*C*H*W) was the output of ReLU -> 2x2 max-pool of a
 *   N*C*(2H)*(2W) tensor, with the max-pool backward and the ReLU derivative folded into the store:
 *   dz[n][c][2i + di][2j + dj] = conv_bwd_data(dy, w)[n][c][i][j]  if arg[n][c][i][j] == 2*di + dj and
 *                                                                   a_pool[n][c][i][j] > 0,   else 0
 *   a_pool, arg: that pooled activation (this layer's forward input) and its window positions, N*C*H*W each, in.
 *   dz: N*C*(2H)*(2W) out, every element written.  Equals cnn_maxpool2_relu_bwd(cnn_conv_bwd_data(dy, w), arg,
 *   a_pool) bit for bit; the pooled-size gradient is never stored.  Workspace as cnn_conv_bwd_data.  Returns
 *   CNN_EUNSUPPORTED (nothing launched) for shapes the tiled kernel does not serve. */
int cnn_conv_bwd_data_unpool_relu(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                  const float* dy, const float* w, const uint8_t* arg, const float* a_pool, float* dz);

/* ---- Section 2.1 "Weight-gradient Update", summed over the per-GPU minibatch (no 1/N):
 *   dw[k][c][r][s] = sum_{n,p,q} x[n][c][p*stride + r - pad][q*stride + s - pad] * dy[n][k][p][q]
 *   x, dy in; dw: K*C*R*S out.  Needs workspace (partial sums of the split contraction,
 *   reduced in a fixed order: results are bitwise repeatable). */
int cnn_conv_bwd_weight(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                        const float* x, const float* dy, float* dw);

/* ---- cnn_conv_bwd_weight for callers that cannot allocate device memory for a workspace (code under HIP graph
 *   capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments, same kernels, same bits; the
 *   partial sums go to a CNN_STATIC_SCRATCH_BYTES array built into the library's code object (every GPU the
 *   library runs on holds its own copy until the process ends) instead of the workspace attached to the context,
 *   which is neither needed nor touched.  The call allocates nothing on the host or the device.  Layers whose
 *   cnn_workspace_bytes(CNN_OP_CONV_BWD_WEIGHT, ...) exceeds CNN_STATIC_SCRATCH_BYTES return CNN_EWORKSPACE with
 *   nothing launched (text via cnn_last_error).  All calls on one GPU share that GPU's array, whatever their
 *   context or stream: calls that overlap in time on one GPU race.  The array keeps the previous call's partial
 *   sums; every call overwrites the part it reads, nothing needs clearing.  CNN_OPT_PROFILE does not record it. */
#define CNN_STATIC_SCRATCH_BYTES (80 << 20)
int cnn_conv_bwd_weight_static(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dy, float* dw);

/* ---- Section 2.1: the fully-connected layer is the same loop nest with k_h = k_w = out_h = out_w = 1.
 *   y[n][o] = sum_i x[n][i] * w[o][i] */
int cnn_fc_fwd(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, float* y);
/*   dx[n][i] = sum_o dy[n][o] * w[o][i]      (skipped when dx == NULL; then w may be NULL)
 *   dw[o][i] = sum_n dy[n][o] * x[n][i]      (skipped when dw == NULL; then x may be NULL) */
int cnn_fc_bwd(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, const float* dy,
               float* dx, float* dw);

/* ---- Fully-connected layers with the neighbouring element-wise activation folded into the GEMM's store (one pass
 *   over the activation tensor less per layer and direction; Section 2.1's loop nest is unchanged):
 *     cnn_fc_fwd_act:      a = act(x W^T)
 *     cnn_fc_bwd_act, cnn_fc_bwd_sgd_act: as cnn_fc_bwd / cnn_fc_bwd_sgd for a layer whose input x IS the output of
 *       `act_in` (the activation behind the previous layer): dz receives the gradient in FRONT of that activation,
 *       dz = (dy W) * act_in'(.) with ReLU' = 1 where x > 0 (else 0) and sigmoid' = x * (1 - x).
 *   act / act_in: CNN_ACT_NONE (the plain call), CNN_ACT_RELU, CNN_ACT_SIGMOID.  Same bits as the plain call followed
 *   by cnn_relu_fwd / cnn_sigmoid_fwd, resp. cnn_relu_bwd(x, .) / cnn_sigmoid_bwd(x, .).  Workspace as the plain
 *   calls.  CNN_EUNSUPPORTED (nothing launched) for shapes only the plain fallback kernels serve (I or O not a
 *   multiple of 4): call the unfused pair there. */
enum { CNN_ACT_NONE = 0, CNN_ACT_RELU = 1, CNN_ACT_SIGMOID = 2 };
int cnn_fc_fwd_act(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, float* a, int act);
int cnn_fc_bwd_act(cnn_ctx* ctx, int N, int I, int O, const float* x, const float* w, const float* dy, float* dz,
                   float* dw, int act_in);
int cnn_fc_bwd_sgd_act(cnn_ctx* ctx, int N, int I, int O, const float* x, float* w, const float* dy, float* dz, float* v,
                       float lr, float momentum, int act_in);

/* ---- SGD step (the paper's "vanilla SGD", Sections 1 and 3.4; no weight decay, no Nesterov):
 *   v <- momentum * v + dw ;  w <- w - lr * v         (v == NULL: w <- w - lr * dw, momentum ignored)
 *   n elements; w and v updated in place.  One launch over the whole (flat) parameter arena.  Bound by HBM (20 bytes
 *   per element with momentum, 12 without); the three arrays are walked in lock step and the rate depends on where
 *   they lie relative to each other: ranges of one allocation, each shifted by a few KB against the next, measured
 *   6.7-6.9 TB/s where three separate allocations of the same size gave 6.3-6.4 TB/s. */
int cnn_sgd_update(cnn_ctx* ctx, size_t n, float* w, const float* dw, float* v, float lr, float momentum);

/* ---- Weight gradient with the SGD step folded into its last stage.  The weight gradient is a two-stage sum: partial
 *   sums over parts of the minibatch, then their reduction (Section 3.1); the update needs each reduced element
 *   exactly once (Section 3.4), so the reduction hands it to the update and dw never reaches memory:
 *     g = the element cnn_conv_bwd_weight / cnn_fc_bwd would store;  v <- momentum * v + g;  w <- w - lr * v
 *     (v == NULL: w <- w - lr * g).  Same arithmetic as cnn_sgd_update on a stored g: identical bits.
 *   w [K][C][R][S] (or [O][I]) and v are updated in place.  The layer's backpropagation needs the weights of this
 *   iteration: issue cnn_conv_bwd_data BEFORE cnn_conv_bwd_weight_sgd; cnn_fc_bwd_sgd computes dx (may be NULL:
 *   first layer) from the old w itself before it updates.  (The paper computes the weight gradient first so that its
 *   exchange between nodes overlaps backpropagation; the update there also lands after backpropagation.)
 *   Workspace: as CNN_OP_CONV_BWD_WEIGHT / CNN_OP_FC_BWD.  Returns CNN_EUNSUPPORTED, with nothing launched and
 *   nothing modified, for shapes only the plain fallback kernels serve: call the unfused pair there. */
int cnn_conv_bwd_weight_sgd(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            const float* x, const float* dy, float* w, float* v, float lr, float momentum);
int cnn_fc_bwd_sgd(cnn_ctx* ctx, int N, int I, int O, const float* x, float* w, const float* dy, float* dx, float* v,
                   float lr, float momentum);

/* ---- Section 2.3's "transpose-weights", kept resident.  Backpropagation runs as a forward convolution of dy with
 *     wT[c][k][r][s] = w[k][c][R-1-r][S-1-s]        (feature maps swapped, kernel taps mirrored; K*C*R*S floats)
 *   cnn_conv_bwd_data and its fused forms make that copy in the workspace on every call.  A caller that keeps wT
 *   beside w saves the copy: cnn_conv_transpose_weights makes it once (and again whenever w is changed by anything
 *   else), cnn_conv_bwd_data_wt takes it instead of w, and cnn_conv_bwd_weight_sgd_wt -- cnn_conv_bwd_weight_sgd that
 *   also stores every updated weight at its place in wT -- keeps it current across training steps.
 *   cnn_conv_bwd_data_wt covers the three backpropagation forms: x_act == NULL: cnn_conv_bwd_data; x_act != NULL,
 *   arg == NULL: cnn_conv_bwd_data_relu; both given: cnn_conv_bwd_data_unpool_relu (x_act = the pooled activation).
 *   Same bits as those calls.  Workspace: as CNN_OP_CONV_BWD_DATA / CNN_OP_CONV_BWD_WEIGHT.  CNN_EUNSUPPORTED
 *   (nothing launched) where the tiled matrix-core kernel does not serve the layer (strided layers, kernels other
 *   than 3x3 / 5x5 / 7x7): use the plain calls there.  cnn_conv_bwd_weight_sgd_wt returns what
 *   cnn_conv_bwd_weight_sgd returns. */
int cnn_conv_transpose_weights(cnn_ctx* ctx, int K, int C, int R, int S, const float* w, float* wT);
int cnn_conv_bwd_data_wt(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                         const float* dy, const float* wT, const float* x_act, const uint8_t* arg, float* dz);
int cnn_conv_bwd_weight_sgd_wt(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dy, float* w, float* v, float* wT, float lr, float momentum);

/* ---- Weight gradient of a first layer whose output went through ReLU and a 2x2 max-pool (Section 3.1: the first
 *   layer has no backpropagation, so the full-size gradient in front of the pool is needed by nobody else):
 *     dw = cnn_conv_bwd_weight(x, cnn_maxpool2_bwd(dpool, arg))
 *   dpool [N][K][P/2][Q/2] is the gradient behind the pool, already multiplied by the ReLU derivative (what
 *   cnn_conv_bwd_data_relu of the next layer stores when given the pooled activation as x_act); arg are the window
 *   positions written by cnn_conv_fwd_relu_pool or cnn_maxpool2_fwd.  The full-size gradient is formed on the way
 *   into LDS and never exists in memory.  The _sgd form folds the update in as cnn_conv_bwd_weight_sgd does.
 *   Workspace: cnn_workspace_bytes(CNN_OP_CONV_BWD_WEIGHT_UNPOOL, ...).  CNN_EUNSUPPORTED (nothing launched) unless
 *   C = 3, 3x3, stride 1, K <= 64 and P, Q even. */
int cnn_conv_bwd_weight_unpool(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               const float* x, const float* dpool, const uint8_t* arg, float* dw);
int cnn_conv_bwd_weight_unpool_sgd(cnn_ctx* ctx, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                   const float* x, const float* dpool, const uint8_t* arg, float* w, float* v, float lr,
                                   float momentum);

/* ---- Section 2.3 data layouts; pure permutations (bit-exact), lanes past C (or K) are written as 0.
 *   activations:        [N][C][H][W]  <->  [N][ceil(C/SW)][H][W][SW]
 *   weights (transpose == 0): [K][C][R][S] <-> [C][ceil(K/SW)][R][S][SW]   (paper: IFM x OFM/SW x KH x KW x SW)
 *   weights (transpose != 0): [K][C][R][S] <-> [K][ceil(C/SW)][R][S][SW]   (paper: "transpose-weights") */
size_t cnn_packed_act_elems(int N, int C, int H, int W, int SW);
size_t cnn_packed_wt_elems(int K, int C, int R, int S, int SW, int transpose);
int cnn_pack_act(cnn_ctx* ctx, int N, int C, int H, int W, int SW, const float* nchw, float* packed);
int cnn_unpack_act(cnn_ctx* ctx, int N, int C, int H, int W, int SW, const float* packed, float* nchw);
int cnn_pack_wt(cnn_ctx* ctx, int K, int C, int R, int S, int SW, int transpose, const float* kcrs, float* packed);
int cnn_unpack_wt(cnn_ctx* ctx, int K, int C, int R, int S, int SW, int transpose, const float* packed, float* kcrs);

/* ---- Glue between layers.  The paper does not describe these; the network workloads need them.
 *   ReLU: a = max(z, 0); dz = da where z > 0 else 0 (uses the forward INPUT z).
 *   2x2 stride-2 max-pool on [planes][H][W] (H, W even): arg (0..3, one byte) = first maximum in
 *   row-major window order; backward routes dy to that position, zero elsewhere.
 *   sigmoid: a = 1/(1+exp(-z)); dz = da * a * (1 - a) (uses the forward OUTPUT a).
 *   softmax cross-entropy: loss_per_sample[n] = -log softmax(z[n])[label[n]];
 *   dz[n][o] = (softmax(z[n])[o] - [o == label[n]]) / N.  dz may be NULL.  label is device memory, int32, each
 *   entry in [0, O): an entry outside that range gives loss_per_sample[n] = NaN and no -1 term in its row of dz
 *   (nothing is read out of bounds). */
int cnn_relu_fwd(cnn_ctx* ctx, size_t n, const float* z, float* a);
int cnn_relu_bwd(cnn_ctx* ctx, size_t n, const float* z, const float* da, float* dz);
int cnn_maxpool2_fwd(cnn_ctx* ctx, size_t planes, int H, int W, const float* x, float* y, uint8_t* arg);
int cnn_maxpool2_bwd(cnn_ctx* ctx, size_t planes, int H, int W, const float* dy, const uint8_t* arg, float* dx);
/* cnn_maxpool2_bwd followed by cnn_relu_bwd in one pass, for a pool that directly follows a ReLU: y is the pool's
 * forward output (so y > 0 exactly where the ReLU input at the argmax was positive); dz is [planes][H][W]. */
int cnn_maxpool2_relu_bwd(cnn_ctx* ctx, size_t planes, int H, int W, const float* dy, const uint8_t* arg,
                          const float* y, float* dz);
int cnn_sigmoid_fwd(cnn_ctx* ctx, size_t n, const float* z, float* a);
int cnn_sigmoid_bwd(cnn_ctx* ctx, size_t n, const float* a, const float* da, float* dz);
int cnn_softmax_xent(cnn_ctx* ctx, int N, int O, const float* z, const int32_t* label,
                     float* loss_per_sample, float* dz);

/* ---- Cache-blocking model (Section 2.2).  fp32 data (size_data = 4 bytes).
 *   cnn_bf_plane: bytes per FLOP of the loop over one (image, input feature, output feature) triple with everything
 *     read from memory: 4 * (out_w*out_h + in_w*in_h + k_w*k_h) / (2 * k_w*k_h*out_w*out_h), in_x = out_x*s + k_x - 1.
 *   cnn_bf_layer: the ratio when the whole layer is read once.
 *   cnn_bf_block_traversal: the ratio of an output block (images x ofm_block x rows x cols) that stays in
 *     accumulators while all ifm input features stream past it (the section's remark that walking along the input
 *     features precludes reading the output block): 4 * (out + ifm*(ofm_block*k_h*k_w + images*in_h*in_w)) /
 *     (2 * out * ifm * k_h*k_w), out = images*ofm_block*rows*cols.
 *   These three run on the host and return -1 for a non-positive argument.
 *
 *   cnn_block_search: the section's exhaustive search, on the GPU.  Over all blocks (b1_0 images, b1_1 output
 *     features, b2_0 input features, b1_2 x b1_3 output pixels, b2_2 x b2_3 kernel taps), b1_1 a multiple of simd
 *     (or ofm itself when ofm < simd), with BS = 4 * (output block + weight block + input block) < cache_bytes, the
 *     one of least B/F = BS / CPB, CPB = 2 * b1_0*b1_1*b2_0*b1_2*b1_3*b2_2*b2_3.  Ties: the first block in loop order
 *     (b1_0, b1_1, b2_0, b1_2, b1_3, b2_2, b2_3 ascending, leftmost slowest).
 *   cnn_block_search_traversal: the same search for a machine that keeps the output block in accumulators
 *     (4 * b1_0*b1_1*b1_2*b1_3 <= acc_bytes) and streams weights and inputs through a double-buffered staging memory
 *     in chunks of b2_0 input features (2 * 4 * b2_0 * (b1_1*k_h*k_w + b1_0*in_h*in_w) <= stage_bytes, b2_0 a
 *     multiple of chunk); minimises cnn_bf_block_traversal.  block[5], block[6] are 0.
 *   result: DEVICE memory, 8-byte aligned, written by kernels on the context's stream (no synchronisation here).
 *   found = 0 (block all 0, bf 0) when no block fits.  feasible = number of blocks that fit.
 *   Workspace: cnn_workspace_bytes(CNN_OP_BLOCK_SEARCH, ...).  CNN_EUNSUPPORTED for layers so large that a block's
 *   byte count would not fit 62 bits. */
typedef struct cnn_block_result {
    int32_t block[7];
    int32_t found;
    double bf;
    uint64_t feasible;
} cnn_block_result;
double cnn_bf_plane(int out_h, int out_w, int k_h, int k_w, int stride);
double cnn_bf_layer(int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride);
double cnn_bf_block_traversal(int ifm, int k_h, int k_w, int stride, int images, int ofm_block, int rows, int cols);
int cnn_block_search(cnn_ctx* ctx, int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride,
                     int64_t cache_bytes, int simd, cnn_block_result* result);
int cnn_block_search_traversal(cnn_ctx* ctx, int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w,
                               int stride, int64_t acc_bytes, int64_t stage_bytes, int simd, int chunk,
                               cnn_block_result* result);

/* The tile this library's planner gives a convolution pass (op = CNN_OP_CONV_FWD, CNN_OP_CONV_FWD_RELU_POOL or
 * CNN_OP_CONV_BWD_DATA), and its cnn_bf_block_traversal ratio, for comparison with what the search finds for the
 * machine's limits.  Host only.  tile[0] output features per workgroup (for backpropagation: input features, the
 * pass's outputs), [1] output rows per tile (rows of the whole minibatch numbered through), [2] output columns,
 * [3] contraction features per staged chunk, [4] contraction slices of the tail workgroups (1 = none; negative:
 * the tiles' chunks are dealt out in equal runs, one per workgroup, and -[4] is the most pieces a tile is cut
 * into), [5] LDS bytes per workgroup, [6] tiles (in the runs mode: workgroups), [7] accumulator capacity in pixels.  For the ratio a tile of whole images
 * counts as [1] / out_h images of out_h rows, any other as one image of [1] rows.  CNN_EUNSUPPORTED where the tiled
 * matrix-core kernel does not serve the shape. */
int cnn_conv_tile_info(int op, int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int32_t* tile,
                       double* bf);

#ifdef __cplusplus
}
#endif
#endif /* CNN_H */
