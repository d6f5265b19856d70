/* CPU oracle for the cache-blocking model of arxiv 1602.06709, Section 2.2.
 *
 * TEST INFRASTRUCTURE ONLY: plain formulas and an exhaustive search written out as the loops they are.  Shares no
 * code with the GPU library.
 *
 * Notation (Section 2.2): a block is b1 = (b1_0 images, b1_1 output features, b1_2 x b1_3 output pixels) of the
 * output and b2 = (b2_0 input features, b2_1 output features, b2_2 x b2_3 kernel taps) of the weights, with
 * b1_1 == b2_1 (one block of output features); the input block it needs has
 * b1_0 * b2_0 * (b1_2*s + b2_2 - 1) * (b1_3*s + b2_3 - 1) elements.
 *   BS  = size_data * (output block + weight block + input block)      bytes resident on chip
 *   CPB = 2 * b1_0 * b1_2 * b1_3 * b2_0 * b2_1 * b2_2 * b2_3           FLOPs done on the block
 *   B/F = BS / CPB, minimised subject to BS < Size_cache.
 * Reading: the printed CPB leaves b2_0 (input features) out; the whole-layer ratio given just before it
 * (2 * minibatch * ofm * ifm * k_w * k_h * out_w * out_h in the denominator) needs it, so it is included here.
 * Reading: "one dimension a multiple of the SIMD width, preferably the output dimension" = the block of output
 * features is a multiple of simd (or all of them when the layer has fewer than simd).
 * Reading: among blocks of equal B/F the first in loop order (b1_0, b1_1, b2_0, b1_2, b1_3, b2_2, b2_3 ascending,
 * leftmost slowest) is reported; the paper does not say.
 *
 * Second model ("traversal", the section's remark that walking along the input features precludes reading the
 * output block): the output block stays in an accumulator memory of acc_bytes for the whole walk over all ifm input
 * features and is written once; weights and inputs stream through a staging memory of stage_bytes that holds two
 * copies (double buffering) of a chunk of b2_0 input features.  Per block
 *   bytes = size_data * (b1_0*b1_1*b1_2*b1_3 + ifm * (b1_1*k_h*k_w + b1_0*in_h*in_w)),  in_x = b1_x*s + k_x - 1
 *   FLOPs = 2 * b1_0 * b1_1 * ifm * b1_2 * b1_3 * k_h * k_w
 * minimised subject to size_data*b1_0*b1_1*b1_2*b1_3 <= acc_bytes and
 * 2*size_data*b2_0*(b1_1*k_h*k_w + b1_0*in_h*in_w) <= stage_bytes.  This is this build's extension of the paper's
 * formulation to a machine with a register file and a scratchpad; it reduces to the whole-layer ratio when the block
 * is the layer and to the single-plane ratio for one image, one feature pair.
 */
#include <omp.h>
#include <stdint.h>
#include <stddef.h>

/* bytes / FLOPs of the loop over one (image, input feature, output feature) triple: everything from memory */
double oracle_bf_plane(int out_h, int out_w, int k_h, int k_w, int stride, int size_data) {
    const double in_h = (double)out_h * stride + k_h - 1, in_w = (double)out_w * stride + k_w - 1;
    return size_data * ((double)out_w * out_h + in_w * in_h + (double)k_w * k_h) / (2.0 * k_w * k_h * out_w * out_h);
}

/* bytes / FLOPs when the whole layer is read once */
double oracle_bf_layer(int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride,
                       int size_data) {
    const double in_h = (double)out_h * stride + k_h - 1, in_w = (double)out_w * stride + k_w - 1;
    const double bytes = size_data * ((double)minibatch * ofm * out_w * out_h + (double)minibatch * ifm * in_w * in_h +
                                      (double)ifm * ofm * k_w * k_h);
    return bytes / (2.0 * minibatch * ofm * ifm * k_w * k_h * out_w * out_h);
}

/* b = (b1_0, b1_1, b2_0, b1_2, b1_3, b2_2, b2_3) */
int64_t oracle_bf_block_bytes(const int32_t* b, int stride, int size_data) {
    const int64_t out = (int64_t)b[0] * b[1] * b[3] * b[4];
    const int64_t wts = (int64_t)b[2] * b[1] * b[5] * b[6];
    const int64_t in = (int64_t)b[0] * b[2] * ((int64_t)b[3] * stride + b[5] - 1) * ((int64_t)b[4] * stride + b[6] - 1);
    return size_data * (out + wts + in);
}
int64_t oracle_bf_block_flops(const int32_t* b) {
    return 2 * (int64_t)b[0] * b[3] * b[4] * b[2] * b[1] * b[5] * b[6];
}

/* traversal model, b = (b1_0, b1_1, b2_0, b1_2, b1_3); the kernel is taken whole */
int64_t oracle_bf_trav_bytes(const int32_t* b, int ifm, int k_h, int k_w, int stride, int size_data) {
    const int64_t in = ((int64_t)b[3] * stride + k_h - 1) * ((int64_t)b[4] * stride + k_w - 1);
    return size_data * ((int64_t)b[0] * b[1] * b[3] * b[4] + (int64_t)ifm * ((int64_t)b[1] * k_h * k_w + b[0] * in));
}
int64_t oracle_bf_trav_flops(const int32_t* b, int ifm, int k_h, int k_w) {
    return 2 * (int64_t)b[0] * b[1] * ifm * b[3] * b[4] * k_h * k_w;
}
int64_t oracle_bf_trav_stage_bytes(const int32_t* b, int k_h, int k_w, int stride, int size_data) {
    const int64_t in = ((int64_t)b[3] * stride + k_h - 1) * ((int64_t)b[4] * stride + k_w - 1);
    return 2 * (int64_t)size_data * b[2] * ((int64_t)b[1] * k_h * k_w + b[0] * in);
}

static int n_ofm_blocks(int ofm, int simd) { return ofm < simd ? 1 : ofm / simd; }
static int ofm_block(int ofm, int simd, int i) { return ofm < simd ? ofm : (i + 1) * simd; }

/* Exhaustive search of the single-cache model.  best[7] as in oracle_bf_block_bytes; returns the number of feasible
 * blocks (0: none fits, best untouched).  Threads split the outermost two loops; the merge keeps the first minimum
 * in loop order. */
uint64_t oracle_bf_search(int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride,
                          int size_data, int64_t cache_bytes, int simd, int32_t* best, double* best_bf) {
    const int nkb = n_ofm_blocks(ofm, simd);
    const int outer = minibatch * nkb;
    uint64_t feasible = 0;
    double g_bf = 0.0;
    int64_t g_idx = -1;
    int32_t g_b[7];
#pragma omp parallel
    {
        double t_bf = 0.0;
        int64_t t_idx = -1;
        int32_t t_b[7];
        uint64_t t_feasible = 0;
#pragma omp for schedule(dynamic, 1)
        for (int o = 0; o < outer; ++o) {
            int32_t b[7];
            b[0] = o / nkb + 1;
            b[1] = ofm_block(ofm, simd, o % nkb);
            int64_t idx = (int64_t)o * ifm * out_h * out_w * k_h * k_w;     /* position in loop order */
            for (b[2] = 1; b[2] <= ifm; ++b[2])
                for (b[3] = 1; b[3] <= out_h; ++b[3])
                    for (b[4] = 1; b[4] <= out_w; ++b[4])
                        for (b[5] = 1; b[5] <= k_h; ++b[5])
                            for (b[6] = 1; b[6] <= k_w; ++b[6], ++idx) {
                                const int64_t bs = oracle_bf_block_bytes(b, stride, size_data);
                                if (!(bs < cache_bytes)) continue;
                                ++t_feasible;
                                const double bf = (double)bs / (double)oracle_bf_block_flops(b);
                                if (t_idx < 0 || bf < t_bf) {      /* loop order within a thread is ascending idx */
                                    t_bf = bf; t_idx = idx;
                                    for (int i = 0; i < 7; ++i) t_b[i] = b[i];
                                }
                            }
        }
#pragma omp critical
        {
            feasible += t_feasible;
            if (t_idx >= 0 && (g_idx < 0 || t_bf < g_bf || (t_bf == g_bf && t_idx < g_idx))) {
                g_bf = t_bf; g_idx = t_idx;
                for (int i = 0; i < 7; ++i) g_b[i] = t_b[i];
            }
        }
    }
    if (g_idx >= 0) {
        for (int i = 0; i < 7; ++i) best[i] = g_b[i];
        *best_bf = g_bf;
    }
    return feasible;
}

/* Exhaustive search of the traversal model.  best[5] = (b1_0, b1_1, b2_0, b1_2, b1_3); loop order as listed.
 * b2_0 runs over multiples of chunk (the granularity the staging works in) up to ifm rounded up. */
uint64_t oracle_bf_trav_search(int minibatch, int ifm, int ofm, int out_h, int out_w, int k_h, int k_w, int stride,
                               int size_data, int64_t acc_bytes, int64_t stage_bytes, int simd, int chunk,
                               int32_t* best, double* best_bf) {
    const int nkb = n_ofm_blocks(ofm, simd);
    const int ncb = (ifm + chunk - 1) / chunk;
    uint64_t feasible = 0;
    double g_bf = 0.0;
    int found = 0;
    int32_t b[5];
    for (b[0] = 1; b[0] <= minibatch; ++b[0])
        for (int kb = 0; kb < nkb; ++kb)
            for (int cb = 1; cb <= ncb; ++cb)
                for (b[3] = 1; b[3] <= out_h; ++b[3])
                    for (b[4] = 1; b[4] <= out_w; ++b[4]) {
                        b[1] = ofm_block(ofm, simd, kb);
                        b[2] = cb * chunk;
                        if ((int64_t)size_data * b[0] * b[1] * b[3] * b[4] > acc_bytes) continue;
                        if (oracle_bf_trav_stage_bytes(b, k_h, k_w, stride, size_data) > stage_bytes) continue;
                        ++feasible;
                        const double bf = (double)oracle_bf_trav_bytes(b, ifm, k_h, k_w, stride, size_data) /
                                          (double)oracle_bf_trav_flops(b, ifm, k_h, k_w);
                        if (!found || bf < g_bf) {
                            g_bf = bf; found = 1;
                            for (int i = 0; i < 5; ++i) best[i] = b[i];
                        }
                    }
    if (found) *best_bf = g_bf;
    return feasible;
}
