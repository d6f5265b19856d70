"""Runs a layer list through the oracle ops (test infrastructure: CPU baseline timing and end-to-end checks).

Between layers the fp64 results are rounded to fp32, as the tensors of an fp32 training run are."""
import time

import numpy as np

import oracle


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def run_step(layers, x, weights, labels=None, upstream=None, timings=None):
    """forward, loss (if labels) and backward in the paper's order (weight gradient before backpropagation,
    the first layer skips backpropagation).  Returns (activations, weight gradients, loss)."""
    acts, args = [], {}
    cur, wi = _f32(x), 0

    def timed(kind, fn):
        t0 = time.perf_counter()
        r = fn()
        if timings is not None:
            timings[kind] = timings.get(kind, 0.0) + time.perf_counter() - t0
        return r

    for i, L in enumerate(layers):
        k = L[0]
        if k == "conv":
            cur = _f32(timed("conv_fwd", lambda: oracle.conv_fwd(cur, weights[wi], L[5], L[6]))); wi += 1
        elif k == "fc":
            cur = _f32(timed("fc_fwd", lambda: oracle.fc_fwd(cur, weights[wi]))); wi += 1
        elif k == "relu":
            cur = _f32(timed("glue", lambda: oracle.relu_fwd(cur)))
        elif k == "sigmoid":
            cur = _f32(timed("glue", lambda: oracle.sigmoid_fwd(cur)))
        elif k == "pool":
            y, a = timed("glue", lambda: oracle.maxpool2_fwd(cur)); args[i] = a; cur = _f32(y)
        elif k == "flatten":
            cur = cur.reshape(cur.shape[0], -1)
        acts.append(cur)
    loss = None
    if labels is not None:
        loss, g = timed("glue", lambda: oracle.softmax_xent(acts[-1], labels)); g = _f32(g)
    else:
        g = _f32(upstream)
    dws = [None] * len(weights)
    for i in range(len(layers) - 1, -1, -1):
        L, k = layers[i], layers[i][0]
        xin = _f32(x) if i == 0 else acts[i - 1]
        if k == "conv":
            wi -= 1
            dws[wi] = timed("conv_bwd_weight", lambda: oracle.conv_bwd_weight(xin, g, L[3], L[4], L[5], L[6]))
            if i:
                g = _f32(timed("conv_bwd_data", lambda: oracle.conv_bwd_data(g, weights[wi], xin.shape[2], xin.shape[3], L[5], L[6])))
        elif k == "fc":
            wi -= 1
            dws[wi] = timed("fc_bwd", lambda: oracle.fc_bwd_weight(xin, g))
            if i:
                g = _f32(timed("fc_bwd", lambda: oracle.fc_bwd_data(g, weights[wi])))
        elif k == "relu":
            g = _f32(timed("glue", lambda: oracle.relu_bwd(xin, g)))
        elif k == "sigmoid":
            g = _f32(timed("glue", lambda: oracle.sigmoid_bwd(acts[i], g)))
        elif k == "pool":
            g = _f32(timed("glue", lambda: oracle.maxpool2_bwd(g, args[i], xin.shape[2], xin.shape[3])))
        elif k == "flatten":
            g = g.reshape(xin.shape)
    return acts, dws, loss
