"""CPU oracle for the conv / FC / SGD training path of arxiv 1602.06709.

TEST INFRASTRUCTURE ONLY.  A plain fp64 loop-nest implementation (C, OpenMP on
the outermost loop) of Section 2.1's three convolution passes, the
fully-connected special case, the SGD update, Section 2.3's blocked layouts and
the glue ops the network workloads need.  It shares nothing with the GPU
library; only tests, the smoke check and the benchmark's CPU-baseline leg may
import it.

All functions take numpy float32 arrays in canonical layouts (NCHW
activations, KCRS weights, [N][I] / [O][I] for FC) and return float64 arrays.
Contractions return (result, S) with S = sum |a*b| over the same terms when
`with_abs=True`.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _lib.oracle_softmax_xent.restype = C.c_double
        _lib.oracle_conv_flops_per_pass.restype = C.c_double
        _lib.oracle_out_dim.restype = C.c_int
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def num_threads():
    return int(lib().oracle_num_threads())


def out_dim(n, k, stride, pad):
    return int(lib().oracle_out_dim(int(n), int(k), int(stride), int(pad)))


def _ret(y, s, with_abs):
    return (y, s) if with_abs else y


def conv_fwd(x, w, stride=1, pad=0, with_abs=False):
    x, w = _f32(x), _f32(w)
    N, Cc, H, W = x.shape
    K, C2, R, S = w.shape
    assert Cc == C2
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    y = np.empty((N, K, P, Q), np.float64)
    s = np.empty_like(y) if with_abs else None
    lib().oracle_conv_fwd(N, Cc, H, W, K, R, S, stride, pad, _p(x), _p(w), _p(y), _p(s))
    return _ret(y, s, with_abs)


def conv_bwd_data(dy, w, H, W, stride=1, pad=0, with_abs=False):
    dy, w = _f32(dy), _f32(w)
    K, Cc, R, S = w.shape
    N = dy.shape[0]
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    assert dy.shape == (N, K, P, Q), (dy.shape, (N, K, P, Q))
    dx = np.empty((N, Cc, H, W), np.float64)
    s = np.empty_like(dx) if with_abs else None
    lib().oracle_conv_bwd_data(N, Cc, H, W, K, R, S, stride, pad, _p(dy), _p(w), _p(dx), _p(s))
    return _ret(dx, s, with_abs)


def conv_bwd_weight(x, dy, R, S, stride=1, pad=0, with_abs=False):
    x, dy = _f32(x), _f32(dy)
    N, Cc, H, W = x.shape
    K = dy.shape[1]
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    assert dy.shape == (N, K, P, Q), (dy.shape, (N, K, P, Q))
    dw = np.empty((K, Cc, R, S), np.float64)
    s = np.empty_like(dw) if with_abs else None
    lib().oracle_conv_bwd_weight(N, Cc, H, W, K, R, S, stride, pad, _p(x), _p(dy), _p(dw), _p(s))
    return _ret(dw, s, with_abs)


def _idx(idx):
    return np.ascontiguousarray(idx, dtype=np.int64).ravel()


def conv_fwd_at(x, w, idx, stride=1, pad=0):
    """(values, S) of conv_fwd at flat indices into y[N][K][P][Q]."""
    x, w, idx = _f32(x), _f32(w), _idx(idx)
    N, Cc, H, W = x.shape
    K, _, R, S = w.shape
    out = np.empty(idx.size, np.float64); s = np.empty(idx.size, np.float64)
    lib().oracle_conv_fwd_at(N, Cc, H, W, K, R, S, stride, pad, _p(x), _p(w),
                             C.c_size_t(idx.size), _p(idx), _p(out), _p(s))
    return out, s


def conv_bwd_data_at(dy, w, H, W, idx, stride=1, pad=0):
    """(values, S) of conv_bwd_data at flat indices into dx[N][C][H][W]."""
    dy, w, idx = _f32(dy), _f32(w), _idx(idx)
    K, Cc, R, S = w.shape
    N = dy.shape[0]
    out = np.empty(idx.size, np.float64); s = np.empty(idx.size, np.float64)
    lib().oracle_conv_bwd_data_at(N, Cc, H, W, K, R, S, stride, pad, _p(dy), _p(w),
                                  C.c_size_t(idx.size), _p(idx), _p(out), _p(s))
    return out, s


def conv_bwd_weight_at(x, dy, R, S, idx, stride=1, pad=0):
    """(values, S) of conv_bwd_weight at flat indices into dw[K][C][R][S]."""
    x, dy, idx = _f32(x), _f32(dy), _idx(idx)
    N, Cc, H, W = x.shape
    K = dy.shape[1]
    out = np.empty(idx.size, np.float64); s = np.empty(idx.size, np.float64)
    lib().oracle_conv_bwd_weight_at(N, Cc, H, W, K, R, S, stride, pad, _p(x), _p(dy),
                                    C.c_size_t(idx.size), _p(idx), _p(out), _p(s))
    return out, s


def fc_fwd(x, w, with_abs=False):
    x, w = _f32(x), _f32(w)
    N, I = x.shape
    O, I2 = w.shape
    assert I == I2
    y = np.empty((N, O), np.float64)
    s = np.empty_like(y) if with_abs else None
    lib().oracle_fc_fwd(N, I, O, _p(x), _p(w), _p(y), _p(s))
    return _ret(y, s, with_abs)


def fc_bwd_data(dy, w, with_abs=False):
    dy, w = _f32(dy), _f32(w)
    N, O = dy.shape
    O2, I = w.shape
    assert O == O2
    dx = np.empty((N, I), np.float64)
    s = np.empty_like(dx) if with_abs else None
    lib().oracle_fc_bwd_data(N, I, O, _p(dy), _p(w), _p(dx), _p(s))
    return _ret(dx, s, with_abs)


def fc_bwd_weight(x, dy, with_abs=False):
    x, dy = _f32(x), _f32(dy)
    N, I = x.shape
    N2, O = dy.shape
    assert N == N2
    dw = np.empty((O, I), np.float64)
    s = np.empty_like(dw) if with_abs else None
    lib().oracle_fc_bwd_weight(N, I, O, _p(x), _p(dy), _p(dw), _p(s))
    return _ret(dw, s, with_abs)


def fc_fwd_at(x, w, idx):
    x, w, idx = _f32(x), _f32(w), _idx(idx)
    N, I = x.shape; O = w.shape[0]
    out = np.empty(idx.size, np.float64); s = np.empty(idx.size, np.float64)
    lib().oracle_fc_fwd_at(N, I, O, _p(x), _p(w), C.c_size_t(idx.size), _p(idx), _p(out), _p(s))
    return out, s


def fc_bwd_data_at(dy, w, idx):
    dy, w, idx = _f32(dy), _f32(w), _idx(idx)
    N, O = dy.shape; I = w.shape[1]
    out = np.empty(idx.size, np.float64); s = np.empty(idx.size, np.float64)
    lib().oracle_fc_bwd_data_at(N, I, O, _p(dy), _p(w), C.c_size_t(idx.size), _p(idx), _p(out), _p(s))
    return out, s


def fc_bwd_weight_at(x, dy, idx):
    x, dy, idx = _f32(x), _f32(dy), _idx(idx)
    N, I = x.shape; O = dy.shape[1]
    out = np.empty(idx.size, np.float64); s = np.empty(idx.size, np.float64)
    lib().oracle_fc_bwd_weight_at(N, I, O, _p(x), _p(dy), C.c_size_t(idx.size), _p(idx), _p(out), _p(s))
    return out, s


def sgd_update(w, g, v=None, lr=0.01, momentum=0.0):
    """Returns (w_new, v_new) in fp64; v_new is None when v is None."""
    w, g = _f32(w).ravel(), _f32(g).ravel()
    assert w.size == g.size
    wo = np.empty(w.size, np.float64)
    if v is not None:
        v = _f32(v).ravel()
        vo = np.empty(w.size, np.float64)
    else:
        vo = None
    lib().oracle_sgd_update(C.c_size_t(w.size), _p(w), _p(g), _p(v), C.c_double(lr),
                            C.c_double(momentum), _p(wo), _p(vo))
    return wo, vo


def pack_act(x, sw):
    x = _f32(x)
    N, Cc, H, W = x.shape
    out = np.empty((N, (Cc + sw - 1) // sw, H, W, sw), np.float32)
    lib().oracle_pack_act(N, Cc, H, W, sw, _p(x), _p(out))
    return out


def unpack_act(packed, Cc):
    packed = _f32(packed)
    N, CB, H, W, sw = packed.shape
    out = np.empty((N, Cc, H, W), np.float32)
    lib().oracle_unpack_act(N, Cc, H, W, sw, _p(packed), _p(out))
    return out


def pack_wt(w, sw, transpose=False):
    w = _f32(w)
    K, Cc, R, S = w.shape
    shape = (K, (Cc + sw - 1) // sw, R, S, sw) if transpose else (Cc, (K + sw - 1) // sw, R, S, sw)
    out = np.empty(shape, np.float32)
    lib().oracle_pack_wt(K, Cc, R, S, sw, int(transpose), _p(w), _p(out))
    return out


def unpack_wt(packed, K, Cc, transpose=False):
    packed = _f32(packed)
    _, _, R, S, sw = packed.shape
    out = np.empty((K, Cc, R, S), np.float32)
    lib().oracle_unpack_wt(K, Cc, R, S, sw, int(transpose), _p(packed), _p(out))
    return out


def relu_fwd(z):
    z = _f32(z); a = np.empty(z.shape, np.float64)
    lib().oracle_relu_fwd(C.c_size_t(z.size), _p(z), _p(a))
    return a


def relu_bwd(z, da):
    z, da = _f32(z), _f32(da); dz = np.empty(z.shape, np.float64)
    lib().oracle_relu_bwd(C.c_size_t(z.size), _p(z), _p(da), _p(dz))
    return dz


def maxpool2_fwd(x):
    x = _f32(x)
    N, Cc, H, W = x.shape
    assert H % 2 == 0 and W % 2 == 0
    y = np.empty((N, Cc, H // 2, W // 2), np.float64)
    arg = np.empty((N, Cc, H // 2, W // 2), np.int32)
    lib().oracle_maxpool2_fwd(C.c_size_t(N * Cc), H, W, _p(x), _p(y), _p(arg))
    return y, arg


def maxpool2_bwd(dy, arg, H, W):
    dy = _f32(dy); arg = np.ascontiguousarray(arg, dtype=np.int32)
    N, Cc = dy.shape[:2]
    dx = np.empty((N, Cc, H, W), np.float64)
    lib().oracle_maxpool2_bwd(C.c_size_t(N * Cc), H, W, _p(dy), _p(arg), _p(dx))
    return dx


def sigmoid_fwd(z):
    z = _f32(z); a = np.empty(z.shape, np.float64)
    lib().oracle_sigmoid_fwd(C.c_size_t(z.size), _p(z), _p(a))
    return a


def sigmoid_bwd(a, da):
    a, da = _f32(a), _f32(da); dz = np.empty(a.shape, np.float64)
    lib().oracle_sigmoid_bwd(C.c_size_t(a.size), _p(a), _p(da), _p(dz))
    return dz


def softmax_xent(z, label):
    """Returns (mean loss, dz) with dz = (softmax - onehot)/N."""
    z = _f32(z); label = np.ascontiguousarray(label, dtype=np.int32)
    N, O = z.shape
    dz = np.empty((N, O), np.float64)
    loss = lib().oracle_softmax_xent(N, O, _p(z), _p(label), _p(dz))
    return float(loss), dz


def conv_flops_per_pass(N, Cc, H, W, K, R, S, stride, pad):
    return float(lib().oracle_conv_flops_per_pass(N, Cc, H, W, K, R, S, stride, pad))


def fc_flops_per_pass(N, I, O):
    """The same formula with k_h = k_w = out_h = out_w = 1."""
    return conv_flops_per_pass(N, I, 1, 1, O, 1, 1, 1, 0)
