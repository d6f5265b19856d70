"""Thin ctypes binding over libcnn.so (declared in include/cnn.h).

Argument marshalling only: every function takes torch CUDA tensors (fp32, contiguous), passes their
device pointers to the C ABI and returns the output tensor.  torch is used for device memory and the
stream, nothing else; there is no CPU or torch fallback -- a missing library is an error.
"""
import ctypes as C
import os

import torch

from . import build as _build

_LIB = None

OP_CONV_FWD, OP_CONV_BWD_DATA, OP_CONV_BWD_WEIGHT, OP_FC_FWD, OP_FC_BWD, OP_CONV_FWD_RELU_POOL = range(6)
EUNSUPPORTED = -2
OPT_FORCE_DIRECT = 0
OPT_PROFILE = 1

_vp, _i, _sz, _f = C.c_void_p, C.c_int, C.c_size_t, C.c_float
_CONV = [_vp] + [_i] * 9 + [_vp] * 3

SIGNATURES = {
    "cnn_create": (_i, [C.POINTER(_vp), _vp]),
    "cnn_destroy": (_i, [_vp]),
    "cnn_set_stream": (_i, [_vp, _vp]),
    "cnn_set_workspace": (_i, [_vp, _vp, _sz]),
    "cnn_set_option": (_i, [_vp, _i, _i]),
    "cnn_workspace_bytes": (_sz, [_i] * 10),
    "cnn_strerror": (C.c_char_p, [_i]),
    "cnn_last_error": (C.c_char_p, [_vp]),
    "cnn_profile_count": (_i, [_vp]),
    "cnn_profile_get": (_i, [_vp, _i, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(C.c_float)]),
    "cnn_profile_reset": (_i, [_vp]),
    "cnn_probe_mfma": (_i, [_vp, _i, _vp, C.POINTER(C.c_double)]),
    "cnn_probe_stream": (_i, [_vp, _i, _sz, _vp, _vp]),
    "cnn_conv_fwd": (_i, _CONV),
    "cnn_conv_bwd_data": (_i, _CONV),
    "cnn_conv_bwd_weight": (_i, _CONV),
    "cnn_conv_bwd_weight_static": (_i, _CONV),
    "cnn_conv_fwd_relu": (_i, _CONV),
    "cnn_conv_bwd_data_relu": (_i, [_vp] + [_i] * 9 + [_vp] * 4),
    "cnn_conv_fwd_relu_pool": (_i, [_vp] + [_i] * 9 + [_vp] * 4),
    "cnn_conv_bwd_data_unpool_relu": (_i, [_vp] + [_i] * 9 + [_vp] * 5),
    "cnn_maxpool2_relu_bwd": (_i, [_vp, _sz, _i, _i, _vp, _vp, _vp, _vp]),
    "cnn_fc_fwd": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp]),
    "cnn_fc_bwd": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "cnn_sgd_update": (_i, [_vp, _sz, _vp, _vp, _vp, _f, _f]),
    "cnn_conv_bwd_weight_sgd": (_i, [_vp] + [_i] * 9 + [_vp] * 4 + [_f, _f]),
    "cnn_conv_transpose_weights": (_i, [_vp] + [_i] * 4 + [_vp] * 2),
    "cnn_conv_bwd_data_wt": (_i, [_vp] + [_i] * 9 + [_vp] * 5),
    "cnn_conv_bwd_weight_sgd_wt": (_i, [_vp] + [_i] * 9 + [_vp] * 5 + [_f, _f]),
    "cnn_fc_bwd_sgd": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _f, _f]),
    "cnn_fc_fwd_act": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _i]),
    "cnn_fc_bwd_act": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _i]),
    "cnn_fc_bwd_sgd_act": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _f, _f, _i]),
    "cnn_conv_bwd_weight_unpool": (_i, [_vp] + [_i] * 9 + [_vp] * 4),
    "cnn_conv_bwd_weight_unpool_sgd": (_i, [_vp] + [_i] * 9 + [_vp] * 5 + [_f, _f]),
    "cnn_bf_plane": (C.c_double, [_i] * 5),
    "cnn_bf_layer": (C.c_double, [_i] * 8),
    "cnn_bf_block_traversal": (C.c_double, [_i] * 8),
    "cnn_block_search": (_i, [_vp] + [_i] * 8 + [C.c_int64, _i, _vp]),
    "cnn_block_search_traversal": (_i, [_vp] + [_i] * 8 + [C.c_int64, C.c_int64, _i, _i, _vp]),
    "cnn_conv_tile_info": (_i, [_i] * 10 + [_vp, C.POINTER(C.c_double)]),
    "cnn_packed_act_elems": (_sz, [_i] * 5),
    "cnn_packed_wt_elems": (_sz, [_i] * 6),
    "cnn_pack_act": (_i, [_vp] + [_i] * 5 + [_vp] * 2),
    "cnn_unpack_act": (_i, [_vp] + [_i] * 5 + [_vp] * 2),
    "cnn_pack_wt": (_i, [_vp] + [_i] * 6 + [_vp] * 2),
    "cnn_unpack_wt": (_i, [_vp] + [_i] * 6 + [_vp] * 2),
    "cnn_relu_fwd": (_i, [_vp, _sz, _vp, _vp]),
    "cnn_relu_bwd": (_i, [_vp, _sz, _vp, _vp, _vp]),
    "cnn_maxpool2_fwd": (_i, [_vp, _sz, _i, _i, _vp, _vp, _vp]),
    "cnn_maxpool2_bwd": (_i, [_vp, _sz, _i, _i, _vp, _vp, _vp]),
    "cnn_sigmoid_fwd": (_i, [_vp, _sz, _vp, _vp]),
    "cnn_sigmoid_bwd": (_i, [_vp, _sz, _vp, _vp, _vp]),
    "cnn_softmax_xent": (_i, [_vp, _i, _i, _vp, _vp, _vp, _vp]),
}


class CnnError(RuntimeError):
    pass


def library_path():
    """The in-tree library, the only one this binding loads."""
    return _build.LIB


def ensure_built():
    """Build the library only if nothing is built (tests, smoke and bench load what is there)."""
    if not os.path.exists(_build.LIB):
        _build.build()
    return _build.LIB


def lib():
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise CnnError(f"{path} is missing: build it with `python -m paper_1602_06709_amd.build` "
                           "(there is no CPU fallback)")
        L = C.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _LIB = L
    return _LIB


def _check(status, ctx=None):
    if status != 0:
        msg = lib().cnn_strerror(status).decode()
        if ctx is not None and status == -4:
            msg += ": " + lib().cnn_last_error(ctx).decode()
        raise CnnError(f"libcnn status {status}: {msg}")


def _t(t, dtype=torch.float32):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise CnnError("expected a contiguous CUDA tensor of dtype %s" % dtype)
    return t.data_ptr()


def out_dim(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


class Context:
    """A cnn_ctx bound to torch's current stream, with a torch-owned workspace that grows on demand."""

    def __init__(self, stream=None):
        self._h = _vp()
        s = stream if stream is not None else torch.cuda.current_stream()
        self.stream = s
        _check(lib().cnn_create(C.byref(self._h), _vp(s.cuda_stream)))
        self._ws = None

    def close(self):
        if self._h:
            lib().cnn_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def set_option(self, option, value):
        _check(lib().cnn_set_option(self._h, option, int(value)))

    def profile(self, on):
        """Turn per-kernel event timing on/off (entries accumulate until profile_reset)."""
        self.set_option(OPT_PROFILE, 1 if on else 0)

    def profile_reset(self):
        _check(lib().cnn_profile_reset(self._h))

    def profile_count(self):
        """Number of profile entries recorded so far (host-side counter)."""
        return lib().cnn_profile_count(self._h)

    def profile_entries(self):
        """[(kernel name, algorithmic flops, milliseconds)] of every kernel launched while profiling was on."""
        out = []
        name, fl, ms = C.c_char_p(), C.c_double(), C.c_float()
        for i in range(lib().cnn_profile_count(self._h)):
            _check(lib().cnn_profile_get(self._h, i, C.byref(name), C.byref(fl), C.byref(ms)), self._h)
            out.append((name.value.decode(), fl.value, ms.value))
        return out

    def reserve(self, nbytes):
        """Make the attached workspace at least nbytes (allocation happens here, never inside the library)."""
        if nbytes and (self._ws is None or self._ws.numel() < nbytes):
            self._ws = torch.empty(int(nbytes), dtype=torch.uint8, device="cuda")
            _check(lib().cnn_set_workspace(self._h, _vp(self._ws.data_ptr()), nbytes))

    def reserve_for(self, op, N, Cc, H, W, K, R, S, stride, pad):
        self.reserve(lib().cnn_workspace_bytes(op, N, Cc, H, W, K, R, S, stride, pad))


# ---------------------------------------------------------------- measurement aids
STREAM_READ, STREAM_WRITE, STREAM_COPY = 0, 1, 2
PROBE_SINK_FLOATS = 512 * 256


def cnn_probe_mfma(ctx, iters, sink):
    """Register-only fp32 matrix-core loop; returns the FLOPs of the launch."""
    assert sink.numel() >= PROBE_SINK_FLOATS
    fl = C.c_double()
    _check(lib().cnn_probe_mfma(ctx.handle, int(iters), _t(sink), C.byref(fl)), ctx.handle)
    return fl.value


def cnn_probe_stream(ctx, mode, src, dst):
    """One read / write / copy pass over dst.numel() floats (src.numel() for a read)."""
    n = src.numel() if mode == STREAM_READ else dst.numel()
    _check(lib().cnn_probe_stream(ctx.handle, mode, n, _t(src) if src is not None else None, _t(dst)), ctx.handle)


# ---------------------------------------------------------------- contractions
def cnn_conv_fwd(ctx, x, w, stride=1, pad=0, out=None, relu=False):
    N, Cc, H, W = x.shape
    K, C2, R, S = w.shape
    assert Cc == C2
    ctx.reserve_for(OP_CONV_FWD, N, Cc, H, W, K, R, S, stride, pad)
    y = out if out is not None else torch.empty((N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)),
                                                dtype=torch.float32, device=x.device)
    fn = lib().cnn_conv_fwd_relu if relu else lib().cnn_conv_fwd
    _check(fn(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(w), _t(y)), ctx.handle)
    return y


def cnn_conv_fwd_relu(ctx, x, w, stride=1, pad=0, out=None):
    return cnn_conv_fwd(ctx, x, w, stride, pad, out, relu=True)


def cnn_conv_fwd_relu_pool(ctx, x, w, stride=1, pad=0, out=None, arg_out=None):
    """maxpool2(relu(conv_fwd(x, w))) and the argmax bytes in one kernel; returns None (nothing launched, outputs
    untouched) when the library does not serve the shape this way."""
    N, Cc, H, W = x.shape
    K, C2, R, S = w.shape
    assert Cc == C2
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    ctx.reserve_for(OP_CONV_FWD_RELU_POOL, N, Cc, H, W, K, R, S, stride, pad)
    a = out if out is not None else torch.empty((N, K, P // 2, Q // 2), dtype=torch.float32, device=x.device)
    arg = arg_out if arg_out is not None else torch.empty((N, K, P // 2, Q // 2), dtype=torch.uint8, device=x.device)
    st = lib().cnn_conv_fwd_relu_pool(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(w), _t(a),
                                      _t(arg, torch.uint8))
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return a, arg


def cnn_conv_bwd_data_unpool_relu(ctx, dy, w, arg, a_pool, stride=1, pad=0, out=None):
    """maxpool2_relu_bwd(conv_bwd_data(dy, w), arg, a_pool) in one kernel; returns None (nothing launched) when the
    library does not serve the shape this way."""
    K, Cc, R, S = w.shape
    N, C2, H, W = a_pool.shape
    assert Cc == C2
    ctx.reserve_for(OP_CONV_BWD_DATA, N, Cc, H, W, K, R, S, stride, pad)
    dz = out if out is not None else torch.empty((N, Cc, 2 * H, 2 * W), dtype=torch.float32, device=dy.device)
    st = lib().cnn_conv_bwd_data_unpool_relu(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(dy), _t(w),
                                             _t(arg, torch.uint8), _t(a_pool), _t(dz))
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return dz


def cnn_conv_bwd_data_relu(ctx, dy, w, x_act, stride=1, pad=0, out=None):
    return cnn_conv_bwd_data(ctx, dy, w, x_act.shape[2], x_act.shape[3], stride, pad, out, x_act=x_act)


def cnn_conv_bwd_data(ctx, dy, w, H, W, stride=1, pad=0, out=None, x_act=None):
    K, Cc, R, S = w.shape
    N = dy.shape[0]
    assert tuple(dy.shape) == (N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad))
    ctx.reserve_for(OP_CONV_BWD_DATA, N, Cc, H, W, K, R, S, stride, pad)
    dx = out if out is not None else torch.empty((N, Cc, H, W), dtype=torch.float32, device=dy.device)
    if x_act is None:
        _check(lib().cnn_conv_bwd_data(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(dy), _t(w), _t(dx)), ctx.handle)
    else:
        assert tuple(x_act.shape) == (N, Cc, H, W)
        _check(lib().cnn_conv_bwd_data_relu(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(dy), _t(w), _t(x_act),
                                            _t(dx)), ctx.handle)
    return dx


def cnn_conv_bwd_weight(ctx, x, dy, R, S, stride=1, pad=0, out=None):
    N, Cc, H, W = x.shape
    K = dy.shape[1]
    assert tuple(dy.shape) == (N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad))
    ctx.reserve_for(OP_CONV_BWD_WEIGHT, N, Cc, H, W, K, R, S, stride, pad)
    dw = out if out is not None else torch.empty((K, Cc, R, S), dtype=torch.float32, device=x.device)
    _check(lib().cnn_conv_bwd_weight(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(dy), _t(dw)), ctx.handle)
    return dw


STATIC_SCRATCH_BYTES = 80 << 20


def cnn_conv_bwd_weight_static(ctx, x, dy, R, S, stride, pad, out):
    """cnn_conv_bwd_weight on the library's built-in scratch array: no workspace is reserved and nothing is
    allocated here or in the library, so the caller passes the output tensor."""
    N, Cc, H, W = x.shape
    K = dy.shape[1]
    assert tuple(dy.shape) == (N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad))
    assert tuple(out.shape) == (K, Cc, R, S)
    _check(lib().cnn_conv_bwd_weight_static(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(dy), _t(out)),
           ctx.handle)
    return out


def cnn_fc_fwd(ctx, x, w, out=None):
    N, I = x.shape
    O, I2 = w.shape
    assert I == I2
    ctx.reserve_for(OP_FC_FWD, N, I, 1, 1, O, 1, 1, 1, 0)
    y = out if out is not None else torch.empty((N, O), dtype=torch.float32, device=x.device)
    _check(lib().cnn_fc_fwd(ctx.handle, N, I, O, _t(x), _t(w), _t(y)), ctx.handle)
    return y


def cnn_fc_bwd(ctx, x, w, dy, need_dx=True, need_dw=True, dx_out=None, dw_out=None):
    N, O = dy.shape
    I = w.shape[1] if w is not None else x.shape[1]
    ctx.reserve_for(OP_FC_BWD, N, I, 1, 1, O, 1, 1, 1, 0)
    dx = dw = None
    if need_dx:
        dx = dx_out if dx_out is not None else torch.empty((N, I), dtype=torch.float32, device=dy.device)
    if need_dw:
        dw = dw_out if dw_out is not None else torch.empty((O, I), dtype=torch.float32, device=dy.device)
    _check(lib().cnn_fc_bwd(ctx.handle, N, I, O, _t(x) if x is not None else None, _t(w) if w is not None else None,
                            _t(dy), _t(dx) if dx is not None else None, _t(dw) if dw is not None else None),
           ctx.handle)
    return dx, dw


ACT = {None: 0, "none": 0, "relu": 1, "sigmoid": 2}


def cnn_fc_fwd_act(ctx, x, w, act, out=None):
    """act(x W^T) in one call; returns None (nothing launched) where the library does not serve the shape this way."""
    N, I = x.shape
    O, I2 = w.shape
    assert I == I2
    ctx.reserve_for(OP_FC_FWD, N, I, 1, 1, O, 1, 1, 1, 0)
    a = out if out is not None else torch.empty((N, O), dtype=torch.float32, device=x.device)
    st = lib().cnn_fc_fwd_act(ctx.handle, N, I, O, _t(x), _t(w), _t(a), ACT[act])
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return a


def cnn_fc_bwd_act(ctx, x, w, dy, act_in, need_dw=True, dz_out=None, dw_out=None):
    """cnn_fc_bwd for a layer whose input x is the output of `act_in`: dz is the gradient in front of that activation.
    Returns None (nothing launched) where the library does not serve the shape this way, else (dz, dw)."""
    N, O = dy.shape
    I = w.shape[1]
    ctx.reserve_for(OP_FC_BWD, N, I, 1, 1, O, 1, 1, 1, 0)
    dz = dz_out if dz_out is not None else torch.empty((N, I), dtype=torch.float32, device=dy.device)
    dw = None
    if need_dw:
        dw = dw_out if dw_out is not None else torch.empty((O, I), dtype=torch.float32, device=dy.device)
    st = lib().cnn_fc_bwd_act(ctx.handle, N, I, O, _t(x), _t(w), _t(dy), _t(dz), _t(dw) if dw is not None else None,
                              ACT[act_in])
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return dz, dw


def cnn_fc_bwd_sgd_act(ctx, x, w, dy, act_in, v=None, dz_out=None, lr=0.01, momentum=0.0):
    """cnn_fc_bwd_sgd with the derivative of the activation that produced x folded into dz.  None where unsupported."""
    N, O = dy.shape
    I = w.shape[1]
    assert tuple(x.shape) == (N, I) and w.shape[0] == O and (v is None or tuple(v.shape) == tuple(w.shape))
    ctx.reserve_for(OP_FC_BWD, N, I, 1, 1, O, 1, 1, 1, 0)
    dz = dz_out if dz_out is not None else torch.empty((N, I), dtype=torch.float32, device=dy.device)
    st = lib().cnn_fc_bwd_sgd_act(ctx.handle, N, I, O, _t(x), _t(w), _t(dy), _t(dz), _t(v) if v is not None else None,
                                  lr, momentum, ACT[act_in])
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return dz, w


def cnn_sgd_update(ctx, w, dw, v=None, lr=0.01, momentum=0.0):
    """In place on w (and v).  w, dw, v are flat views of equal length."""
    n = w.numel()
    assert dw.numel() == n and (v is None or v.numel() == n)
    _check(lib().cnn_sgd_update(ctx.handle, n, _t(w), _t(dw), _t(v) if v is not None else None, lr, momentum),
           ctx.handle)
    return w


def cnn_conv_bwd_weight_sgd(ctx, x, dy, w, v=None, stride=1, pad=0, lr=0.01, momentum=0.0):
    """The weight gradient of (x, dy) applied to w (and v) in place, without storing it; returns None (nothing
    launched, w untouched) when the library does not serve the shape this way."""
    N, Cc, H, W = x.shape
    K, C2, R, S = w.shape
    assert Cc == C2 and (v is None or tuple(v.shape) == tuple(w.shape))
    assert tuple(dy.shape) == (N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad))
    ctx.reserve_for(OP_CONV_BWD_WEIGHT, N, Cc, H, W, K, R, S, stride, pad)
    st = lib().cnn_conv_bwd_weight_sgd(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(dy), _t(w),
                                       _t(v) if v is not None else None, lr, momentum)
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return w


def cnn_conv_transpose_weights(ctx, w, out=None):
    """wT[c][k][r][s] = w[k][c][R-1-r][S-1-s] (Section 2.3's transpose-weights with mirrored taps); None where the
    library does not serve the kernel size."""
    K, Cc, R, S = w.shape
    wT = out if out is not None else torch.empty((Cc, K, R, S), dtype=torch.float32, device=w.device)
    st = lib().cnn_conv_transpose_weights(ctx.handle, K, Cc, R, S, _t(w), _t(wT))
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return wT


def cnn_conv_bwd_data_wt(ctx, dy, wT, H, W, stride=1, pad=0, x_act=None, arg=None, out=None):
    """Backpropagation from the resident transpose-weights; x_act / arg select the ReLU and un-pool + ReLU forms (then
    out is [N][C][2H][2W]).  None (nothing launched) where the tiled kernel does not serve the layer."""
    Cc, K, R, S = wT.shape
    N = dy.shape[0]
    assert tuple(dy.shape) == (N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad))
    ctx.reserve_for(OP_CONV_BWD_DATA, N, Cc, H, W, K, R, S, stride, pad)
    shape = (N, Cc, 2 * H, 2 * W) if arg is not None else (N, Cc, H, W)
    dz = out if out is not None else torch.empty(shape, dtype=torch.float32, device=dy.device)
    assert tuple(dz.shape) == shape
    st = lib().cnn_conv_bwd_data_wt(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(dy), _t(wT),
                                    _t(x_act) if x_act is not None else None,
                                    _t(arg, torch.uint8) if arg is not None else None, _t(dz))
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return dz


def cnn_conv_bwd_weight_sgd_wt(ctx, x, dy, w, wT, v=None, stride=1, pad=0, lr=0.01, momentum=0.0):
    """cnn_conv_bwd_weight_sgd that also keeps the resident transpose-weights wT current; None where unsupported."""
    N, Cc, H, W = x.shape
    K, C2, R, S = w.shape
    assert Cc == C2 and tuple(wT.shape) == (Cc, K, R, S) and (v is None or tuple(v.shape) == tuple(w.shape))
    assert tuple(dy.shape) == (N, K, out_dim(H, R, stride, pad), out_dim(W, S, stride, pad))
    ctx.reserve_for(OP_CONV_BWD_WEIGHT, N, Cc, H, W, K, R, S, stride, pad)
    st = lib().cnn_conv_bwd_weight_sgd_wt(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(dy), _t(w),
                                          _t(v) if v is not None else None, _t(wT), lr, momentum)
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return w


OP_CONV_BWD_WEIGHT_UNPOOL = 7


def conv_bwd_weight_unpool_serves(N, Cc, H, W, K, R, S, stride, pad):
    return lib().cnn_workspace_bytes(OP_CONV_BWD_WEIGHT_UNPOOL, N, Cc, H, W, K, R, S, stride, pad) > 0


def cnn_conv_bwd_weight_unpool(ctx, x, dpool, arg, R, S, stride=1, pad=0, out=None, w=None, v=None, lr=0.01, momentum=0.0):
    """dw = conv_bwd_weight(x, maxpool2_bwd(dpool, arg)) without the full-size gradient; with w given, the SGD step
    on w (and v) instead of storing dw.  Returns None (nothing launched) where the library does not serve the shape."""
    N, Cc, H, W = x.shape
    K = dpool.shape[1]
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    assert tuple(dpool.shape) == (N, K, P // 2, Q // 2) and tuple(arg.shape) == tuple(dpool.shape)
    ctx.reserve_for(OP_CONV_BWD_WEIGHT_UNPOOL, N, Cc, H, W, K, R, S, stride, pad)
    if w is not None:
        st = lib().cnn_conv_bwd_weight_unpool_sgd(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(dpool),
                                                  _t(arg, torch.uint8), _t(w), _t(v) if v is not None else None, lr, momentum)
        res = w
    else:
        res = out if out is not None else torch.empty((K, Cc, R, S), dtype=torch.float32, device=x.device)
        st = lib().cnn_conv_bwd_weight_unpool(ctx.handle, N, Cc, H, W, K, R, S, stride, pad, _t(x), _t(dpool),
                                              _t(arg, torch.uint8), _t(res))
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return res


def cnn_fc_bwd_sgd(ctx, x, w, dy, v=None, need_dx=True, dx_out=None, lr=0.01, momentum=0.0):
    """dx from the old w (when asked for), then the weight gradient applied to w (and v) in place; returns None
    (nothing launched) when the library does not serve the shape this way, else (dx, w)."""
    N, O = dy.shape
    I = w.shape[1]
    assert tuple(x.shape) == (N, I) and w.shape[0] == O and (v is None or tuple(v.shape) == tuple(w.shape))
    ctx.reserve_for(OP_FC_BWD, N, I, 1, 1, O, 1, 1, 1, 0)
    dx = None
    if need_dx:
        dx = dx_out if dx_out is not None else torch.empty((N, I), dtype=torch.float32, device=dy.device)
    st = lib().cnn_fc_bwd_sgd(ctx.handle, N, I, O, _t(x), _t(w), _t(dy), _t(dx) if dx is not None else None,
                              _t(v) if v is not None else None, lr, momentum)
    if st == EUNSUPPORTED:
        return None
    _check(st, ctx.handle)
    return dx, w


# ---------------------------------------------------------------- cache-blocking model (Section 2.2)
OP_BLOCK_SEARCH = 6


def _block_result(buf, n):
    """(block tuple or None, B/F, feasible count) from the 48-byte cnn_block_result in `buf` (a uint8 tensor)."""
    import numpy as np
    raw = buf.cpu().numpy().tobytes()
    blk = np.frombuffer(raw, np.int32, 8, 0)
    bf = float(np.frombuffer(raw, np.float64, 1, 32)[0])
    feasible = int(np.frombuffer(raw, np.uint64, 1, 40)[0])
    return (tuple(int(v) for v in blk[:n]) if blk[7] else None), bf, feasible


def cnn_block_search(ctx, layer, cache_bytes, simd):
    """layer = (minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride).  Returns (block[7] or None, B/F, feasible)."""
    ctx.reserve_for(OP_BLOCK_SEARCH, 1, 1, 1, 1, 1, 1, 1, 1, 0)
    res = torch.zeros(48, dtype=torch.uint8, device="cuda")
    _check(lib().cnn_block_search(ctx.handle, *[int(v) for v in layer], int(cache_bytes), int(simd), res.data_ptr()),
           ctx.handle)
    return _block_result(res, 7)


def cnn_block_search_traversal(ctx, layer, acc_bytes, stage_bytes, simd, chunk):
    """Returns (block[5] = (images, ofm block, ifm chunk, rows, cols) or None, B/F, feasible)."""
    ctx.reserve_for(OP_BLOCK_SEARCH, 1, 1, 1, 1, 1, 1, 1, 1, 0)
    res = torch.zeros(48, dtype=torch.uint8, device="cuda")
    _check(lib().cnn_block_search_traversal(ctx.handle, *[int(v) for v in layer], int(acc_bytes), int(stage_bytes),
                                            int(simd), int(chunk), res.data_ptr()), ctx.handle)
    return _block_result(res, 5)


def cnn_conv_tile_info(op, N, Cc, H, W, K, R, S, stride, pad):
    """(tile[8], B/F) of the planner's tile for a convolution pass, or None where the tiled kernel does not serve."""
    tile = (C.c_int32 * 8)()
    bf = C.c_double(0.0)
    st = lib().cnn_conv_tile_info(op, N, Cc, H, W, K, R, S, stride, pad, C.cast(tile, C.c_void_p), C.byref(bf))
    if st == EUNSUPPORTED:
        return None
    _check(st, None)
    return list(tile), bf.value


# ---------------------------------------------------------------- layouts (Section 2.3)
def cnn_pack_act(ctx, x, sw):
    N, Cc, H, W = x.shape
    out = torch.empty((N, (Cc + sw - 1) // sw, H, W, sw), dtype=torch.float32, device=x.device)
    assert out.numel() == lib().cnn_packed_act_elems(N, Cc, H, W, sw)
    _check(lib().cnn_pack_act(ctx.handle, N, Cc, H, W, sw, _t(x), _t(out)), ctx.handle)
    return out


def cnn_unpack_act(ctx, packed, Cc):
    N, CB, H, W, sw = packed.shape
    out = torch.empty((N, Cc, H, W), dtype=torch.float32, device=packed.device)
    _check(lib().cnn_unpack_act(ctx.handle, N, Cc, H, W, sw, _t(packed), _t(out)), ctx.handle)
    return out


def cnn_pack_wt(ctx, w, sw, transpose=False):
    K, Cc, R, S = w.shape
    shape = (K, (Cc + sw - 1) // sw, R, S, sw) if transpose else (Cc, (K + sw - 1) // sw, R, S, sw)
    out = torch.empty(shape, dtype=torch.float32, device=w.device)
    assert out.numel() == lib().cnn_packed_wt_elems(K, Cc, R, S, sw, int(transpose))
    _check(lib().cnn_pack_wt(ctx.handle, K, Cc, R, S, sw, int(transpose), _t(w), _t(out)), ctx.handle)
    return out


def cnn_unpack_wt(ctx, packed, K, Cc, transpose=False):
    _, _, R, S, sw = packed.shape
    out = torch.empty((K, Cc, R, S), dtype=torch.float32, device=packed.device)
    _check(lib().cnn_unpack_wt(ctx.handle, K, Cc, R, S, sw, int(transpose), _t(packed), _t(out)), ctx.handle)
    return out


# ---------------------------------------------------------------- glue
def cnn_relu_fwd(ctx, z, out=None):
    a = out if out is not None else torch.empty_like(z)
    _check(lib().cnn_relu_fwd(ctx.handle, z.numel(), _t(z), _t(a)), ctx.handle)
    return a


def cnn_relu_bwd(ctx, z, da, out=None):
    dz = out if out is not None else torch.empty_like(z)
    _check(lib().cnn_relu_bwd(ctx.handle, z.numel(), _t(z), _t(da), _t(dz)), ctx.handle)
    return dz


def cnn_maxpool2_fwd(ctx, x, out=None, arg_out=None):
    N, Cc, H, W = x.shape
    y = out if out is not None else torch.empty((N, Cc, H // 2, W // 2), dtype=torch.float32, device=x.device)
    arg = arg_out if arg_out is not None else torch.empty((N, Cc, H // 2, W // 2), dtype=torch.uint8, device=x.device)
    _check(lib().cnn_maxpool2_fwd(ctx.handle, N * Cc, H, W, _t(x), _t(y), _t(arg, torch.uint8)), ctx.handle)
    return y, arg


def cnn_maxpool2_bwd(ctx, dy, arg, H, W, out=None):
    N, Cc = dy.shape[:2]
    dx = out if out is not None else torch.empty((N, Cc, H, W), dtype=torch.float32, device=dy.device)
    _check(lib().cnn_maxpool2_bwd(ctx.handle, N * Cc, H, W, _t(dy), _t(arg, torch.uint8), _t(dx)), ctx.handle)
    return dx


def cnn_maxpool2_relu_bwd(ctx, dy, arg, y, H, W, out=None):
    N, Cc = dy.shape[:2]
    dz = out if out is not None else torch.empty((N, Cc, H, W), dtype=torch.float32, device=dy.device)
    _check(lib().cnn_maxpool2_relu_bwd(ctx.handle, N * Cc, H, W, _t(dy), _t(arg, torch.uint8), _t(y), _t(dz)), ctx.handle)
    return dz


def cnn_sigmoid_fwd(ctx, z, out=None):
    a = out if out is not None else torch.empty_like(z)
    _check(lib().cnn_sigmoid_fwd(ctx.handle, z.numel(), _t(z), _t(a)), ctx.handle)
    return a


def cnn_sigmoid_bwd(ctx, a, da, out=None):
    dz = out if out is not None else torch.empty_like(a)
    _check(lib().cnn_sigmoid_bwd(ctx.handle, a.numel(), _t(a), _t(da), _t(dz)), ctx.handle)
    return dz


def cnn_softmax_xent(ctx, z, label, loss_out=None, dz_out=None):
    N, O = z.shape
    loss = loss_out if loss_out is not None else torch.empty((N,), dtype=torch.float32, device=z.device)
    dz = dz_out if dz_out is not None else torch.empty_like(z)
    _check(lib().cnn_softmax_xent(ctx.handle, N, O, _t(z), _t(label, torch.int32), _t(loss), _t(dz)), ctx.handle)
    return loss, dz
