"""CPU oracle for the cache-blocking model of arxiv 1602.06709, Section 2.2 (bytes-to-FLOPs ratios of a
convolution layer, of a block of it, and the exhaustive search for the block of least B/F that fits a cache).

TEST INFRASTRUCTURE ONLY; the arithmetic lives in blocking_oracle.c, this module marshals arguments.
A layer is (minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride); a block of the single-cache model is
(b1_0 images, b1_1 output features, b2_0 input features, b1_2, b1_3 output pixels, b2_2, b2_3 kernel taps);
a block of the traversal model is its first five entries.
"""
import ctypes as C

import numpy as np

from . import lib as _lib

_ready = False


def _L():
    global _ready
    L = _lib()
    if not _ready:
        L.oracle_bf_plane.restype = C.c_double
        L.oracle_bf_layer.restype = C.c_double
        for f in ("oracle_bf_block_bytes", "oracle_bf_block_flops", "oracle_bf_trav_bytes", "oracle_bf_trav_flops",
                  "oracle_bf_trav_stage_bytes"):
            getattr(L, f).restype = C.c_int64
        L.oracle_bf_search.restype = C.c_uint64
        L.oracle_bf_trav_search.restype = C.c_uint64
        _ready = True
    return L


def _blk(b, n):
    a = np.ascontiguousarray(np.asarray(b, dtype=np.int32))
    assert a.shape == (n,)
    return a, a.ctypes.data_as(C.c_void_p)


def bf_plane(out_h, out_w, k_h, k_w, stride=1, size_data=4):
    return _L().oracle_bf_plane(out_h, out_w, k_h, k_w, stride, size_data)


def bf_layer(minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride=1, size_data=4):
    return _L().oracle_bf_layer(minibatch, ifm, ofm, out_h, out_w, k_h, k_w, stride, size_data)


def block_bytes(block, stride=1, size_data=4):
    a, p = _blk(block, 7)
    return _L().oracle_bf_block_bytes(p, stride, size_data)


def block_flops(block):
    a, p = _blk(block, 7)
    return _L().oracle_bf_block_flops(p)


def block_bf(block, stride=1, size_data=4):
    return block_bytes(block, stride, size_data) / block_flops(block)


def search(layer, cache_bytes, simd, size_data=4):
    """Exhaustive search; returns (block[7] or None, B/F, number of feasible blocks)."""
    n, c, k, p, q, r, s, st = layer
    best = np.zeros(7, np.int32)
    bf = C.c_double(0.0)
    cnt = _L().oracle_bf_search(n, c, k, p, q, r, s, st, size_data, C.c_int64(cache_bytes), simd,
                                best.ctypes.data_as(C.c_void_p), C.byref(bf))
    return (best if cnt else None), bf.value, cnt


def trav_bytes(block, ifm, k_h, k_w, stride=1, size_data=4):
    a, p = _blk(block, 5)
    return _L().oracle_bf_trav_bytes(p, ifm, k_h, k_w, stride, size_data)


def trav_flops(block, ifm, k_h, k_w):
    a, p = _blk(block, 5)
    return _L().oracle_bf_trav_flops(p, ifm, k_h, k_w)


def trav_stage_bytes(block, k_h, k_w, stride=1, size_data=4):
    a, p = _blk(block, 5)
    return _L().oracle_bf_trav_stage_bytes(p, k_h, k_w, stride, size_data)


def trav_search(layer, acc_bytes, stage_bytes, simd, chunk, size_data=4):
    """Exhaustive search of the traversal model; returns (block[5] or None, B/F, number of feasible blocks)."""
    n, c, k, p, q, r, s, st = layer
    best = np.zeros(5, np.int32)
    bf = C.c_double(0.0)
    cnt = _L().oracle_bf_trav_search(n, c, k, p, q, r, s, st, size_data, C.c_int64(acc_bytes), C.c_int64(stage_bytes),
                                     simd, chunk, best.ctypes.data_as(C.c_void_p), C.byref(bf))
    return (best if cnt else None), bf.value, cnt
