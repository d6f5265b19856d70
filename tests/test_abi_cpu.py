"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares,
and its host-side logic (validation, workspace planning) behaves -- no kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_1602_06709_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    binding.ensure_built()
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    hdr = open(os.path.join(ROOT, "include", "cnn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(cnn_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 27
    for name in declared:
        assert hasattr(L, name), f"{name} declared in include/cnn.h but not exported"
    assert declared == set(binding.SIGNATURES), declared ^ set(binding.SIGNATURES)


def test_status_strings(L):
    assert L.cnn_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert L.cnn_strerror(code) not in (b"ok", b"unknown status")
    assert L.cnn_strerror(-99) == b"unknown status"


def test_validation_rejects_before_any_launch(L):
    h = C.c_void_p()
    assert L.cnn_create(C.byref(h), None) == 0
    try:
        buf = (C.c_float * 64)()
        p = C.cast(buf, C.c_void_p)
        # null tensor, zero / negative dims, stride 0, negative pad, kernel larger than the padded image
        assert L.cnn_conv_fwd(h, 1, 1, 4, 4, 1, 3, 3, 1, 1, None, p, p) == -1
        assert L.cnn_conv_fwd(h, 0, 1, 4, 4, 1, 3, 3, 1, 1, p, p, p) == -1
        assert L.cnn_conv_fwd(h, 1, 1, 4, 4, 1, 3, 3, 0, 1, p, p, p) == -1
        assert L.cnn_conv_bwd_data(h, 1, 1, 4, 4, 1, 3, 3, 1, -1, p, p, p) == -1
        assert L.cnn_conv_bwd_weight(h, 1, 1, 2, 2, 1, 5, 5, 1, 0, p, p, p) == -1
        assert L.cnn_fc_fwd(h, 4, 0, 8, p, p, p) == -1
        assert L.cnn_fc_bwd(h, 4, 8, 8, p, p, None, p, p) == -1
        assert L.cnn_fc_bwd(h, 4, 8, 8, None, p, p, None, p) == -1          # dw asked for without x
        assert L.cnn_sgd_update(h, 0, p, p, None, 0.1, 0.0) == -1
        # weight gradient folded into the update: null w, bad dims; with the plain kernels forced the call is refused
        # (-2) before anything is launched; a tiled shape without a workspace is -3
        assert L.cnn_conv_bwd_weight_sgd(h, 1, 1, 4, 4, 1, 3, 3, 1, 1, p, p, None, None, 0.1, 0.0) == -1
        assert L.cnn_conv_bwd_weight_sgd(h, 1, 1, 4, 4, 1, 3, 3, 0, 1, p, p, p, None, 0.1, 0.0) == -1
        assert L.cnn_set_option(h, 0, 1) == 0
        assert L.cnn_conv_bwd_weight_sgd(h, 2, 5, 9, 9, 7, 3, 3, 1, 1, p, p, p, None, 0.1, 0.0) == -2
        assert L.cnn_set_option(h, 0, 0) == 0
        assert L.cnn_conv_bwd_weight_sgd(h, 4, 64, 56, 56, 64, 3, 3, 1, 1, p, p, p, p, 0.1, 0.9) == -3
        assert L.cnn_fc_bwd_sgd(h, 4, 8, 8, None, p, p, p, None, 0.1, 0.0) == -1
        assert L.cnn_fc_bwd_sgd(h, 4, 8, 0, p, p, p, p, None, 0.1, 0.0) == -1
        assert L.cnn_fc_bwd_sgd(h, 5, 6, 10, p, p, p, p, None, 0.1, 0.0) == -2
        assert L.cnn_relu_fwd(h, 8, None, p) == -1
        assert L.cnn_maxpool2_fwd(h, 1, 3, 4, p, p, None) == -1            # odd height
        assert L.cnn_softmax_xent(h, 0, 10, p, p, p, p) == -1
        assert L.cnn_pack_act(h, 1, 3, 2, 2, 0, p, p) == -1
        assert L.cnn_set_option(h, 12345, 1) == -1
        assert L.cnn_set_workspace(h, None, 16) == -1
        # more than 2^31-1 elements in a tensor: unsupported, not a crash
        assert L.cnn_conv_fwd(h, 4096, 1024, 224, 224, 64, 3, 3, 1, 1, p, p, p) == -2
        # weight gradient of a tiled shape without a workspace attached
        assert L.cnn_conv_bwd_weight(h, 4, 64, 56, 56, 64, 3, 3, 1, 1, p, p, p) == -3
        assert L.cnn_last_error(h) == b""
        # the allocation-free weight gradient: same validation; a layer beyond its built-in scratch array is refused
        assert L.cnn_conv_bwd_weight_static(h, 1, 1, 4, 4, 1, 3, 3, 1, 1, p, None, p) == -1
        assert L.cnn_conv_bwd_weight_static(h, 1, 1, 2, 2, 1, 5, 5, 1, 0, p, p, p) == -1
        assert L.cnn_conv_bwd_weight_static(h, 2, 2048, 14, 14, 2048, 3, 3, 1, 1, p, p, p) == -3
        assert b"built-in scratch" in L.cnn_last_error(h)
    finally:
        assert L.cnn_destroy(h) == 0
    assert L.cnn_destroy(None) == -1


def test_workspace_planning(L):
    ws = L.cnn_workspace_bytes
    # a forward whose tiles fill whole rounds of the 256 compute units needs no scratch; one with an overhang keeps
    # partial tiles of the sliced tail; unknown shapes need none (they run on the plain kernels)
    assert ws(binding.OP_CONV_FWD, 64, 256, 56, 56, 256, 3, 3, 1, 1) == 0
    assert ws(binding.OP_CONV_FWD, 64, 512, 28, 28, 512, 3, 3, 1, 1) == 128 * 2 * 128 * 224 * 4
    # the fused conv -> ReLU -> pool call plans whole row pairs; here that is the same tiling
    assert ws(binding.OP_CONV_FWD_RELU_POOL, 64, 512, 28, 28, 512, 3, 3, 1, 1) == 128 * 2 * 128 * 224 * 4
    assert ws(binding.OP_CONV_FWD_RELU_POOL, 2, 8, 7, 7, 16, 3, 3, 1, 1) == 0      # odd output: not served, no scratch
    assert ws(binding.OP_CONV_BWD_WEIGHT, 2, 5, 9, 13, 7, 3, 2, 2, 1) == 0
    # first-layer weight gradient: private copies of dw, one per split of the minibatch's rows
    b = ws(binding.OP_CONV_BWD_WEIGHT, 2, 3, 32, 32, 16, 3, 3, 1, 1)
    assert b > 0 and b % (16 * 3 * 9 * 4) == 0
    # backpropagation keeps one mirrored transpose of the weights
    assert ws(binding.OP_CONV_BWD_DATA, 64, 256, 56, 56, 256, 3, 3, 1, 1) == 256 * 256 * 9 * 4
    # weight gradient: a whole number of private copies of dw
    b = ws(binding.OP_CONV_BWD_WEIGHT, 64, 256, 56, 56, 256, 3, 3, 1, 1)
    assert b > 0 and b % (256 * 256 * 9 * 4) == 0
    # split-K partials for the small-minibatch FC forward; none when there are tiles enough
    b = ws(binding.OP_FC_FWD, 64, 25088, 1, 1, 4096, 1, 1, 1, 0)
    assert b > 0 and b % (64 * 4096 * 4) == 0
    assert ws(binding.OP_FC_FWD, 0, 25088, 1, 1, 4096, 1, 1, 1, 0) == 0
    # every layer of every workload plans without error and stays far below the device memory
    for cfg in (1, 2, 3, 4, 5):
        wl = synth.workload(cfg)
        shp = [tuple(wl.input_shape)] + synth.shapes(wl)
        for i, Ly in enumerate(wl.layers):
            if Ly[0] == "conv":
                s = shp[i]
                for op in (0, 1, 2):
                    assert ws(op, s[0], Ly[1], s[2], s[3], Ly[2], Ly[3], Ly[4], Ly[5], Ly[6]) < (8 << 30)
            elif Ly[0] == "fc":
                for op in (3, 4):
                    assert ws(op, shp[i][0], Ly[1], 1, 1, Ly[2], 1, 1, 1, 0) < (8 << 30)


def test_packed_sizes(L):
    assert L.cnn_packed_act_elems(2, 11, 3, 5, 8) == 2 * 2 * 3 * 5 * 8
    assert L.cnn_packed_wt_elems(13, 11, 3, 2, 8, 0) == 11 * 2 * 3 * 2 * 8
    assert L.cnn_packed_wt_elems(13, 11, 3, 2, 8, 1) == 13 * 2 * 3 * 2 * 8
    assert L.cnn_packed_act_elems(2, 11, 3, 5, 0) == 0


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding._build, "LIB", str(tmp_path / "nope.so"))
    with pytest.raises(binding.CnnError):
        binding.lib()


def test_blocking_model_host_functions_match_the_oracle(L):
    from oracle import blocking as OB
    for (n, c, k, p, q, r, s_, st) in [(6, 512, 1024, 12, 12, 3, 3, 1), (2, 3, 96, 56, 56, 11, 11, 4), (5, 7, 9, 4, 6, 2, 3, 2)]:
        assert L.cnn_bf_plane(p, q, r, s_, st) == pytest.approx(OB.bf_plane(p, q, r, s_, st), rel=1e-14)
        assert L.cnn_bf_layer(n, c, k, p, q, r, s_, st) == pytest.approx(OB.bf_layer(n, c, k, p, q, r, s_, st), rel=1e-14)
        for blk in [(1, 8, 4, 2, 3), (n, k, c, p, q), (2, 16, 4, 1, q)]:
            want = OB.trav_bytes(blk, c, r, s_, st) / OB.trav_flops(blk, c, r, s_)
            assert L.cnn_bf_block_traversal(c, r, s_, st, blk[0], blk[1], blk[3], blk[4]) == pytest.approx(want, rel=1e-14)
    assert L.cnn_bf_plane(0, 3, 3, 3, 1) == -1.0 and L.cnn_bf_layer(1, 1, 1, 1, 1, 1, 1, 0) == -1.0
    assert round(L.cnn_bf_plane(12, 12, 3, 3, 1), 2) == 0.54 and round(L.cnn_bf_layer(6, 512, 1024, 12, 12, 3, 3, 1), 3) == 0.003


def test_tile_report_and_block_search_validation(L):
    from oracle import blocking as OB
    tile = (C.c_int32 * 8)()
    bf = C.c_double()
    tp = C.cast(tile, C.c_void_p)
    # VGG-A 128 -> 256 features at 56x56, minibatch 64: 128-feature tiles of whole output rows
    assert L.cnn_conv_tile_info(0, 64, 128, 56, 56, 256, 3, 3, 1, 1, tp, C.byref(bf)) == 0
    t = list(tile)
    assert t[0] == 128 and t[2] == 56 and t[3] == 4 and t[1] * t[2] <= t[7] and 0 < t[5] <= 160 * 1024
    assert t[6] == 2 * -(-64 * 56 // t[1])
    want = OB.trav_bytes((1, t[0], t[3], t[1], t[2]), 128, 3, 3) / OB.trav_flops((1, t[0], t[3], t[1], t[2]), 128, 3, 3)
    assert bf.value == pytest.approx(want, rel=1e-14)
    # the tile's ratio lies between the whole layer's and the unblocked loop's, and below the chip's own
    # 8 TB/s / 157.3 TFLOP/s = 0.051 bytes per FLOP
    assert OB.bf_layer(64, 128, 256, 56, 56, 3, 3) < bf.value < 0.051 < OB.bf_plane(56, 56, 3, 3)
    # backpropagation: the pass's outputs are the layer's input features
    # 224 tiles on 256 compute units: chunks dealt out in equal runs, 7/8 of a tile per workgroup, two pieces per tile
    assert L.cnn_conv_tile_info(0, 64, 512, 14, 14, 512, 3, 3, 1, 1, tp, C.byref(bf)) == 0
    assert list(tile)[4] == -3 and list(tile)[6] == 256 and list(tile)[1] == 16
    assert L.cnn_conv_tile_info(1, 64, 64, 112, 112, 128, 3, 3, 1, 1, tp, C.byref(bf)) == 0 and tile[0] == 64
    assert L.cnn_conv_tile_info(0, 2, 5, 9, 9, 7, 7, 7, 2, 0, tp, C.byref(bf)) == -2      # no tiled kernel for 7x7 / 2
    assert L.cnn_conv_tile_info(2, 64, 128, 56, 56, 256, 3, 3, 1, 1, tp, C.byref(bf)) == -1
    assert L.cnn_conv_tile_info(0, 64, 128, 56, 56, 256, 3, 3, 1, 1, None, C.byref(bf)) == -1
    h = C.c_void_p()
    assert L.cnn_create(C.byref(h), None) == 0
    try:
        res = (C.c_double * 6)()
        rp = C.cast(res, C.c_void_p)
        assert L.cnn_block_search(h, 1, 8, 8, 4, 4, 3, 3, 1, 4096, 8, None) == -1
        assert L.cnn_block_search(h, 0, 8, 8, 4, 4, 3, 3, 1, 4096, 8, rp) == -1
        assert L.cnn_block_search(h, 1, 8, 8, 4, 4, 3, 3, 1, 0, 8, rp) == -1
        assert L.cnn_block_search(h, 1, 8, 8, 4, 4, 3, 3, 1, 4096, 0, rp) == -1
        assert L.cnn_block_search_traversal(h, 1, 8, 8, 4, 4, 3, 3, 1, 4096, 4096, 8, 0, rp) == -1
        assert L.cnn_block_search(h, 1, 8, 8, 4, 4, 3, 3, 1, 4096, 8, rp) == -3                # no workspace attached
        assert L.cnn_block_search(h, 1 << 20, 1 << 20, 1 << 20, 1 << 10, 1 << 10, 3, 3, 1, 4096, 8, rp) == -2
        assert L.cnn_workspace_bytes(6, 0, 0, 0, 0, 0, 0, 0, 0, 0) > 0
    finally:
        assert L.cnn_destroy(h) == 0


def test_parameter_arrays_are_cut_from_one_block():
    # weights, gradients and momentum of a network are ranges of one allocation: disjoint, in order, each start
    # 16-byte aligned (the update reads them as float4) and shifted against its neighbours
    import torch
    from paper_1602_06709_amd.net import carve_arrays
    for n in (4, 1000, 4096, 132851392 // 64):
        arrs = carve_arrays(n, 3, "cpu")
        assert [a.numel() for a in arrs] == [n] * 3 and all(a.dtype == torch.float32 for a in arrs)
        ptr = [a.data_ptr() for a in arrs]
        assert all(p % 16 == 0 for p in ptr)
        assert ptr[0] + 4 * n <= ptr[1] and ptr[1] + 4 * n <= ptr[2]
        assert (ptr[1] - ptr[0]) != (ptr[2] - ptr[1])
        base = arrs[0].untyped_storage().data_ptr()
        assert all(a.untyped_storage().data_ptr() == base for a in arrs)
        assert all(float(a.abs().sum()) == 0.0 for a in arrs)


def test_bench_refuses_more_than_one_gpu():
    # one GPU per box: the benchmark says so and exits before touching a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
