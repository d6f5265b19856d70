"""Seeded synthetic workloads: layer tables and input generators.

This module holds no arithmetic of the method -- only the shapes of the five
benchmark workloads and the random tensors fed, identically, to the GPU library
and to the CPU oracle.  Nothing from ImageNet or Switchboard is used; synthetic
tensors of the same shapes stand in for them (Section 5 of the paper measures
on those datasets).

Layer entries:
  ("conv", C, K, R, S, stride, pad)   ("relu",)   ("pool",)   ("flatten",)
  ("fc", I, O)                        ("sigmoid",)
A network ends in a softmax cross-entropy loss when `loss` is True; otherwise an
upstream gradient of the last layer's output shape is supplied.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

SEED_ROOT = 160206709


def rng(config_id: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([SEED_ROOT, int(config_id), int(tensor_id)]))


def _conv3(c, k):
    return ("conv", c, k, 3, 3, 1, 1)


VGG_A_CONV = [
    _conv3(3, 64), ("relu",), ("pool",),
    _conv3(64, 128), ("relu",), ("pool",),
    _conv3(128, 256), ("relu",), _conv3(256, 256), ("relu",), ("pool",),
    _conv3(256, 512), ("relu",), _conv3(512, 512), ("relu",), ("pool",),
    _conv3(512, 512), ("relu",), _conv3(512, 512), ("relu",), ("pool",),
]
VGG_A_FC = [("flatten",), ("fc", 25088, 4096), ("relu",), ("fc", 4096, 4096), ("relu",), ("fc", 4096, 1000)]

OVERFEAT_FAST = [
    ("conv", 3, 96, 11, 11, 4, 0), ("relu",), ("pool",),
    ("conv", 96, 256, 5, 5, 1, 0), ("relu",), ("pool",),
    _conv3(256, 512), ("relu",), _conv3(512, 1024), ("relu",), _conv3(1024, 1024), ("relu",), ("pool",),
    ("flatten",), ("fc", 36864, 3072), ("relu",), ("fc", 3072, 4096), ("relu",), ("fc", 4096, 1000),
]

DNN7 = ([("fc", 440, 2048), ("sigmoid",)]
        + [x for _ in range(5) for x in (("fc", 2048, 2048), ("sigmoid",))]
        + [("fc", 2048, 9304)])


@dataclass
class Workload:
    config_id: int
    name: str
    layers: List[Tuple]
    input_shape: Tuple[int, ...]          # including the minibatch
    loss: bool                            # softmax cross-entropy at the end
    n_classes: int = 0
    lr: float = 0.01
    momentum: float = 0.0
    sgd: bool = False
    init: str = "he"                      # "he" | "glorot" | "uniform"
    notes: str = ""
    extra: dict = field(default_factory=dict)


def workload(config_id: int, N: int = None) -> Workload:
    """The five workloads.  N overrides the per-GPU minibatch (used for slices)."""
    if config_id == 1:
        n = N or 2
        return Workload(1, "single_conv_3x3", [("conv", 3, 16, 3, 3, 1, 1)], (n, 3, 32, 32), False,
                        lr=0.01, momentum=0.0, sgd=True, init="uniform")
    if config_id == 2:
        n = N or 4
        return Workload(2, "vgg_a_conv_stack", list(VGG_A_CONV), (n, 3, 224, 224), False, init="he")
    if config_id == 3:
        n = N or 64
        return Workload(3, "vgg_a_full", list(VGG_A_CONV) + list(VGG_A_FC), (n, 3, 224, 224), True,
                        n_classes=1000, lr=0.001, momentum=0.9, sgd=True, init="he")   # 0.01 diverges from a He start
    if config_id == 4:
        n = N or 64
        return Workload(4, "overfeat_fast", list(OVERFEAT_FAST), (n, 3, 231, 231), True,
                        n_classes=1000, sgd=False, init="he")
    if config_id == 5:
        n = N or 1024
        return Workload(5, "dnn7_fc", list(DNN7), (n, 440), True, n_classes=9304,
                        lr=0.01, momentum=0.0, sgd=True, init="glorot")
    raise ValueError(f"unknown config {config_id}")


def out_hw(h, w, layer):
    _, _, _, R, S, st, pad = layer
    return (h + 2 * pad - R) // st + 1, (w + 2 * pad - S) // st + 1


def shapes(wl: Workload):
    """Activation shape after every layer (list aligned with wl.layers), starting from the input."""
    shp = tuple(wl.input_shape)
    out = []
    for L in wl.layers:
        kind = L[0]
        if kind == "conv":
            n, c, h, w = shp
            assert c == L[1], (shp, L)
            p, q = out_hw(h, w, L)
            shp = (n, L[2], p, q)
        elif kind == "pool":
            n, c, h, w = shp
            assert h % 2 == 0 and w % 2 == 0, shp
            shp = (n, c, h // 2, w // 2)
        elif kind == "flatten":
            shp = (shp[0], int(np.prod(shp[1:])))
        elif kind == "fc":
            assert shp[1] == L[1], (shp, L)
            shp = (shp[0], L[2])
        out.append(shp)
    return out


def weight_shapes(wl: Workload):
    ws = []
    for L in wl.layers:
        if L[0] == "conv":
            ws.append((L[2], L[1], L[3], L[4]))
        elif L[0] == "fc":
            ws.append((L[2], L[1]))
    return ws


def make_weights(wl: Workload):
    """One fp32 array per conv / fc layer.  He-normal: std = sqrt(2/fan_in), fan_in = C*R*S or I.
    Glorot-uniform: U(-a, a), a = sqrt(6/(I+O)).  'uniform': U[-1, 1]."""
    out = []
    for j, shp in enumerate(weight_shapes(wl)):
        g = rng(wl.config_id, 100 + j)
        fan_in = int(np.prod(shp[1:]))
        if wl.init == "he":
            w = g.standard_normal(shp, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))
        elif wl.init == "glorot":
            a = np.sqrt(6.0 / (shp[0] + shp[1]))
            w = g.uniform(-a, a, shp).astype(np.float32)
        else:
            w = g.uniform(-1.0, 1.0, shp).astype(np.float32)
        out.append(np.ascontiguousarray(w, dtype=np.float32))
    return out


def make_input(wl: Workload):
    g = rng(wl.config_id, 0)
    if wl.config_id == 1:
        return g.uniform(-1.0, 1.0, wl.input_shape).astype(np.float32)
    return g.standard_normal(wl.input_shape, dtype=np.float32)


def make_labels(wl: Workload):
    g = rng(wl.config_id, 1)
    return g.integers(0, wl.n_classes, size=wl.input_shape[0]).astype(np.int32)


def make_upstream(wl: Workload):
    """N(0,1) gradient with the shape of the network's last activation (for workloads without a loss)."""
    g = rng(wl.config_id, 2)
    return g.standard_normal(shapes(wl)[-1], dtype=np.float32)


def randn(config_id, tensor_id, shape, scale=1.0):
    return (rng(config_id, tensor_id).standard_normal(shape, dtype=np.float32) * np.float32(scale))


def uniform(config_id, tensor_id, shape, lo=-1.0, hi=1.0):
    return rng(config_id, tensor_id).uniform(lo, hi, shape).astype(np.float32)


def sample_indices(config_id, tensor_id, total, count):
    """`count` distinct-ish flat indices in [0, total) for sampled parity (sorted, int64)."""
    g = rng(config_id, tensor_id)
    if total <= count:
        return np.arange(total, dtype=np.int64)
    return np.unique(g.integers(0, total, size=count, dtype=np.int64))
