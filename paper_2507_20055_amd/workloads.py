"""Seeded synthetic workloads: random ReLU networks and L-infinity input boxes.

This module only *generates inputs* (weights, biases, input points, boxes,
labels).  It holds none of the certifier's arithmetic, so both the CPU oracle's
tests and the GPU path's tests may draw their inputs from it.

The five configurations mirror the shapes, batch sizes and perturbation scales
of the fully-connected and convolutional MNIST / CIFAR10 networks in the
paper's evaluation (Tables 1 and 5 name them "6x500", "ConvSmall", "ConvBig",
...; the paper gives no layer dimensions or weights, so random networks of
matching shape stand in for the trained ones).

Recipe (identical for every configuration):
  * ``rng = numpy.random.default_rng(seed)``; for each parametrised layer in
    network order draw the weight tensor, then the bias vector;
  * fully-connected nets: W ~ N(0, 1/fan_in); conv nets: He-normal,
    W ~ N(0, 2/fan_in) with fan_in = Ci*kh*kw (conv) or in-features (FC);
    bias ~ N(0, 0.01^2);
  * inputs x ~ U[0,1]^n0 from ``default_rng(seed + 1000)``;
  * everything is drawn in float64 and rounded once to float32; the float32
    values are the network.  Box: lo = max(x-eps, 0), hi = min(x+eps, 1),
    computed in float32.
  * label = argmax of a float64 forward pass on x (ties -> lowest index).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass
class Layer:
    kind: str                                  # "affine" | "conv" | "relu" | "add"
    W: Optional[np.ndarray] = None             # affine: [out, in]; conv: [Co, Ci, kh, kw]
    b: Optional[np.ndarray] = None             # [out] or [Co]
    stride: int = 1
    pad: int = 0
    in_shape: Optional[Tuple[int, int, int]] = None   # conv only: (Ci, H, W)
    skip: int = -1                             # add only: layer index (0 = input) whose output is added to the layer below

    @property
    def out_shape(self) -> Tuple[int, int, int]:
        assert self.kind == "conv"
        Ci, H, W = self.in_shape
        Co, _, kh, kw = self.W.shape
        Ho = (H + 2 * self.pad - kh) // self.stride + 1
        Wo = (W + 2 * self.pad - kw) // self.stride + 1
        return (Co, Ho, Wo)


@dataclass
class Network:
    n_in: int
    layers: List[Layer] = field(default_factory=list)

    def sizes(self) -> List[int]:
        """Number of neurons after every layer (index 0 = input)."""
        out = [self.n_in]
        for L in self.layers:
            if L.kind == "affine":
                out.append(int(L.W.shape[0]))
            elif L.kind == "conv":
                c, h, w = L.out_shape
                out.append(c * h * w)
            else:                                  # relu, add: same size as the layer below
                out.append(out[-1])
        return out


@dataclass
class Workload:
    name: str
    net: Network
    x: np.ndarray        # [B, n0] float32
    lo: np.ndarray       # [B, n0] float32
    hi: np.ndarray       # [B, n0] float32
    label: np.ndarray    # [B] int32
    eps: float


def conv_forward(x: np.ndarray, L: Layer) -> np.ndarray:
    """Plain zero-padded cross-correlation, x: [B, Ci*H*W] flattened (C,H,W)."""
    Ci, H, W = L.in_shape
    Co, _, kh, kw = L.W.shape
    _, Ho, Wo = L.out_shape
    s, p = L.stride, L.pad
    B = x.shape[0]
    xp = np.zeros((B, Ci, H + 2 * p, W + 2 * p), dtype=x.dtype)
    xp[:, :, p:p + H, p:p + W] = x.reshape(B, Ci, H, W)
    out = np.zeros((B, Co, Ho, Wo), dtype=x.dtype)
    Wk = L.W.astype(x.dtype)
    for ky in range(kh):
        for kx in range(kw):
            patch = xp[:, :, ky:ky + s * Ho:s, kx:kx + s * Wo:s]      # [B, Ci, Ho, Wo]
            out += np.einsum("bchw,oc->bohw", patch, Wk[:, :, ky, kx])
    out += L.b.astype(x.dtype).reshape(1, Co, 1, 1)
    return out.reshape(B, -1)


def forward(net: Network, x: np.ndarray, upto: Optional[int] = None) -> List[np.ndarray]:
    """Concrete evaluation in x's dtype; returns the activation after every layer."""
    acts = [x]
    h = x
    for L in net.layers[:upto]:
        if L.kind == "affine":
            h = h @ L.W.astype(x.dtype).T + L.b.astype(x.dtype)
        elif L.kind == "conv":
            h = conv_forward(h, L)
        elif L.kind == "add":
            h = h + acts[L.skip]
        else:
            h = np.maximum(h, 0)
        acts.append(h)
    return acts


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.astype(np.float32))


def make_fc(rng, dims: List[int], he: bool = False) -> Network:
    net = Network(n_in=dims[0])
    for i in range(1, len(dims)):
        fan_in = dims[i - 1]
        std = np.sqrt((2.0 if he else 1.0) / fan_in)
        W = rng.normal(0.0, std, size=(dims[i], fan_in))
        b = rng.normal(0.0, 0.01, size=(dims[i],))
        net.layers.append(Layer("affine", _f32(W), _f32(b)))
        if i != len(dims) - 1:
            net.layers.append(Layer("relu"))
    return net


def make_conv(rng, in_shape, convs, fcs) -> Network:
    """convs: list of (Co, k, stride, pad); fcs: list of out-features. He-normal."""
    Ci, H, W = in_shape
    net = Network(n_in=Ci * H * W)
    shape = in_shape
    for (Co, k, s, p) in convs:
        fan_in = shape[0] * k * k
        Wt = rng.normal(0.0, np.sqrt(2.0 / fan_in), size=(Co, shape[0], k, k))
        b = rng.normal(0.0, 0.01, size=(Co,))
        L = Layer("conv", _f32(Wt), _f32(b), stride=s, pad=p, in_shape=shape)
        net.layers.append(L)
        net.layers.append(Layer("relu"))
        shape = L.out_shape
    n = shape[0] * shape[1] * shape[2]
    for i, f in enumerate(fcs):
        Wt = rng.normal(0.0, np.sqrt(2.0 / n), size=(f, n))
        b = rng.normal(0.0, 0.01, size=(f,))
        net.layers.append(Layer("affine", _f32(Wt), _f32(b)))
        if i != len(fcs) - 1:
            net.layers.append(Layer("relu"))
        n = f
    return net


def make_res_fc(rng, n_in: int, width: int, blocks: int, n_out: int, std_scale: float = 1.0, bias_std: float = 0.01) -> Network:
    """Fully-connected residual network: affine(n_in -> width), ReLU, then `blocks` times
    [affine, ReLU, affine, add(block input), ReLU] at constant width, then affine(width -> n_out).
    W ~ N(0, std_scale^2 / fan_in), bias ~ N(0, bias_std^2), drawn in network order (weight, then bias)."""
    net = Network(n_in=n_in)

    def affine(n_to, n_from):
        W = rng.normal(0.0, std_scale / np.sqrt(n_from), size=(n_to, n_from))
        b = rng.normal(0.0, bias_std, size=(n_to,))
        net.layers.append(Layer("affine", _f32(W), _f32(b)))

    affine(width, n_in)
    net.layers.append(Layer("relu"))
    for _ in range(blocks):
        src = len(net.layers)                  # layer index of the block's input (output of the ReLU just added)
        affine(width, width)
        net.layers.append(Layer("relu"))
        affine(width, width)
        net.layers.append(Layer("add", skip=src))
        net.layers.append(Layer("relu"))
    affine(n_out, width)
    return net


def make_res_conv(rng, in_shape, width: int, blocks: int, k: int, tail, fcs) -> Network:
    """Convolutional residual network: conv(Ci -> width, k x k, stride 1, same padding), ReLU, `blocks` times
    [conv, ReLU, conv, add(block input), ReLU] at constant shape, then the convolutions in `tail`
    ((Co, k, stride, pad), each followed by ReLU) and the fully-connected layers `fcs`.  He-normal, k odd."""
    assert k % 2 == 1
    Ci, H, W = in_shape
    net = Network(n_in=Ci * H * W)
    shape = in_shape

    def conv(Co, kk, s, p):
        nonlocal shape
        fan_in = shape[0] * kk * kk
        Wt = rng.normal(0.0, np.sqrt(2.0 / fan_in), size=(Co, shape[0], kk, kk))
        b = rng.normal(0.0, 0.01, size=(Co,))
        L = Layer("conv", _f32(Wt), _f32(b), stride=s, pad=p, in_shape=shape)
        net.layers.append(L)
        shape = L.out_shape

    conv(width, k, 1, k // 2)
    net.layers.append(Layer("relu"))
    for _ in range(blocks):
        src = len(net.layers)
        conv(width, k, 1, k // 2)
        net.layers.append(Layer("relu"))
        conv(width, k, 1, k // 2)
        net.layers.append(Layer("add", skip=src))
        net.layers.append(Layer("relu"))
    for (Co, kk, s, p) in tail:
        conv(Co, kk, s, p)
        net.layers.append(Layer("relu"))
    n = shape[0] * shape[1] * shape[2]
    for i, f in enumerate(fcs):
        Wt = rng.normal(0.0, np.sqrt(2.0 / n), size=(f, n))
        b = rng.normal(0.0, 0.01, size=(f,))
        net.layers.append(Layer("affine", _f32(Wt), _f32(b)))
        if i != len(fcs) - 1:
            net.layers.append(Layer("relu"))
        n = f
    return net


def make_inputs(net: Network, seed: int, batch: int, eps: float):
    rng = np.random.default_rng(seed + 1000)
    x = _f32(rng.uniform(0.0, 1.0, size=(batch, net.n_in)))
    e = np.float32(eps)
    lo = np.maximum(x - e, np.float32(0.0)).astype(np.float32)
    hi = np.minimum(x + e, np.float32(1.0)).astype(np.float32)
    y = forward(net, x.astype(np.float64))[-1]
    label = np.argmax(y, axis=1).astype(np.int32)
    return x, lo, hi, label


# name -> (builder, seed, batch, eps list)
def _cfg1(rng): return make_fc(rng, [784, 100, 100, 100, 10])
def _cfg2(rng): return make_fc(rng, [784] + [500] * 6 + [10])
def _cfg3(rng): return make_conv(rng, (3, 32, 32), [(16, 4, 2, 1), (32, 4, 2, 1)], [100, 10])
def _cfg4(rng): return make_conv(rng, (3, 32, 32),
                                 [(32, 3, 1, 1), (32, 4, 2, 1), (64, 3, 1, 1), (64, 4, 2, 1)],
                                 [512, 512, 10])
def _cfg5(rng): return make_fc(rng, [1024] + [1024] * 9 + [10])
# residual stand-ins (the paper's "Skip" MNIST network is named in Table 5 without its layers)
def _res_fc(rng): return make_res_fc(rng, 784, 512, 3, 10)
def _res_conv(rng): return make_res_conv(rng, (1, 28, 28), 16, 2, 3, [(32, 4, 2, 1)], [100, 10])


CONFIGS = {
    "cfg1": dict(build=_cfg1, seed=0, batch=1, eps=[0.01]),
    "cfg2": dict(build=_cfg2, seed=0, batch=32, eps=[0.005, 0.01, 0.02]),
    "cfg3": dict(build=_cfg3, seed=1, batch=32, eps=[2.0 / 255.0]),
    "cfg4": dict(build=_cfg4, seed=2, batch=16, eps=[1.0 / 255.0]),
    "cfg5": dict(build=_cfg5, seed=3, batch=64, eps=[0.005]),
    "res_fc": dict(build=_res_fc, seed=4, batch=32, eps=[0.001]),
    "res_conv": dict(build=_res_conv, seed=5, batch=16, eps=[0.003]),
}


def make_workload(name: str, eps_index: int = 0, batch: Optional[int] = None) -> Workload:
    """Build one of the five named configurations (optionally only the first
    ``batch`` inputs of it: inputs are drawn for the full batch and then cut,
    so a sub-batch is a prefix of the full workload)."""
    cfg = CONFIGS[name]
    rng = np.random.default_rng(cfg["seed"])
    net = cfg["build"](rng)
    eps = cfg["eps"][eps_index]
    x, lo, hi, label = make_inputs(net, cfg["seed"], cfg["batch"], eps)
    if batch is not None:
        x, lo, hi, label = x[:batch], lo[:batch], hi[:batch], label[:batch]
    return Workload(f"{name}/eps={eps:g}", net, x, lo, hi, label, eps)


def random_small_net(seed: int, dims: List[int], bias_std: float = 0.3) -> Network:
    """Small FC net with O(1) weights for unit tests (many unstable ReLUs)."""
    rng = np.random.default_rng(seed)
    net = Network(n_in=dims[0])
    for i in range(1, len(dims)):
        W = rng.normal(0.0, 1.0 / np.sqrt(dims[i - 1]), size=(dims[i], dims[i - 1]))
        b = rng.normal(0.0, bias_std, size=(dims[i],))
        net.layers.append(Layer("affine", _f32(W), _f32(b)))
        if i != len(dims) - 1:
            net.layers.append(Layer("relu"))
    return net


def random_small_conv(seed: int, in_shape, convs, fcs, bias_std: float = 0.1) -> Network:
    rng = np.random.default_rng(seed)
    net = make_conv(rng, in_shape, convs, fcs)
    for L in net.layers:
        if L.b is not None:
            L.b = _f32(rng.normal(0.0, bias_std, size=L.b.shape))
    return net


def random_small_res(seed: int, n_in: int, width: int, blocks: int, n_out: int, bias_std: float = 0.3) -> Network:
    """Small residual FC net with O(1) weights for unit tests."""
    return make_res_fc(np.random.default_rng(seed), n_in, width, blocks, n_out, 1.0, bias_std)


def random_small_res_conv(seed: int, in_shape, width: int, blocks: int, k: int, tail, fcs, bias_std: float = 0.1) -> Network:
    rng = np.random.default_rng(seed)
    net = make_res_conv(rng, in_shape, width, blocks, k, tail, fcs)
    for L in net.layers:
        if L.b is not None:
            L.b = _f32(rng.normal(0.0, bias_std, size=L.b.shape))
    return net


def random_box(seed: int, n: int, batch: int, eps: float, lo_clip=None, hi_clip=None):
    rng = np.random.default_rng(seed)
    x = _f32(rng.uniform(-1.0, 1.0, size=(batch, n)))
    lo = (x - np.float32(eps)).astype(np.float32)
    hi = (x + np.float32(eps)).astype(np.float32)
    if lo_clip is not None:
        lo = np.maximum(lo, np.float32(lo_clip))
    if hi_clip is not None:
        hi = np.minimum(hi, np.float32(hi_clip))
    return x, lo, hi
