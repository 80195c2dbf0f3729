"""Seeded sweep over random small networks (convolutional and residual): GPU path against the float64 oracle.

The shapes are drawn so that the layers fall on the different convolution kernels (few / up to 16 / 32 / more input
channels, both strides, padding 0 and 1, patch rows and dense rows), with and without depth limits, labels and the
fused route.  Every configuration is a valid one; the comparison is the element-by-element one of the parity tests."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle                                             # noqa: E402
from paper_2507_20055_amd import workloads as wl          # noqa: E402
from tests.parity_util import compare_with_oracle         # noqa: E402


def _binding():
    from paper_2507_20055_amd import binding
    return binding


def _random_conv(rng):
    C = int(rng.choice([1, 3, 4])); H = int(rng.integers(6, 15)); W = int(rng.integers(6, 15))
    nconv = int(rng.integers(2, 5))
    convs = []
    h, w = H, W
    for _ in range(nconv):
        for _try in range(20):
            co = int(rng.choice([4, 8, 16, 16, 24, 32, 40])); k = int(rng.choice([2, 3, 4]))
            s = int(rng.choice([1, 1, 2])); p = int(rng.choice([0, 1]))
            ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
            if ho >= 1 and wo >= 1 and co * ho * wo <= 2600:
                convs.append((co, k, s, p)); h, w = ho, wo
                break
        else:
            break
    fcs = [max(2, int(rng.integers(3, 14))) for _ in range(int(rng.integers(1, 3)))]
    return (C, H, W), convs, fcs


def _options(rng, nl):
    kw, okw = {}, {}
    mode = rng.random()
    if mode < 0.3:
        d = int(rng.integers(0, nl + 1))
        kw, okw = dict(max_backsub_depth=d), dict(max_depth=d)
    elif mode < 0.4:
        d = int(rng.integers(0, 4)); f = int(rng.choice([-1, 2, 5]))
        kw, okw = dict(max_backsub_depth=d, final_backsub_depth=f), dict(max_depth=d, max_depth_last=f)
    return kw, okw, int(rng.random() < 0.85)


def _check(net, rng, seed, allow_final=True):
    B = int(rng.integers(1, 4))
    eps = float(rng.choice([0.01, 0.05, 0.1]))
    x, lo, hi = wl.random_box(seed + 1, net.n_in, B, eps)
    n_out = net.layers[-1].W.shape[0]
    label = rng.integers(0, n_out, size=B).astype(np.int32) if rng.random() < 0.8 else None
    kw, okw, fuse = _options(rng, len(net.layers))
    if not allow_final:
        kw.pop("final_backsub_depth", None); okw.pop("max_depth_last", None)
    gnet = _binding().Network(net)
    try:
        g = gnet.certify(lo, hi, label, fuse=fuse, **kw)
        o = oracle.run(net, lo, hi, label=label, **okw)
        # at most one input may leave the element-by-element comparison after a lambda near-tie, and only at the
        # network's last ReLU layer (everything below it is then still compared)
        last_relu = max(i + 1 for i, L in enumerate(net.layers) if L.kind == "relu")
        compare_with_oracle(net, lo, hi, g, o, label, max_flipped_inputs=1, min_flip_layer=last_relu)
    finally:
        gnet.close()


@pytest.mark.parametrize("seed", list(range(1000, 1024)))
def test_random_conv_network(seed):
    rng = np.random.default_rng(seed)
    shape, convs, fcs = _random_conv(rng)
    assert convs
    _check(wl.random_small_conv(seed, shape, convs, fcs), rng, seed)


@pytest.mark.parametrize("seed", list(range(5000, 5016)))
def test_random_residual_network(seed):
    rng = np.random.default_rng(seed)
    if rng.random() < 0.7:
        shape = (int(rng.choice([1, 2, 3])), int(rng.integers(5, 11)), int(rng.integers(5, 11)))
        width = int(rng.choice([4, 8, 8, 16, 16])); blocks = int(rng.integers(1, 3)); k = int(rng.choice([1, 3, 3]))
        tail = [] if rng.random() < 0.4 else [(int(rng.choice([8, 16, 32])), int(rng.choice([3, 4])), int(rng.choice([1, 2])), 1)]
        fcs = [max(2, int(rng.integers(3, 10))) for _ in range(int(rng.integers(1, 3)))]
        net = wl.random_small_res_conv(seed, shape, width, blocks, k, tail, fcs)
    else:
        net = wl.random_small_res(seed, int(rng.integers(6, 40)), int(rng.choice([8, 20, 36, 64, 100])), int(rng.integers(1, 4)),
                                  int(rng.integers(2, 8)))
    _check(net, rng, seed, allow_final=False)
