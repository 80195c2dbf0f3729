"""Pins for the oracle's Add layer (residual networks): an expression then holds terms of several layers at once.

The paper prints no Add transformer (its specification language only names two predecessors prev0, prev1), so the
reading -- L = U = prev0 + prev1 with l, u by back-substitution, deepest layer replaced first (Section 4.2) -- is
pinned here against what the mathematics fixes: exact equivalences with chain networks, brute force with the
neuron-level transcription of map / traverse, and soundness on sampled points."""
import copy

import numpy as np
import pytest

import oracle
from oracle import neuron_level
from paper_2507_20055_amd import workloads as wl
from paper_2507_20055_amd.workloads import Layer, Network


def _box(seed, n, B, eps):
    return wl.random_box(seed, n, B, eps)


def test_single_affine_branch_equals_chain_with_w_plus_identity():
    """x + (W x + b) = (W + I) x + b: back-substitution composes affine maps exactly, so every later layer's bounds
    equal those of the chain network with the block folded into one affine layer."""
    rng = np.random.default_rng(5)
    n0, m, k = 5, 6, 4
    W1, b1 = rng.normal(size=(m, n0)).astype(np.float32), rng.normal(size=m).astype(np.float32)
    # entries on a coarse binary grid so that W2 + I is exact in float32
    W2 = (np.round(rng.normal(size=(m, m)) * 8) / 8).astype(np.float32)
    b2 = rng.normal(size=m).astype(np.float32)
    W3, b3 = rng.normal(size=(k, m)).astype(np.float32), rng.normal(size=k).astype(np.float32)
    res = Network(n0, [Layer("affine", W1, b1), Layer("relu"), Layer("affine", W2, b2), Layer("add", skip=2),
                       Layer("relu"), Layer("affine", W3, b3)])
    chain = Network(n0, [Layer("affine", W1, b1), Layer("relu"), Layer("affine", (W2 + np.eye(m, dtype=np.float32)), b2),
                         Layer("relu"), Layer("affine", W3, b3)])
    x, lo, hi = _box(6, n0, 4, 0.3)
    label = np.array([0, 1, 2, 3], np.int32)
    a = oracle.run(res, lo, hi, label=label)
    c = oracle.run(chain, lo, hi, label=label)
    np.testing.assert_allclose(a.l[4], c.l[3], rtol=1e-12, atol=1e-12)     # the Add layer = the folded affine layer
    np.testing.assert_allclose(a.u[4], c.u[3], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a.l[6], c.l[5], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a.u[6], c.u[5], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a.margin, c.margin, rtol=1e-12, atol=1e-12)
    assert (a.verdict == c.verdict).all()
    assert np.abs(a.l[3] - a.l[4]).max() > 1e-3                             # the skip term is really there


def test_zero_branch_is_an_identity_affine_layer():
    """With a zero branch the Add neuron is 0 + eta_skip: exactly an affine layer with identity weights placed on the
    skip operand (its bounds come from back-substitution, which for a ReLU operand need not equal the ReLU's own
    interval), so the whole network equals that chain network."""
    net = wl.random_small_res(11, 4, 5, 1, 3)
    # layers: affine, relu, [affine, relu, affine, add(skip=2), relu], affine
    net.layers[4].W[:] = 0
    net.layers[4].b[:] = 0
    ident = Layer("affine", np.eye(5, dtype=np.float32), np.zeros(5, np.float32))
    chain = Network(net.n_in, [net.layers[0], net.layers[1], ident, Layer("relu"), net.layers[7]])
    x, lo, hi = _box(12, 4, 3, 0.2)
    label = np.array([0, 1, 2], np.int32)
    a = oracle.run(net, lo, hi, label=label)
    c = oracle.run(chain, lo, hi, label=label)
    for ka, kc in ((6, 3), (7, 4), (8, 5)):
        np.testing.assert_allclose(a.l[ka], c.l[kc], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(a.u[ka], c.u[kc], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a.margin, c.margin, rtol=1e-12, atol=1e-12)
    assert (a.verdict == c.verdict).all()


def _skip_variants():
    base = wl.random_small_res(21, 3, 4, 2, 3)
    yield "two blocks", base
    # skip taken from the input itself and from a pre-activation layer
    rng = np.random.default_rng(22)
    n = 3
    mk = lambda: Layer("affine", rng.normal(size=(n, n)).astype(np.float32), rng.normal(size=n).astype(np.float32) * 0.3)
    yield "skip from the input", Network(n, [mk(), Layer("relu"), mk(), Layer("add", skip=0), Layer("relu"), mk()])
    yield "skip from an affine layer", Network(n, [mk(), Layer("relu"), mk(), Layer("relu"), mk(), Layer("add", skip=3),
                                                   Layer("relu"), mk()])
    yield "nested skips", Network(n, [mk(), Layer("relu"), mk(), Layer("relu"), mk(), Layer("add", skip=4), mk(),
                                      Layer("add", skip=2), Layer("relu"), mk()])
    yield "the layer below added twice", Network(n, [mk(), Layer("relu"), mk(), Layer("add", skip=3), mk()])
    # Add layers whose operand below is a ReLU layer or another Add layer (no weight rows to start from)
    yield "Add above a ReLU layer", Network(n, [mk(), Layer("relu"), mk(), Layer("relu"), Layer("add", skip=2), mk()])
    yield "Add above an Add layer", Network(n, [mk(), Layer("relu"), mk(), Layer("add", skip=2), Layer("add", skip=1),
                                                Layer("relu"), mk()])
    yield "ReLU layer added to itself", Network(n, [mk(), Layer("relu"), Layer("add", skip=2), Layer("relu"), mk()])


@pytest.mark.parametrize("name,net", list(_skip_variants()))
@pytest.mark.parametrize("depth,depth_last", [(-1, None), (0, None), (1, None), (2, None), (3, -1), (0, -1)])
def test_c_oracle_matches_neuron_level_transcription(name, net, depth, depth_last):
    x, lo, hi = _box(23, net.n_in, 2, 0.25)
    n_out = net.sizes()[-1]
    label = np.array([0, n_out - 1], np.int32)
    o = oracle.run(net, lo, hi, label=label, max_depth=depth, max_depth_last=depth_last)
    for bi in range(2):
        shapes, margins, verdict = neuron_level.certify(net, lo[bi], hi[bi], label=int(label[bi]), max_iters=depth,
                                                        max_iters_last=depth_last)
        for k in range(len(net.layers) + 1):
            np.testing.assert_allclose(o.l[k][bi], [s.l for s in shapes[k]], rtol=1e-10, atol=1e-10, err_msg=f"{name} l[{k}]")
            np.testing.assert_allclose(o.u[k][bi], [s.u for s in shapes[k]], rtol=1e-10, atol=1e-10, err_msg=f"{name} u[{k}]")
        np.testing.assert_allclose(o.margin[bi], margins, rtol=1e-10, atol=1e-10)
        assert o.verdict[bi] == verdict


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_bounds_contain_sampled_activations(seed):
    net = wl.random_small_res(seed, 6, 8, 2, 4)
    x, lo, hi = _box(seed + 1, 6, 3, 0.1)
    o = oracle.run(net, lo, hi)
    rng = np.random.default_rng(seed + 2)
    for _ in range(200):
        t = rng.uniform(size=lo.shape)
        p = lo.astype(np.float64) * (1 - t) + hi.astype(np.float64) * t
        acts = wl.forward(net, p)
        for k, a in enumerate(acts):
            assert (a >= o.l[k] - 1e-9).all() and (a <= o.u[k] + 1e-9).all(), k
    # corners of the box as well
    for p in (lo.astype(np.float64), hi.astype(np.float64)):
        for k, a in enumerate(wl.forward(net, p)):
            assert (a >= o.l[k] - 1e-9).all() and (a <= o.u[k] + 1e-9).all()


def test_symbolic_export_of_a_residual_layer_reproduces_its_bounds():
    net = wl.random_small_res(41, 4, 5, 1, 3)
    x, lo, hi = _box(42, 4, 2, 0.2)
    k = 6                                                  # the Add layer
    o = oracle.run(net, lo, hi, sym_layer=k)
    lo64, hi64 = lo.astype(np.float64), hi.astype(np.float64)
    cl, cu = o.sym["cl"], o.sym["cu"]
    l = o.sym["kl"] + (np.maximum(cl, 0) * lo64[:, None, :] + np.minimum(cl, 0) * hi64[:, None, :]).sum(-1)
    u = o.sym["ku"] + (np.maximum(cu, 0) * hi64[:, None, :] + np.minimum(cu, 0) * lo64[:, None, :]).sum(-1)
    np.testing.assert_allclose(l, o.l[k], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(u, o.u[k], rtol=1e-12, atol=1e-12)
    # and the input-level expressions are sound: evaluate them on sampled points
    rng = np.random.default_rng(43)
    for _ in range(50):
        t = rng.uniform(size=lo.shape)
        p = lo64 * (1 - t) + hi64 * t
        a = wl.forward(net, p)[k]
        assert ((cl * p[:, None, :]).sum(-1) + o.sym["kl"] <= a + 1e-9).all()
        assert ((cu * p[:, None, :]).sum(-1) + o.sym["ku"] >= a - 1e-9).all()


def test_malformed_add_layers_are_rejected():
    net = wl.random_small_res(51, 3, 4, 1, 2)
    bad = copy.deepcopy(net)
    bad.layers[5].skip = 0                                # input has 3 neurons, the block 4
    with pytest.raises((ValueError, AssertionError)):
        oracle.run(bad, *_box(52, 3, 1, 0.1)[1:])
    with pytest.raises((ValueError, AssertionError)):
        oracle.run(net, *_box(52, 3, 1, 0.1)[1:], certifier="reusecert")


def test_relu_layer_added_to_itself_is_twice_the_layer():
    """ReLU(h) + ReLU(h) = 2 ReLU(h): the network equals the chain network with the affine layer 2 I in place of the Add
    layer (an Add layer whose operand below is a ReLU layer starts from coefficient 1 on each operand)."""
    rng = np.random.default_rng(41)
    n0, m, k = 4, 5, 3
    A1 = Layer("affine", rng.normal(size=(m, n0)).astype(np.float32), rng.normal(size=m).astype(np.float32))
    A2 = Layer("affine", rng.normal(size=(k, m)).astype(np.float32), rng.normal(size=k).astype(np.float32))
    res = Network(n0, [A1, Layer("relu"), Layer("add", skip=2), Layer("relu"), A2])
    twice = Layer("affine", 2 * np.eye(m, dtype=np.float32), np.zeros(m, np.float32))
    chain = Network(n0, [A1, Layer("relu"), twice, Layer("relu"), A2])
    x, lo, hi = _box(42, n0, 3, 0.4)
    label = np.array([0, 1, 2], np.int32)
    a = oracle.run(res, lo, hi, label=label)
    c = oracle.run(chain, lo, hi, label=label)
    for k_ in range(1, 6):
        np.testing.assert_allclose(a.l[k_], c.l[k_], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(a.u[k_], c.u[k_], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a.margin, c.margin, rtol=1e-12, atol=1e-12)
