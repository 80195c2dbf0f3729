"""Parity of the HIP path on residual networks (Add layers: expressions with blocks on two layers at once)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle                                            # noqa: E402
from paper_2507_20055_amd import workloads as wl         # noqa: E402
from paper_2507_20055_amd.workloads import Layer, Network  # noqa: E402
from tests.parity_util import compare_with_oracle        # noqa: E402


def _binding():
    from paper_2507_20055_amd import binding
    return binding


def _check(net, lo, hi, label, fuses=(1, 0)):
    b = _binding()
    gnet = b.Network(net)
    o = oracle.run(net, lo, hi, label=label)
    for fuse in fuses:
        g = gnet.certify(lo, hi, label, fuse=fuse)
        compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


@pytest.mark.parametrize("seed,n_in,width,blocks,n_out,B", [(1, 6, 8, 1, 3, 2), (2, 20, 40, 2, 5, 3), (3, 33, 70, 3, 10, 4),
                                                           (4, 64, 130, 2, 10, 5)])
def test_small_residual_fc(seed, n_in, width, blocks, n_out, B):
    net = wl.random_small_res(seed, n_in, width, blocks, n_out)
    x, lo, hi = wl.random_box(seed + 10, n_in, B, 0.05)
    label = np.arange(B, dtype=np.int32) % n_out
    _check(net, lo, hi, label)


def _mk(rng, n_to, n_from):
    return Layer("affine", (rng.normal(size=(n_to, n_from)) / np.sqrt(n_from)).astype(np.float32),
                 (rng.normal(size=n_to) * 0.3).astype(np.float32))


def _variants():
    rng = np.random.default_rng(7)
    n = 36
    yield "skip from the input", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("add", skip=0), Layer("relu"),
                                             _mk(rng, 4, n)])
    yield "skip from an affine layer", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("relu"), _mk(rng, n, n),
                                                   Layer("add", skip=3), Layer("relu"), _mk(rng, 4, n)])
    yield "nested skips", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("relu"), _mk(rng, n, n),
                                      Layer("add", skip=4), _mk(rng, n, n), Layer("add", skip=2), Layer("relu"), _mk(rng, 5, n)])
    yield "two skips onto one layer", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("add", skip=2),
                                                  _mk(rng, n, n), Layer("add", skip=2), Layer("relu"), _mk(rng, 3, n)])
    yield "affine directly above the Add layer", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("add", skip=2),
                                                             _mk(rng, 6, n)])
    yield "Add as the last layer", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("add", skip=1)])
    # Add layers whose operand below has no weight rows (a ReLU layer, another Add layer): the expressions start as unit rows
    yield "Add above a ReLU layer", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("relu"), Layer("add", skip=2),
                                                _mk(rng, 5, n)])
    yield "Add above an Add layer", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("add", skip=2),
                                                Layer("add", skip=1), Layer("relu"), _mk(rng, 4, n)])
    yield "pre-activation blocks", Network(n, [_mk(rng, n, n), Layer("relu"), _mk(rng, n, n), Layer("relu"), Layer("add", skip=1),
                                               _mk(rng, n, n), Layer("relu"), Layer("add", skip=5), _mk(rng, 4, n)])


@pytest.mark.parametrize("name,net", list(_variants()))
def test_skip_topologies(name, net):
    x, lo, hi = wl.random_box(8, net.n_in, 3, 0.04)
    n_out = net.sizes()[-1]
    label = (np.arange(3, dtype=np.int32) % n_out) if net.layers[-1].kind == "affine" else None
    _check(net, lo, hi, label)


@pytest.mark.parametrize("shape,width,blocks,k,tail,fcs", [((2, 6, 6), 4, 1, 3, [], [5, 3]),
                                                          ((3, 8, 8), 8, 2, 3, [(8, 4, 2, 1)], [10, 4]),
                                                          ((1, 9, 7), 16, 1, 3, [(8, 3, 2, 0)], [6, 3]),
                                                          ((3, 10, 10), 8, 1, 5, [(16, 4, 2, 1)], [7, 4])])
def test_small_residual_conv(shape, width, blocks, k, tail, fcs):
    net = wl.random_small_res_conv(9, shape, width, blocks, k, tail, fcs)
    B = 3
    x, lo, hi = wl.random_box(10, net.n_in, B, 0.03)
    label = np.arange(B, dtype=np.int32) % fcs[-1]
    _check(net, lo, hi, label)


def _conv_layer(rng, Co, shape, k, s_, p):
    Wt = (rng.normal(size=(Co, shape[0], k, k)) * np.sqrt(2.0 / (shape[0] * k * k))).astype(np.float32)
    return Layer("conv", Wt, (rng.normal(size=Co) * 0.1).astype(np.float32), stride=s_, pad=p, in_shape=shape)


def test_add_above_relu_on_a_convolutional_network():
    """Spatial layers: the Add layer's own expressions are 1x1 identity cores over the ReLU layer below it."""
    rng = np.random.default_rng(17)
    shape = (2, 7, 6)
    c1 = _conv_layer(rng, 4, shape, 3, 1, 1)
    c2 = _conv_layer(rng, 4, c1.out_shape, 3, 1, 1)
    c3 = _conv_layer(rng, 8, c2.out_shape, 4, 2, 1)
    n3 = int(np.prod(c3.out_shape))
    net = Network(int(np.prod(shape)), [c1, Layer("relu"), c2, Layer("relu"), Layer("add", skip=2), c3, Layer("relu"),
                                        _mk(rng, 6, n3), Layer("relu"), _mk(rng, 3, 6)])
    x, lo, hi = wl.random_box(18, net.n_in, 3, 0.03)
    label = np.array([0, 1, 2], np.int32)
    _check(net, lo, hi, label)
    b = _binding()
    gnet = b.Network(net)
    for depth, last in ((0, None), (1, None), (2, None), (3, None), (2, -1)):
        o = oracle.run(net, lo, hi, label=label, max_depth=depth, max_depth_last=last)
        g = gnet.certify(lo, hi, label, max_backsub_depth=depth, final_backsub_depth=-2 if last is None else last)
        compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


def test_reusecert_is_refused_on_residual_networks():
    b = _binding()
    net = wl.random_small_res(5, 6, 8, 1, 3)
    x, lo, hi = wl.random_box(6, 6, 2, 0.05)
    gnet = b.Network(net)
    with pytest.raises(b.DpcError) as e:
        gnet.certify(lo, hi, None, certifier="reusecert")
    assert e.value.code == 2
    gnet.close()


def _depth_nets():
    yield "fc", wl.random_small_res(41, 12, 36, 2, 4)
    for name, net in _variants():
        yield name, net
    yield "conv", wl.random_small_res_conv(42, (2, 6, 6), 8, 1, 3, [(8, 4, 2, 1)], [5, 3])
    yield "conv, two blocks", wl.random_small_res_conv(43, (3, 8, 8), 4, 2, 3, [], [6, 3])


@pytest.mark.parametrize("name,net", list(_depth_nets()))
def test_depth_limited_traversals_on_residual_networks(name, net):
    """DeepPoly_p, IBP (p = 0) and CROWN-IBP on networks with Add layers: a traversal may stop while a block still waits
    on a skip connection; the expression is then concretised over both layers it holds."""
    b = _binding()
    B = 2
    x, lo, hi = wl.random_box(44, net.n_in, B, 0.03)
    n_out = net.sizes()[-1]
    label = (np.arange(B, dtype=np.int32) % n_out) if net.layers[-1].kind == "affine" else None
    gnet = b.Network(net)
    for depth, last in ((0, None), (1, None), (2, None), (3, None), (4, None), (5, None), (0, -1), (2, -1)):
        o = oracle.run(net, lo, hi, label=label, max_depth=depth, max_depth_last=last)
        for fuse in (1, 0):
            g = gnet.certify(lo, hi, label, max_backsub_depth=depth, final_backsub_depth=-2 if last is None else last, fuse=fuse)
            try:
                compare_with_oracle(net, lo, hi, g, o, label)
            except AssertionError as e:
                raise AssertionError(f"{name}: depth {depth}, last {last}, fuse {fuse}: {e}")
    gnet.close()


def test_graph_replay_on_a_residual_network():
    import torch
    b = _binding()
    net = wl.random_small_res(12, 20, 40, 2, 5)
    gnet = b.Network(net)
    stream = torch.cuda.Stream()
    prev = None
    for rep in range(4):
        x, lo, hi = wl.random_box(20 + rep, 20, 3, 0.05)
        label = np.arange(3, dtype=np.int32) % 5
        o = oracle.run(net, lo, hi, label=label)
        prev = gnet.certify(lo, hi, label, stream=stream.cuda_stream, reuse=prev)
        compare_with_oracle(net, lo, hi, prev, o, label)
    gnet.close()


@pytest.mark.parametrize("name,sample", [("res_fc", 4), ("res_conv", 1)])
def test_residual_workloads_full_batch_gpu_sampled_oracle(name, sample):
    """The bench configuration at its full batch on the GPU; the oracle bounds a prefix of the inputs (the library
    treats inputs independently, so the prefix's results must not depend on the batch)."""
    b = _binding()
    w = wl.make_workload(name)
    gnet = b.Network(w.net)
    g = gnet.certify(w.lo, w.hi, w.label)
    o = oracle.run(w.net, w.lo[:sample], w.hi[:sample], label=w.label[:sample])

    class Prefix:
        def concrete(self, k):
            l, u = g.concrete(k)
            return l[:sample], u[:sample]

        def relaxation(self, k):
            return tuple(a[:sample] for a in g.relaxation(k))

        def verdict(self):
            v, m = g.verdict()
            return v[:sample], m[:sample]

    compare_with_oracle(w.net, w.lo[:sample], w.hi[:sample], Prefix(), o, w.label[:sample], max_flipped_inputs=1)
    gl, gu = g.concrete(len(w.net.layers))
    assert (gl <= gu).all()
    gnet.close()


@pytest.mark.parametrize("conv", [False, True])
def test_symbolic_bounds_of_the_output_layer_on_a_residual_network(conv):
    """keep_symbolic = 1: the input-level expressions of the last layer against the oracle's export."""
    b = _binding()
    if conv:
        net = wl.random_small_res_conv(15, (2, 6, 6), 4, 1, 3, [], [5, 3])
    else:
        net = wl.random_small_res(15, 12, 20, 2, 4)
    B = 2
    x, lo, hi = wl.random_box(16, net.n_in, B, 0.04)
    nl = len(net.layers)
    o = oracle.run(net, lo, hi, sym_layer=nl)
    gnet = b.Network(net)
    g = gnet.certify(lo, hi, None, keep_symbolic=1)
    for side, (ck, kk) in enumerate((("cl", "kl"), ("cu", "ku"))):
        c, k = g.symbolic(nl, side)
        scale = np.abs(o.sym[ck]).max()
        assert np.abs(c - o.sym[ck]).max() <= 1e-4 * scale + 1e-6
        np.testing.assert_allclose(k, o.sym[kk], rtol=1e-4, atol=1e-5)
    compare_with_oracle(net, lo, hi, g, o, None)
    gnet.close()


def test_empty_and_single_input_batches_on_a_residual_network():
    b = _binding()
    net = wl.random_small_res(17, 10, 16, 1, 3)
    gnet = b.Network(net)
    g0 = gnet.certify(np.zeros((0, 10), np.float32), np.zeros((0, 10), np.float32), np.zeros((0,), np.int32))
    assert g0.concrete(len(net.layers))[0].shape == (0, 3)
    x, lo, hi = wl.random_box(18, 10, 1, 0.05)
    label = np.array([1], np.int32)
    o = oracle.run(net, lo, hi, label=label)
    compare_with_oracle(net, lo, hi, gnet.certify(lo, hi, label), o, label)
    gnet.close()
