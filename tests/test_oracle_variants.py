"""Pins for the oracle's ReuseCert and SkipPoly variants (Appendix C): a hand-derived example, closed forms,
special cases that reduce to DeepPoly, brute force against the neuron-level transcription, sampled soundness.
Nothing here touches the GPU library."""
import numpy as np
import pytest

import oracle
from oracle import neuron_level
from paper_2507_20055_amd import workloads as wl
from tests.test_oracle_pins import read_golden, fc_net, _samples


def _hand_net():
    g = read_golden("net_2_2_2_2.txt")
    net = fc_net(2, [(g["W1"].reshape(2, 2), g["b1"]), (g["W2"].reshape(2, 2), g["b2"]), (g["W3"].reshape(2, 2), g["b3"])])
    return g, net


def test_reusecert_hand_example():
    g, net = _hand_net()
    e = read_golden("reusecert_2_2_2_2.txt")
    lo, hi, lab = g["lo"][None], g["hi"][None], g["label"].astype(np.int32)
    tol = dict(rtol=0, atol=1e-12)
    r = oracle.run(net, lo, hi, label=lab, certifier="reusecert", sym_layer=3)
    np.testing.assert_allclose(r.l[1][0], e["l1"], **tol)
    np.testing.assert_allclose(r.u[1][0], e["u1"], **tol)
    np.testing.assert_allclose(r.l[3][0], e["l3"], **tol)
    np.testing.assert_allclose(r.u[3][0], e["u3"], **tol)
    np.testing.assert_allclose(r.lam[4][0], e["lam2"], **tol)
    np.testing.assert_allclose(r.mu[4][0], e["mu2"], **tol)
    np.testing.assert_allclose(r.nu[4][0], e["nu2"], **tol)
    np.testing.assert_allclose(r.sym["cl"][0].ravel(), e["stored3_lower_coeff"], **tol)
    np.testing.assert_allclose(r.sym["kl"][0], e["stored3_lower_const"], **tol)
    np.testing.assert_allclose(r.sym["cu"][0].ravel(), e["stored3_upper_coeff"], **tol)
    np.testing.assert_allclose(r.sym["ku"][0], e["stored3_upper_const"], **tol)
    np.testing.assert_allclose(r.l[5][0], e["l5"], **tol)
    np.testing.assert_allclose(r.u[5][0], e["u5"], **tol)
    np.testing.assert_allclose(r.margin[0], e["margin"], **tol)
    assert r.verdict[0] == int(e["verdict"][0])
    # the neuron-level transcription reaches the same numbers
    sh, m, v = neuron_level.certify(net, lo[0], hi[0], label=int(lab[0]), certifier="reusecert")
    np.testing.assert_allclose([s.l for s in sh[5]], e["l5"], **tol)
    np.testing.assert_allclose([s.u for s in sh[5]], e["u5"], **tol)
    np.testing.assert_allclose(m, e["margin"], **tol)
    assert v == 0 and all(s.l == 0.0 and s.u == 0.0 for s in sh[3] + sh[2] + sh[4])     # middle layers: (0, 0, L, U)


@pytest.mark.parametrize("seed,dims", [(1, [5, 7, 4]), (2, [3, 6, 2]), (3, [8, 3])])
def test_reusecert_equals_deeppoly_up_to_two_affine_layers(seed, dims):
    """One ReLU layer: the single replacement step of ReuseCert is the whole DeepPoly traversal."""
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 5, dims[0], 3, 0.4)
    lab = np.arange(3, dtype=np.int32) % dims[-1]
    a = oracle.run(net, lo, hi, label=lab)
    b = oracle.run(net, lo, hi, label=lab, certifier="reusecert")
    for k in range(1, len(net.layers) + 1, 2):
        np.testing.assert_allclose(b.l[k], a.l[k], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(b.u[k], a.u[k], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(b.margin, a.margin, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed,dims", [(4, [3, 4, 4, 3]), (5, [2, 5, 4, 5, 3]), (6, [4, 3, 3, 3, 3, 2])])
def test_reusecert_matches_neuron_level(seed, dims):
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 7, dims[0], 2, 0.5)
    lab = np.array([0, 1], np.int32)
    last = len(net.layers)
    for sym in range(1, last + 1, 2):
        r = oracle.run(net, lo, hi, label=lab, certifier="reusecert", sym_layer=sym)
        for bi in range(2):
            sh, m, v = neuron_level.certify(net, lo[bi], hi[bi], label=int(lab[bi]), certifier="reusecert")
            np.testing.assert_allclose(m, r.margin[bi], rtol=1e-10, atol=1e-12)
            assert v == r.verdict[bi]
            for k in (1, last):
                np.testing.assert_allclose([s.l for s in sh[k]], r.l[k][bi], rtol=1e-10, atol=1e-12)
                np.testing.assert_allclose([s.u for s in sh[k]], r.u[k][bi], rtol=1e-10, atol=1e-12)
            for k in range(1, last, 2):      # concretised stored bounds, as the ReLU transformer computes them
                np.testing.assert_allclose([s.cl for s in sh[k]], r.l[k][bi], rtol=1e-10, atol=1e-12)
                np.testing.assert_allclose([s.cu for s in sh[k]], r.u[k][bi], rtol=1e-10, atol=1e-12)
            if sym < last:                   # stored input-level expressions of a middle (or the first) layer
                for i, s in enumerate(sh[sym]):
                    cl = [s.L.terms.get((0, p), 0.0) for p in range(dims[0])]
                    cu = [s.U.terms.get((0, p), 0.0) for p in range(dims[0])]
                    assert all(n[0] == 0 for n in list(s.L.terms) + list(s.U.terms))     # input level only
                    np.testing.assert_allclose(cl, r.sym["cl"][bi, i], rtol=1e-10, atol=1e-12)
                    np.testing.assert_allclose(cu, r.sym["cu"][bi, i], rtol=1e-10, atol=1e-12)
                    np.testing.assert_allclose(s.L.const, r.sym["kl"][bi, i], rtol=1e-10, atol=1e-12)
                    np.testing.assert_allclose(s.U.const, r.sym["ku"][bi, i], rtol=1e-10, atol=1e-12)


def test_reusecert_closed_forms():
    rng = np.random.default_rng(11)
    dims = [5, 6, 6, 6, 4]
    net = wl.random_small_net(12, dims)
    x, lo, hi = wl.random_box(13, 5, 2, 0.2)
    # eps = 0: every stored bound collapses onto the forward pass
    r = oracle.run(net, x, x, certifier="reusecert")
    acts = wl.forward(net, x.astype(np.float64))
    for k in range(1, len(net.layers) + 1, 2):
        np.testing.assert_allclose(r.l[k], acts[k], rtol=1e-9, atol=1e-9)
        np.testing.assert_allclose(r.u[k], acts[k], rtol=1e-9, atol=1e-9)
    # all neurons stably active (large biases, non-negative later weights): the network is linear on the box and
    # the bounds are those of the composed affine map, W+ lo + W- hi + b
    for i, L in enumerate(net.layers):
        if L.kind == "affine":
            if i > 0:
                L.W = np.abs(L.W)
            L.b = (np.abs(L.b) + 10.0).astype(np.float32)
    r = oracle.run(net, lo, hi, certifier="reusecert")
    Weff, beff = np.eye(5), np.zeros(5)
    for L in net.layers:
        if L.kind == "affine":
            Weff = L.W.astype(np.float64) @ Weff
            beff = L.W.astype(np.float64) @ beff + L.b.astype(np.float64)
    lo64, hi64 = lo.astype(np.float64), hi.astype(np.float64)
    pos, neg = np.maximum(Weff, 0), np.minimum(Weff, 0)
    last = len(net.layers)
    np.testing.assert_allclose(r.l[last], lo64 @ pos.T + hi64 @ neg.T + beff, rtol=1e-10)
    np.testing.assert_allclose(r.u[last], hi64 @ pos.T + lo64 @ neg.T + beff, rtol=1e-10)
    del rng


@pytest.mark.parametrize("seed,dims,eps", [(21, [4, 6, 6, 3], 0.3), (22, [6, 8, 8, 8, 4], 0.15)])
def test_reusecert_soundness_by_sampling(seed, dims, eps):
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 50, dims[0], 2, eps)
    lab = np.array([0, 1], np.int32)
    last = len(net.layers)
    for sym in range(1, last + 1, 2):
        r = oracle.run(net, lo, hi, label=lab, certifier="reusecert", sym_layer=sym)
        for bi in range(2):
            pts = _samples(lo[bi].astype(np.float64), hi[bi].astype(np.float64), 5000, seed)
            acts = wl.forward(net, pts)
            for k in range(1, last + 1, 2):
                assert np.all(acts[k] >= r.l[k][bi] - 1e-9) and np.all(acts[k] <= r.u[k][bi] + 1e-9)
            if sym < last:       # the stored expressions bound the neuron pointwise, and concretise to l, u
                symlo = pts @ r.sym["cl"][bi].T + r.sym["kl"][bi]
                symup = pts @ r.sym["cu"][bi].T + r.sym["ku"][bi]
                assert np.all(symlo <= acts[sym] + 1e-9) and np.all(acts[sym] <= symup + 1e-9)
                assert np.all(symlo >= r.l[sym][bi] - 1e-9) and np.all(symup <= r.u[sym][bi] + 1e-9)
            y = acts[-1]
            t = lab[bi]
            others = [o for o in range(dims[-1]) if o != t]
            assert np.all(r.margin[bi] <= (y[:, [t]] - y[:, others]).min(axis=0) + 1e-9)


def test_reusecert_rejects_unsupported_topology():
    net = wl.Network(n_in=3)
    net.layers.append(wl.Layer("affine", np.ones((2, 3), np.float32), np.zeros(2, np.float32)))
    net.layers.append(wl.Layer("affine", np.ones((2, 2), np.float32), np.zeros(2, np.float32)))
    with pytest.raises(ValueError):
        oracle.run(net, np.zeros((1, 3), np.float32), np.ones((1, 3), np.float32), certifier="reusecert")


@pytest.mark.parametrize("seed,dims", [(31, [3, 4, 4, 3]), (32, [2, 5, 4, 5, 3])])
def test_skippoly_computes_deeppoly_bounds(seed, dims):
    """SkipPoly writes the ReLU bounds over the neurons two layers back; the traversal then takes half as many
    steps and reaches the same expressions (Section 6.1: no loss of precision)."""
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 3, dims[0], 1, 0.5)
    r = oracle.run(net, lo, hi, label=np.array([1], np.int32))
    sh, m, v = neuron_level.certify(net, lo[0], hi[0], label=1, certifier="skippoly")
    for k in range(1, len(net.layers) + 1):
        np.testing.assert_allclose([s.l for s in sh[k]], r.l[k][0], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose([s.u for s in sh[k]], r.u[k][0], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(m, r.margin[0], rtol=1e-10, atol=1e-12)
    # and the ReLU neurons' polyhedral bounds really skip a layer
    assert all(n[0] == 0 for s in sh[2] for n in list(s.L.terms) + list(s.U.terms))
    assert all(n[0] == 2 for s in sh[4] for n in list(s.L.terms) + list(s.U.terms))


# ---------------------------------------------------------------- CROWN-IBP (Appendix C): interval bounds, last layer back-substituted
def test_crownibp_hand_example():
    g, net = _hand_net()
    e = read_golden("crownibp_2_2_2_2.txt")
    lo, hi, lab = g["lo"][None], g["hi"][None], g["label"].astype(np.int32)
    tol = dict(rtol=0, atol=1e-12)
    r = oracle.run(net, lo, hi, label=lab, max_depth=0, max_depth_last=-1)
    for k, key in ((3, "3"), (5, "5")):
        np.testing.assert_allclose(r.l[k][0], e["l" + key], **tol)
        np.testing.assert_allclose(r.u[k][0], e["u" + key], **tol)
    np.testing.assert_allclose(r.lam[4][0], e["lam2"], **tol)
    np.testing.assert_allclose(r.mu[4][0], e["mu2"], **tol)
    np.testing.assert_allclose(r.nu[4][0], e["nu2"], **tol)
    np.testing.assert_allclose(r.margin[0], e["margin"], **tol)
    assert r.verdict[0] == 0
    sh, m, v = neuron_level.certify(net, lo[0], hi[0], label=int(lab[0]), max_iters=0, max_iters_last=-1)
    np.testing.assert_allclose([s.l for s in sh[5]], e["l5"], **tol)
    np.testing.assert_allclose([s.u for s in sh[5]], e["u5"], **tol)
    np.testing.assert_allclose(m, e["margin"], **tol)


@pytest.mark.parametrize("seed,dims", [(41, [4, 6, 5, 3]), (42, [3, 5, 5, 5, 4])])
def test_crownibp_structure(seed, dims):
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 2, dims[0], 2, 0.4)
    lab = np.array([0, 1], np.int32)
    last = len(net.layers)
    r = oracle.run(net, lo, hi, label=lab, max_depth=0, max_depth_last=-1)
    ibp = oracle.run(net, lo, hi, max_depth=0)
    full = oracle.run(net, lo, hi, label=lab)
    # hidden layers: plain interval propagation; the last layer is something else (back-substituted bounds need not
    # be tighter than interval bounds, so only the difference is asserted)
    for k in range(1, last):
        np.testing.assert_array_equal(r.l[k], ibp.l[k])
        np.testing.assert_array_equal(r.u[k], ibp.u[k])
    assert not np.allclose(r.l[last], ibp.l[last]) and not np.allclose(r.l[last], full.l[last])
    # brute force: the neuron-level transcription with the same limits
    for bi in range(2):
        sh, m, v = neuron_level.certify(net, lo[bi], hi[bi], label=int(lab[bi]), max_iters=0, max_iters_last=-1)
        np.testing.assert_allclose([s.l for s in sh[last]], r.l[last][bi], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose([s.u for s in sh[last]], r.u[last][bi], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(m, r.margin[bi], rtol=1e-10, atol=1e-12)
        # sound
        pts = _samples(lo[bi].astype(np.float64), hi[bi].astype(np.float64), 4000, seed)
        acts = wl.forward(net, pts)
        for k in range(1, last + 1):
            assert np.all(acts[k] >= r.l[k][bi] - 1e-9) and np.all(acts[k] <= r.u[k][bi] + 1e-9)
    # one hidden layer: its bounds are interval bounds under DeepPoly too, so the two certifiers coincide
    net2 = wl.random_small_net(seed, dims[:2] + dims[-1:])
    a = oracle.run(net2, lo, hi, label=lab % dims[-1])
    b = oracle.run(net2, lo, hi, label=lab % dims[-1], max_depth=0, max_depth_last=-1)
    np.testing.assert_allclose(b.l[3], a.l[3], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(b.margin, a.margin, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- ReuseCert through convolution layers
@pytest.mark.parametrize("convs", [[(3, 3, 1, 1), (4, 4, 2, 1)], [(2, 4, 2, 1), (3, 3, 1, 0)], [(3, 3, 2, 0)]])
def test_reusecert_conv_equals_its_dense_expansion(convs):
    """A convolution layer is an affine layer whose weight matrix is the expanded kernel (Section 3.3): ReuseCert on a
    convolutional network equals ReuseCert on the network with every convolution written out as that matrix (built by
    pushing unit vectors through an ordinary convolution), which the fully-connected pins above cover."""
    from tests.test_oracle_pins import _conv_as_dense
    net = wl.random_small_conv(61, (2, 7, 6), convs, [5, 3])
    dense = wl.Network(n_in=net.n_in)
    for L in net.layers:
        if L.kind == "conv":
            M, b = _conv_as_dense(L)
            dense.layers.append(wl.Layer("affine", M, b))
        else:
            dense.layers.append(L)
    x, lo, hi = wl.random_box(62, net.n_in, 2, 0.05)
    lab = np.array([0, 2], np.int32)
    last = len(net.layers)
    for sym in range(1, last + 1, 2):
        a = oracle.run(net, lo, hi, label=lab, certifier="reusecert", sym_layer=sym)
        d = oracle.run(dense, lo, hi, label=lab, certifier="reusecert", sym_layer=sym)
        for k in range(1, last + 1, 2):
            np.testing.assert_allclose(a.l[k], d.l[k], rtol=1e-11, atol=1e-11)
            np.testing.assert_allclose(a.u[k], d.u[k], rtol=1e-11, atol=1e-11)
        for key in ("cl", "kl", "cu", "ku"):
            np.testing.assert_allclose(a.sym[key], d.sym[key], rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(a.margin, d.margin, rtol=1e-11, atol=1e-11)
        assert np.array_equal(a.verdict, d.verdict)


def test_reusecert_conv_matches_neuron_level_and_is_sound():
    net = wl.random_small_conv(63, (1, 5, 4), [(2, 3, 1, 1), (3, 2, 1, 0)], [4, 3])
    x, lo, hi = wl.random_box(64, net.n_in, 2, 0.3)
    lab = np.array([1, 2], np.int32)
    last = len(net.layers)
    r = oracle.run(net, lo, hi, label=lab, certifier="reusecert")
    for bi in range(2):
        sh, m, v = neuron_level.certify(net, lo[bi], hi[bi], label=int(lab[bi]), certifier="reusecert")
        np.testing.assert_allclose(m, r.margin[bi], rtol=1e-10, atol=1e-12)
        assert v == r.verdict[bi]
        for k in (1, last):
            np.testing.assert_allclose([s.l for s in sh[k]], r.l[k][bi], rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose([s.u for s in sh[k]], r.u[k][bi], rtol=1e-10, atol=1e-12)
        for k in range(1, last, 2):
            np.testing.assert_allclose([s.cl for s in sh[k]], r.l[k][bi], rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose([s.cu for s in sh[k]], r.u[k][bi], rtol=1e-10, atol=1e-12)
        pts = _samples(lo[bi].astype(np.float64), hi[bi].astype(np.float64), 3000, 65)
        acts = wl.forward(net, pts)
        for k in range(1, last + 1, 2):
            assert np.all(acts[k] >= r.l[k][bi] - 1e-9) and np.all(acts[k] <= r.u[k][bi] + 1e-9)
