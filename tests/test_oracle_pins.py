"""Pins for the CPU oracle: hand-derived examples, closed forms, invariants,
library reductions and brute force.  None of these compare the oracle with
itself, and none touch the GPU library."""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import neuron_level
from paper_2507_20055_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    d = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            d[k] = np.array([float(t) for t in v])
    return d


def fc_net(n_in, mats):
    net = wl.Network(n_in=n_in)
    for i, (W, b) in enumerate(mats):
        net.layers.append(wl.Layer("affine", np.asarray(W, np.float32), np.asarray(b, np.float32)))
        if i != len(mats) - 1:
            net.layers.append(wl.Layer("relu"))
    return net


# ---------------------------------------------------------------- hand-derived examples
def test_hand_2_2_2():
    g = read_golden("net_2_2_2.txt")
    net = fc_net(2, [(g["W1"].reshape(2, 2), g["b1"]), (g["W2"].reshape(2, 2), g["b2"])])
    r = oracle.run(net, g["lo"][None], g["hi"][None], label=g["label"].astype(np.int32), sym_layer=3)
    tol = dict(rtol=0, atol=1e-12)
    np.testing.assert_allclose(r.l[1][0], g["l1"], **tol)
    np.testing.assert_allclose(r.u[1][0], g["u1"], **tol)
    np.testing.assert_allclose(r.lam[2][0], g["lam"], **tol)
    np.testing.assert_allclose(r.mu[2][0], g["mu"], **tol)
    np.testing.assert_allclose(r.nu[2][0], g["nu"], **tol)
    np.testing.assert_allclose(r.l[2][0], g["l2"], **tol)
    np.testing.assert_allclose(r.u[2][0], g["u2"], **tol)
    np.testing.assert_allclose(r.l[3][0], g["l3"], **tol)
    np.testing.assert_allclose(r.u[3][0], g["u3"], **tol)
    np.testing.assert_allclose(r.sym["cl"][0].ravel(), g["sym_lower_coeff"], **tol)
    np.testing.assert_allclose(r.sym["kl"][0], g["sym_lower_const"], **tol)
    np.testing.assert_allclose(r.sym["cu"][0].ravel(), g["sym_upper_coeff"], **tol)
    np.testing.assert_allclose(r.sym["ku"][0], g["sym_upper_const"], **tol)
    np.testing.assert_allclose(r.margin[0], g["margin"], **tol)
    assert r.verdict[0] == int(g["verdict"][0])
    # the property row's lower expression over the input (derived in the fixture's header)
    m = oracle.run(net, g["lo"][None], g["hi"][None], label=g["label"].astype(np.int32), sym_layer=4)
    np.testing.assert_allclose(m.sym["cl"][0].ravel(), g["margin_sym_coeff"], **tol)
    np.testing.assert_allclose(m.sym["kl"][0], g["margin_sym_const"], **tol)


def test_hand_2_2_2_2():
    g = read_golden("net_2_2_2_2.txt")
    net = fc_net(2, [(g["W1"].reshape(2, 2), g["b1"]), (g["W2"].reshape(2, 2), g["b2"]),
                     (g["W3"].reshape(2, 2), g["b3"])])
    r = oracle.run(net, g["lo"][None], g["hi"][None], label=g["label"].astype(np.int32), sym_layer=5)
    tol = dict(rtol=0, atol=1e-12)
    np.testing.assert_allclose(r.l[1][0], g["l1"], **tol)
    np.testing.assert_allclose(r.u[1][0], g["u1"], **tol)
    for k, s in ((2, "1"), (4, "2")):
        np.testing.assert_allclose(r.lam[k][0], g["lam" + s], **tol)
        np.testing.assert_allclose(r.mu[k][0], g["mu" + s], **tol)
        np.testing.assert_allclose(r.nu[k][0], g["nu" + s], **tol)
    np.testing.assert_allclose(r.l[3][0], g["l3"], **tol)
    np.testing.assert_allclose(r.u[3][0], g["u3"], **tol)
    np.testing.assert_allclose(r.l[5][0], g["l5"], **tol)
    np.testing.assert_allclose(r.u[5][0], g["u5"], **tol)
    np.testing.assert_allclose(r.sym["cl"][0].ravel(), g["sym_lower_coeff"], **tol)
    np.testing.assert_allclose(r.sym["kl"][0], g["sym_lower_const"], **tol)
    np.testing.assert_allclose(r.sym["cu"][0].ravel(), g["sym_upper_coeff"], **tol)
    np.testing.assert_allclose(r.sym["ku"][0], g["sym_upper_const"], **tol)
    np.testing.assert_allclose(r.margin[0], g["margin"], **tol)
    assert r.verdict[0] == 0


@pytest.mark.parametrize("l,u,lam,mu,nu", [
    (-1.0, 1.0, 1.0, 0.5, 0.5),      # tie l+u == 0 goes to the ">=" branch
    (-1.0, 0.5, 0.0, 1.0 / 3.0, 1.0 / 3.0),
    (0.0, 2.0, 1.0, 1.0, 0.0),       # l >= 0 tested first
    (-2.0, 0.0, 0.0, 0.0, 0.0),      # then u <= 0
    (0.5, 2.0, 1.0, 1.0, 0.0),
    (-2.0, -0.5, 0.0, 0.0, 0.0),
])
def test_relu_branches(l, u, lam, mu, nu):
    # one input neuron in [l, u], identity affine, ReLU, identity affine
    net = fc_net(1, [([[1.0]], [0.0]), ([[1.0]], [0.0])])
    r = oracle.run(net, np.array([[l]], np.float32), np.array([[u]], np.float32))
    assert r.lam[2][0, 0] == lam
    np.testing.assert_allclose(r.mu[2][0, 0], mu, rtol=1e-7)
    np.testing.assert_allclose(r.nu[2][0, 0], nu, rtol=1e-7, atol=1e-15)
    assert r.l[2][0, 0] == max(l, 0.0) and r.u[2][0, 0] == max(u, 0.0)
    # upper bound of relu over [l,u] via the chord is max(u,0); lower via lambda
    np.testing.assert_allclose(r.u[3][0, 0], max(u, 0.0), rtol=1e-7, atol=1e-15)
    np.testing.assert_allclose(r.l[3][0, 0], lam * l, rtol=1e-7, atol=1e-15)


# ---------------------------------------------------------------- closed forms
def _affine_only(net):
    """Drop the ReLU layers (test helper)."""
    out = wl.Network(n_in=net.n_in)
    out.layers = [L for L in net.layers if L.kind != "relu"]
    return out


def test_no_relu_is_exact_linear_bound():
    net = _affine_only(wl.random_small_net(5, [7, 9, 6, 4]))
    x, lo, hi = wl.random_box(11, 7, 3, 0.2)
    r = oracle.run(net, lo, hi)
    Weff = np.eye(7)
    beff = np.zeros(7)
    for k, L in enumerate(net.layers, start=1):
        W = L.W.astype(np.float64)
        Weff = W @ Weff
        beff = W @ beff + L.b.astype(np.float64)
        Wp, Wn = np.maximum(Weff, 0), np.minimum(Weff, 0)
        lo64, hi64 = lo.astype(np.float64), hi.astype(np.float64)
        np.testing.assert_allclose(r.l[k], lo64 @ Wp.T + hi64 @ Wn.T + beff, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(r.u[k], hi64 @ Wp.T + lo64 @ Wn.T + beff, rtol=1e-12, atol=1e-12)


def test_eps_zero_is_forward_pass():
    net = wl.random_small_net(6, [8, 10, 10, 5])
    x, _, _ = wl.random_box(12, 8, 4, 0.0)
    r = oracle.run(net, x, x)
    acts = wl.forward(net, x.astype(np.float64))
    for k in range(len(acts)):
        np.testing.assert_allclose(r.l[k], acts[k], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(r.u[k], acts[k], rtol=1e-12, atol=1e-12)


def test_all_active_net_is_linear():
    net = wl.random_small_net(7, [6, 8, 8, 3])
    first = True
    for L in net.layers:
        if L.kind == "affine":
            if not first:
                L.W = np.abs(L.W)        # positive weights on positive activations
            first = False
            L.b = (L.b + np.float32(50.0)).astype(np.float32)   # every pre-activation stays > 0
    x, lo, hi = wl.random_box(13, 6, 2, 0.3)
    r = oracle.run(net, lo, hi)
    lin = oracle.run(_affine_only(net), lo, hi)
    aff = [k for k, L in enumerate(net.layers, start=1) if L.kind != "relu"]
    for j, k in enumerate(aff, start=1):
        np.testing.assert_allclose(r.l[k], lin.l[j], rtol=1e-12)
        np.testing.assert_allclose(r.u[k], lin.u[j], rtol=1e-12)
        assert np.all(r.l[k] > 0)


def test_first_layer_is_interval_arithmetic():
    net = wl.random_small_net(8, [12, 9, 4])
    x, lo, hi = wl.random_box(14, 12, 5, 0.1)
    r = oracle.run(net, lo, hi)
    W = net.layers[0].W.astype(np.float64)
    b = net.layers[0].b.astype(np.float64)
    c, rad = (lo.astype(np.float64) + hi) / 2, (hi.astype(np.float64) - lo) / 2
    np.testing.assert_allclose(r.l[1], c @ W.T + b - rad @ np.abs(W).T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(r.u[1], c @ W.T + b + rad @ np.abs(W).T, rtol=1e-12, atol=1e-12)


def test_depth_zero_is_interval_propagation_everywhere():
    """DeepPoly_p with p = 0: every affine layer is bounded from the stored l,u of
    the layer below -- the IBP transformer of the paper's Appendix C."""
    net = wl.random_small_net(9, [6, 7, 5, 3])
    x, lo, hi = wl.random_box(15, 6, 3, 0.2)
    r = oracle.run(net, lo, hi, max_depth=0)
    l, u = lo.astype(np.float64), hi.astype(np.float64)
    for k, L in enumerate(net.layers, start=1):
        if L.kind == "relu":
            l, u = np.maximum(l, 0), np.maximum(u, 0)
        else:
            W = L.W.astype(np.float64)
            Wp, Wn = np.maximum(W, 0), np.minimum(W, 0)
            l, u = l @ Wp.T + u @ Wn.T + L.b, u @ Wp.T + l @ Wn.T + L.b
        np.testing.assert_allclose(r.l[k], l, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(r.u[k], u, rtol=1e-12, atol=1e-12)
    full = oracle.run(net, lo, hi)
    deep = oracle.run(net, lo, hi, max_depth=100)
    for k in range(len(full.l)):
        np.testing.assert_array_equal(full.l[k], deep.l[k])
        np.testing.assert_array_equal(full.u[k], deep.u[k])


# ---------------------------------------------------------------- library reduction: conv == dense
def _conv_as_dense(L):
    """Expanded matrix of a conv layer obtained by pushing unit vectors through
    an ordinary convolution (independent of the oracle's index arithmetic)."""
    Ci, H, W = L.in_shape
    n_in = Ci * H * W
    zero_b = wl.Layer("conv", L.W, np.zeros_like(L.b), L.stride, L.pad, L.in_shape)
    M = wl.conv_forward(np.eye(n_in, dtype=np.float64), zero_b).T       # [n_out, n_in]
    Co, Ho, Wo = L.out_shape
    b = np.repeat(L.b.astype(np.float64), Ho * Wo)
    return M.astype(np.float32), b.astype(np.float32)


@pytest.mark.parametrize("convs", [[(3, 3, 1, 1), (4, 4, 2, 1)], [(2, 4, 2, 1), (3, 3, 1, 0)], [(3, 3, 2, 0)]])
def test_conv_equals_dense_expansion(convs):
    net = wl.random_small_conv(21, (2, 7, 6), convs, [5, 3])
    dense = wl.Network(n_in=net.n_in)
    for L in net.layers:
        if L.kind == "conv":
            M, b = _conv_as_dense(L)
            dense.layers.append(wl.Layer("affine", M, b))
        else:
            dense.layers.append(L)
    x, lo, hi = wl.random_box(22, net.n_in, 2, 0.05)
    lab = np.array([0, 2], np.int32)
    a = oracle.run(net, lo, hi, label=lab)
    d = oracle.run(dense, lo, hi, label=lab)
    for k in range(len(a.l)):
        np.testing.assert_allclose(a.l[k], d.l[k], rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(a.u[k], d.u[k], rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(a.margin, d.margin, rtol=1e-11, atol=1e-11)


# ---------------------------------------------------------------- brute force: neuron-level transcription
@pytest.mark.parametrize("seed,dims", [(1, [3, 4, 3, 2]), (2, [2, 5, 5, 5, 3]), (3, [4, 3, 2])])
def test_matches_neuron_level_fc(seed, dims):
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 100, dims[0], 2, 0.4)
    lab = np.array([0, dims[-1] - 1], np.int32)
    r = oracle.run(net, lo, hi, label=lab)
    for bi in range(2):
        shapes, margins, verdict = neuron_level.certify(net, lo[bi], hi[bi], label=int(lab[bi]))
        for k in range(len(shapes)):
            np.testing.assert_allclose(r.l[k][bi], [s.l for s in shapes[k]], rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(r.u[k][bi], [s.u for s in shapes[k]], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(r.margin[bi], margins, rtol=1e-12, atol=1e-12)
        assert r.verdict[bi] == verdict


def test_matches_neuron_level_conv_and_depth():
    net = wl.random_small_conv(31, (2, 5, 5), [(2, 3, 1, 1), (3, 4, 2, 1)], [4, 3])
    x, lo, hi = wl.random_box(32, net.n_in, 1, 0.1)
    for depth in (-1, 0, 1, 2, 3, 4):
        r = oracle.run(net, lo, hi, label=np.array([1], np.int32), max_depth=depth)
        shapes, margins, verdict = neuron_level.certify(net, lo[0], hi[0], label=1, max_iters=depth)
        for k in range(len(shapes)):
            np.testing.assert_allclose(r.l[k][0], [s.l for s in shapes[k]], rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(r.u[k][0], [s.u for s in shapes[k]], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(r.margin[0], margins, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- invariants
def _samples(lo, hi, n, seed, corners=True):
    rng = np.random.default_rng(seed)
    d = lo.shape[0]
    pts = lo + (hi - lo) * rng.uniform(size=(n, d))
    # points on the boundary matter most: snap a random subset of coordinates to lo/hi
    snap = rng.integers(0, 3, size=(n, d))
    pts = np.where(snap == 0, lo, np.where(snap == 1, hi, pts))
    if corners and d <= 12:
        cs = np.array(list(itertools.product(*[(lo[i], hi[i]) for i in range(d)])))
        pts = np.concatenate([pts, cs])
    return pts


@pytest.mark.parametrize("seed,dims,eps", [(1, [4, 6, 6, 3], 0.3), (2, [6, 8, 8, 8, 4], 0.15), (3, [3, 5, 2], 1.0)])
def test_soundness_by_sampling_fc(seed, dims, eps):
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 50, dims[0], 2, eps)
    last = len(net.layers)
    lab = np.array([0, 1], np.int32)
    r = oracle.run(net, lo, hi, label=lab, sym_layer=last)
    for bi in range(2):
        pts = _samples(lo[bi].astype(np.float64), hi[bi].astype(np.float64), 10000, seed)
        acts = wl.forward(net, pts)
        for k in range(len(acts)):
            assert np.all(r.l[k][bi] <= r.u[k][bi] + 1e-12)
            assert np.all(acts[k] >= r.l[k][bi] - 1e-9), f"layer {k} lower bound violated"
            assert np.all(acts[k] <= r.u[k][bi] + 1e-9), f"layer {k} upper bound violated"
        # input-level symbolic bounds of the output layer hold pointwise
        symlo = pts @ r.sym["cl"][bi].T + r.sym["kl"][bi]
        symup = pts @ r.sym["cu"][bi].T + r.sym["ku"][bi]
        assert np.all(symlo <= acts[-1] + 1e-9) and np.all(acts[-1] <= symup + 1e-9)
        # ... and their extrema over the box are the concrete bounds
        assert np.all(symlo >= r.l[last][bi] - 1e-9) and np.all(symup <= r.u[last][bi] + 1e-9)
        y = acts[-1]
        t = lab[bi]
        others = [o for o in range(dims[-1]) if o != t]
        true_m = (y[:, [t]] - y[:, others]).min(axis=0)
        assert np.all(r.margin[bi] <= true_m + 1e-9)
        if r.verdict[bi]:
            assert np.all(np.argmax(y, axis=1) == t)


def test_soundness_by_sampling_conv():
    net = wl.random_small_conv(41, (2, 6, 6), [(3, 3, 1, 1), (4, 4, 2, 1)], [6, 3])
    x, lo, hi = wl.random_box(42, net.n_in, 1, 0.08)
    r = oracle.run(net, lo, hi)
    pts = _samples(lo[0].astype(np.float64), hi[0].astype(np.float64), 4000, 5, corners=False)
    acts = wl.forward(net, pts)
    for k in range(len(acts)):
        assert np.all(acts[k] >= r.l[k][0] - 1e-9) and np.all(acts[k] <= r.u[k][0] + 1e-9)


def test_relu_symbolic_bounds_contain_relu():
    """lam*h <= relu(h) <= mu*h + nu on [l,u] for every ReLU neuron."""
    net = wl.random_small_net(4, [5, 30, 30, 4])
    x, lo, hi = wl.random_box(54, 5, 1, 0.5)
    r = oracle.run(net, lo, hi)
    for k in r.lam:
        l, u = r.l[k - 1][0], r.u[k - 1][0]
        for t in np.linspace(0, 1, 11):
            h = l + t * (u - l)
            assert np.all(r.lam[k][0] * h <= np.maximum(h, 0) + 1e-12)
            assert np.all(r.mu[k][0] * h + r.nu[k][0] >= np.maximum(h, 0) - 1e-12)
        # the kinds of neuron the test is meant to see are all present
    unstable = sum(int(np.sum((r.l[k - 1] < 0) & (r.u[k - 1] > 0))) for k in r.lam)
    assert unstable > 5


def test_batch_independence_and_permutation_invariance():
    net = wl.random_small_net(10, [5, 7, 6, 3])
    x, lo, hi = wl.random_box(60, 5, 4, 0.25)
    lab = np.array([0, 1, 2, 0], np.int32)
    r = oracle.run(net, lo, hi, label=lab)
    for bi in range(4):
        s = oracle.run(net, lo[bi:bi + 1], hi[bi:bi + 1], label=lab[bi:bi + 1])
        for k in range(len(r.l)):
            np.testing.assert_array_equal(r.l[k][bi], s.l[k][0])
            np.testing.assert_array_equal(r.u[k][bi], s.u[k][0])
        np.testing.assert_array_equal(r.margin[bi], s.margin[0])
    # permute the neurons of the first hidden layer
    perm = np.random.default_rng(0).permutation(7)
    pnet = wl.Network(n_in=5)
    L0, L2 = net.layers[0], net.layers[2]
    pnet.layers = [wl.Layer("affine", L0.W[perm], L0.b[perm]), wl.Layer("relu"),
                   wl.Layer("affine", L2.W[:, perm], L2.b)] + net.layers[3:]
    p = oracle.run(pnet, lo, hi, label=lab)
    np.testing.assert_allclose(p.l[1], r.l[1][:, perm], rtol=1e-13)
    for k in range(3, len(r.l)):
        np.testing.assert_allclose(p.l[k], r.l[k], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(p.u[k], r.u[k], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(p.margin, r.margin, rtol=1e-12, atol=1e-13)


def test_unfused_repeat_multiply_reduce_equals_one_step():
    """One traverse iteration through an affine layer is the [m,n,n]-style
    repeat / multiply / reduce of Section 3.2, i.e. an inner product (the Matmul
    rewrite of Section 4.3).  Checked on the input-level expression of layer 2
    of a ReLU-free net: coefficients must be W2 @ W1, constant W2 @ b1 + b2."""
    net = _affine_only(wl.random_small_net(12, [4, 5, 3]))
    x, lo, hi = wl.random_box(70, 4, 1, 0.1)
    r = oracle.run(net, lo, hi, sym_layer=2)
    W1, W2 = net.layers[0].W.astype(np.float64), net.layers[1].W.astype(np.float64)
    rep = W2[:, :, None] * W1[None, :, :]            # [m, n, n'] element-wise product of the repeats
    np.testing.assert_allclose(r.sym["cl"][0], rep.sum(axis=1), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(r.sym["cu"][0], rep.sum(axis=1), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(r.sym["kl"][0], W2 @ net.layers[0].b + net.layers[1].b, rtol=1e-13)


def test_rejects_malformed_input():
    net = wl.random_small_net(1, [3, 3, 2])
    lo = np.zeros((1, 3), np.float32)
    with pytest.raises(ValueError):
        oracle.run(net, lo + 1, lo)                       # lo > hi
    with pytest.raises(ValueError):
        oracle.run(net, lo, lo, label=np.array([5], np.int32))


def test_symbolic_bounds_of_every_layer_and_of_the_property_rows_hold_pointwise():
    """Input-level expressions of hidden affine / convolution layers and of the margin rows: their extrema over the box
    are the layer's l, u (the margins), and they bound the concrete values at sampled points and box corners."""
    rng = np.random.default_rng(5)
    for net in (wl.random_small_net(51, [6, 9, 8, 7, 4]), wl.random_small_conv(52, (2, 5, 5), [(3, 3, 1, 1), (4, 3, 2, 0)], [6, 3])):
        x, lo, hi = wl.random_box(53, net.n_in, 2, 0.2)
        lab = np.array([1, 2], np.int32)
        lo64, hi64 = lo.astype(np.float64), hi.astype(np.float64)
        pts = [lo64[b] + (hi64[b] - lo64[b]) * np.concatenate([rng.uniform(size=(400, net.n_in)), rng.integers(0, 2, size=(64, net.n_in))])
               for b in range(2)]
        acts = [wl.forward(net, p) for p in pts]
        nl = len(net.layers)
        for k in [i + 1 for i, L in enumerate(net.layers) if L.kind != "relu"] + [nl + 1]:
            r = oracle.run(net, lo, hi, label=lab, sym_layer=k)
            cl, kl = r.sym["cl"], r.sym["kl"]
            ext_l = kl + (np.maximum(cl, 0) * lo64[:, None, :] + np.minimum(cl, 0) * hi64[:, None, :]).sum(-1)
            if k <= nl:
                cu, ku = r.sym["cu"], r.sym["ku"]
                ext_u = ku + (np.maximum(cu, 0) * hi64[:, None, :] + np.minimum(cu, 0) * lo64[:, None, :]).sum(-1)
                np.testing.assert_allclose(ext_l, r.l[k], rtol=1e-12, atol=1e-12)
                np.testing.assert_allclose(ext_u, r.u[k], rtol=1e-12, atol=1e-12)
            else:
                np.testing.assert_allclose(ext_l, r.margin, rtol=1e-12, atol=1e-12)
            for b in range(2):
                if k <= nl:
                    val = acts[b][k]
                    assert np.all(pts[b] @ cl[b].T + kl[b] <= val + 1e-9) and np.all(val <= pts[b] @ cu[b].T + ku[b] + 1e-9)
                else:
                    out = acts[b][nl]
                    others = [o for o in range(out.shape[1]) if o != lab[b]]
                    val = out[:, [lab[b]]] - out[:, others]
                    assert np.all(pts[b] @ cl[b].T + kl[b] <= val + 1e-9)
