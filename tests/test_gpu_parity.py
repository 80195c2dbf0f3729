"""End-to-end parity of the HIP path (through the C ABI) against the float64 CPU oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle                                            # noqa: E402
from paper_2507_20055_amd import workloads as wl         # noqa: E402
from tests.parity_util import compare_with_oracle        # noqa: E402


def _binding():
    from paper_2507_20055_amd import binding
    return binding


def _run_both(net, lo, hi, label, **kw):
    b = _binding()
    gnet = b.Network(net)
    g = gnet.certify(lo, hi, label, **kw)
    o = oracle.run(net, lo, hi, label=label, max_depth=kw.get("max_backsub_depth", -1))
    return gnet, g, o


@pytest.mark.parametrize("seed,dims,B,eps", [(1, [5, 7, 6, 3], 3, 0.3), (2, [20, 33, 65, 40, 10], 4, 0.1),
                                             (3, [7, 130, 5], 2, 0.2), (4, [3, 2], 1, 0.5), (5, [64, 257, 129, 10], 5, 0.05)])
def test_small_fc(seed, dims, B, eps):
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 10, dims[0], B, eps)
    label = np.arange(B, dtype=np.int32) % dims[-1] if dims[-1] >= 2 else None
    gnet, g, o = _run_both(net, lo, hi, label)
    compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


def test_hand_example_on_gpu():
    from tests.test_oracle_pins import read_golden, fc_net
    gd = read_golden("net_2_2_2_2.txt")
    net = fc_net(2, [(gd["W1"].reshape(2, 2), gd["b1"]), (gd["W2"].reshape(2, 2), gd["b2"]), (gd["W3"].reshape(2, 2), gd["b3"])])
    b = _binding()
    gnet = b.Network(net)
    g = gnet.certify(gd["lo"][None].astype(np.float32), gd["hi"][None].astype(np.float32), gd["label"].astype(np.int32),
                     keep_symbolic=1)
    l5, u5 = g.concrete(5)
    np.testing.assert_allclose(l5[0], gd["l5"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(u5[0], gd["u5"], rtol=1e-5, atol=1e-6)
    v, m = g.verdict()
    np.testing.assert_allclose(m[0], gd["margin"], rtol=1e-5)
    assert v[0] == 0
    cl, kl = g.symbolic(5, 0)
    cu, ku = g.symbolic(5, 1)
    np.testing.assert_allclose(cl[0].ravel(), gd["sym_lower_coeff"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(ku[0], gd["sym_upper_const"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(cu[0].ravel(), gd["sym_upper_coeff"], rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(kl[0], gd["sym_lower_const"], rtol=1e-5, atol=1e-6)
    gnet.close()


@pytest.mark.parametrize("convs,fcs,shape", [([(3, 3, 1, 1), (4, 4, 2, 1)], [6, 3], (2, 6, 6)),
                                             ([(4, 4, 2, 1), (8, 4, 2, 1)], [10, 4], (3, 12, 12)),
                                             ([(4, 3, 1, 1), (4, 4, 2, 1), (8, 3, 1, 1), (8, 4, 2, 1)], [16, 16, 5], (3, 8, 8)),
                                             ([(3, 3, 2, 0)], [4], (1, 7, 9)),
                                             # channel counts the MFMA convolution kernels take
                                             ([(8, 3, 1, 1), (8, 4, 2, 1), (16, 3, 1, 1)], [12, 4], (3, 10, 10)),
                                             ([(16, 4, 2, 1), (40, 3, 1, 0), (8, 3, 2, 1)], [9, 3], (2, 13, 11)),
                                             # one kernel for ReLU step + first layer + concretisation: 32 and 8 channels,
                                             # 4 and 1 input channels, both strides
                                             ([(32, 3, 1, 1), (16, 4, 2, 0)], [8, 3], (4, 9, 9)),
                                             ([(8, 4, 2, 1), (8, 3, 1, 1), (16, 3, 1, 1)], [5, 3], (1, 10, 10)),
                                             # more than 256 positions per row: several entry blocks, bands of input rows
                                             ([(8, 3, 1, 1), (8, 3, 1, 1)], [6, 3], (1, 17, 17))])
def test_small_conv(convs, fcs, shape):
    net = wl.random_small_conv(7, shape, convs, fcs)
    B = 3
    x, lo, hi = wl.random_box(8, net.n_in, B, 0.05)
    label = np.arange(B, dtype=np.int32) % fcs[-1]
    gnet, g, o = _run_both(net, lo, hi, label)
    compare_with_oracle(net, lo, hi, g, o, label)
    g0 = gnet.certify(lo, hi, label, fuse=0)             # every step its own kernel: same bounds
    compare_with_oracle(net, lo, hi, g0, o, label)
    gnet.close()


@pytest.mark.parametrize("seed,dims,B", [(31, [40, 64, 96, 33, 10], 3), (32, [100, 500, 500, 300, 40], 2), (33, [16, 32, 7], 5)])
def test_fused_and_unfused_paths_agree(seed, dims, B):
    """fuse=1 (ReLU step / concretisation inside the contraction's epilogue) and fuse=0 (every step its own
    kernel) are two routes through the same arithmetic; both must match the oracle."""
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 1, dims[0], B, 0.05)
    label = np.arange(B, dtype=np.int32) % dims[-1]
    b = _binding()
    gnet = b.Network(net)
    o = oracle.run(net, lo, hi, label=label)
    for fuse in (1, 0):
        g = gnet.certify(lo, hi, label, fuse=fuse)
        compare_with_oracle(net, lo, hi, g, o, label)
        p = gnet.certify(lo, hi, label, fuse=fuse, profile=1).profile()
        if fuse == 0:
            assert p["relax_launches"] >= p["contract_launches"]
    gnet.close()


def test_merged_and_separate_final_pass_agree():
    """Output-layer bounds and margins share one traversal by default; the two-pass route must give the same."""
    b = _binding()
    net = wl.random_small_net(61, [20, 48, 40, 7])
    x, lo, hi = wl.random_box(62, 20, 4, 0.08)
    label = np.array([0, 3, 6, 2], np.int32)
    gnet = b.Network(net)
    o = oracle.run(net, lo, hi, label=label)
    for merge in (1, 0):
        b.dpc_tuning_set("merge_final", merge)
        try:
            g = gnet.certify(lo, hi, label)
            compare_with_oracle(net, lo, hi, g, o, label)
        finally:
            b.dpc_tuning_set("merge_final", 1)
    gnet.close()


@pytest.mark.parametrize("kind", ["fc", "conv", "single"])
def test_symbolic_bounds_of_last_layer(kind):
    """keep_symbolic = 1: the input-level polyhedral bounds of the output neurons against the oracle's, and their
    extrema over the box against the concrete bounds (conv nets exercise the (H,W,C) -> (C,H,W) read-out)."""
    if kind == "fc":
        net = wl.random_small_net(41, [9, 40, 33, 6])
    elif kind == "conv":
        net = wl.random_small_conv(42, (2, 6, 5), [(4, 3, 1, 1), (4, 4, 2, 1)], [8, 4])
    else:
        net = wl.random_small_net(43, [7, 5])
    B = 3
    x, lo, hi = wl.random_box(44, net.n_in, B, 0.1)
    b = _binding()
    gnet = b.Network(net)
    last = len(net.layers)
    g = gnet.certify(lo, hi, None, keep_symbolic=1)
    o = oracle.run(net, lo, hi, sym_layer=last)
    l, u = g.concrete(last)
    for side, (oc, ok, bound) in enumerate(((o.sym["cl"], o.sym["kl"], l), (o.sym["cu"], o.sym["ku"], u))):
        c, k = g.symbolic(last, side)
        scale = np.abs(oc).max() + 1e-30
        assert np.all(np.abs(c - oc) <= 1e-5 * scale + 1e-4 * np.abs(oc))
        assert np.all(np.abs(k - ok) <= 1e-5 + 1e-4 * np.abs(ok))
        pos, neg = np.maximum(c.astype(np.float64), 0), np.minimum(c.astype(np.float64), 0)
        lo64, hi64 = lo.astype(np.float64)[:, None, :], hi.astype(np.float64)[:, None, :]
        ext = k + ((pos * lo64 + neg * hi64) if side == 0 else (pos * hi64 + neg * lo64)).sum(-1)
        np.testing.assert_allclose(ext, bound, rtol=1e-4, atol=1e-4)
    with pytest.raises(b.DpcError):
        gnet.certify(lo, hi, None).symbolic(last, 0)          # not kept
    gnet.close()


@pytest.mark.parametrize("kind", ["fc", "conv", "conv_first_patch", "res_fc", "res_conv"])
def test_symbolic_bounds_of_every_layer(kind):
    """keep_symbolic = 2: the input-level polyhedral bounds of every affine / convolution / Add layer and of the property
    rows against the oracle's (convolution layers' rows arrive at the input as patches and are written out dense; rows
    and columns come back in (C,H,W) order)."""
    if kind == "fc":
        net = wl.random_small_net(141, [9, 40, 33, 36, 6])
    elif kind == "conv":
        net = wl.random_small_conv(142, (2, 7, 6), [(4, 3, 1, 1), (8, 4, 2, 1), (8, 3, 1, 0)], [8, 4])
    elif kind == "conv_first_patch":
        net = wl.random_small_conv(143, (3, 8, 8), [(8, 4, 2, 1)], [5])
    elif kind == "res_fc":
        net = wl.random_small_res(144, 12, 20, 2, 5)
    else:
        net = wl.random_small_res_conv(145, (2, 6, 6), 4, 1, 3, [(8, 4, 2, 1)], [6, 3])
    B = 2
    x, lo, hi = wl.random_box(146, net.n_in, B, 0.05)
    nK = net.layers[-1].W.shape[0]
    label = np.array([0, nK - 1], np.int32)
    b = _binding()
    gnet = b.Network(net)
    nl = len(net.layers)
    g = gnet.certify(lo, hi, label, keep_symbolic=2)
    compare_with_oracle(net, lo, hi, g, oracle.run(net, lo, hi, label=label), label)

    def check(c, k, oc, ok):
        scale = np.abs(oc).max() + 1e-30
        assert c.shape == oc.shape and k.shape == ok.shape
        assert np.all(np.abs(c - oc) <= 1e-5 * scale + 1e-4 * np.abs(oc)), np.abs(c - oc).max()
        assert np.all(np.abs(k - ok) <= 1e-5 + 1e-4 * np.abs(ok))

    for k in range(1, nl + 1):
        if net.layers[k - 1].kind == "relu":
            with pytest.raises(b.DpcError):
                g.symbolic(k, 0)
            continue
        o = oracle.run(net, lo, hi, label=label, sym_layer=k)
        check(*g.symbolic(k, 0), o.sym["cl"], o.sym["kl"])
        check(*g.symbolic(k, 1), o.sym["cu"], o.sym["ku"])
    o = oracle.run(net, lo, hi, label=label, sym_layer=nl + 1)
    check(*g.margin_symbolic(), o.sym["cl"], o.sym["kl"])
    # keep_symbolic = 1 keeps the last layer and the property rows only
    g1 = gnet.certify(lo, hi, label, keep_symbolic=1)
    check(*g1.margin_symbolic(), o.sym["cl"], o.sym["kl"])
    with pytest.raises(b.DpcError):
        g1.symbolic(1, 0)
    with pytest.raises(b.DpcError):
        gnet.certify(lo, hi, label, keep_symbolic=2, max_backsub_depth=2, final_backsub_depth=-1)
    gnet.close()


@pytest.mark.parametrize("kind", ["fc", "conv"])
def test_skippoly_shapes_and_bounds(kind):
    """certifier = SkipPoly: bounds, margins and verdicts equal DeepPoly's (oracle), and the ReLU neurons' polyhedral
    bounds over the neurons two layers back equal those of the neuron-level oracle's SkipPoly, term by term."""
    from oracle import neuron_level
    if kind == "fc":
        net = wl.random_small_net(151, [5, 7, 6, 8, 3])
    else:
        net = wl.random_small_conv(152, (2, 5, 4), [(3, 3, 1, 1), (4, 3, 2, 0)], [5, 3])
    B = 2
    x, lo, hi = wl.random_box(153, net.n_in, B, 0.15)
    label = np.array([0, 2], np.int32)
    b = _binding()
    gnet = b.Network(net)
    g = gnet.certify(lo, hi, label, certifier="skippoly")
    compare_with_oracle(net, lo, hi, g, oracle.run(net, lo, hi, label=label), label)
    sizes = gnet.sizes
    for bi in range(B):
        sh, margins, verdict = neuron_level.certify(net, lo[bi], hi[bi], label=int(label[bi]), certifier="skippoly")
        np.testing.assert_allclose(g.verdict()[1][bi], margins, rtol=1e-4, atol=1e-5)
        for k, L in enumerate(net.layers, start=1):
            if L.kind != "relu":
                continue
            for side, name in ((0, "L"), (1, "U")):
                c, cst = g.relu_symbolic(k, side)
                want = np.zeros((sizes[k], sizes[k - 2]))
                wcst = np.zeros(sizes[k])
                for i, s_ in enumerate(sh[k]):
                    e = getattr(s_, name)
                    assert all(n[0] == k - 2 for n in e.terms)
                    for (_, p), v in e.terms.items():
                        want[i, p] = v
                    wcst[i] = e.const
                np.testing.assert_allclose(c[bi], want, rtol=1e-4, atol=1e-6)
                np.testing.assert_allclose(cst[bi], wcst, rtol=1e-4, atol=1e-6)
    with pytest.raises(b.DpcError):
        gnet.certify(lo, hi, label).relu_symbolic(2, 0)                      # not the SkipPoly certifier
    with pytest.raises(b.DpcError):
        gnet.certify(lo, hi, label, certifier="skippoly", max_backsub_depth=2)
    gnet.close()


@pytest.mark.parametrize("R", [1, 31, 32, 33, 64, 100])
def test_rows_per_group_around_the_fusion_threshold(R):
    """The fused epilogue needs >= 32 rows per (side, input) group; layers on both sides of that threshold, with
    tiles straddling group boundaries, must agree with the oracle."""
    net = wl.random_small_net(50 + R, [24, R, R, 5])
    B = 5
    x, lo, hi = wl.random_box(51, 24, B, 0.05)
    label = np.arange(B, dtype=np.int32) % 5
    gnet, g, o = _run_both(net, lo, hi, label)
    compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


@pytest.mark.parametrize("depth", [0, 1, 2, 3, 5])
def test_depth_limited(depth):
    net = wl.random_small_net(11, [12, 20, 18, 16, 6])
    x, lo, hi = wl.random_box(12, 12, 3, 0.1)
    label = np.array([0, 1, 2], np.int32)
    gnet, g, o = _run_both(net, lo, hi, label, max_backsub_depth=depth)
    compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


@pytest.mark.parametrize("depth,final", [(1, -2), (2, -2), (3, -2), (4, -2), (6, -2), (0, -1), (2, 5)])
def test_depth_limited_conv(depth, final):
    """Depth limits on a convolutional network whose layers take the kernels that apply the ReLU step while they
    load rows: a traversal that stops between a ReLU layer and the convolution below it must not use them."""
    net = wl.random_small_conv(17, (3, 10, 10), [(8, 3, 1, 1), (8, 4, 2, 1), (16, 3, 1, 1)], [12, 4])
    x, lo, hi = wl.random_box(18, net.n_in, 3, 0.05)
    label = np.array([0, 1, 3], np.int32)
    b = _binding()
    gnet = b.Network(net)
    kw = dict(max_backsub_depth=depth) if final == -2 else dict(max_backsub_depth=depth, final_backsub_depth=final)
    g = gnet.certify(lo, hi, label, **kw)
    o = oracle.run(net, lo, hi, label=label, max_depth=depth) if final == -2 else \
        oracle.run(net, lo, hi, label=label, max_depth=depth, max_depth_last=final)
    compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


@pytest.mark.parametrize("depth,final", [(3, -2), (2, 5), (4, -1), (2, -1)])
def test_depth_limited_call_after_a_full_one_on_the_same_network(depth, final):
    """A full-depth call leaves packed ReLU parameters behind in the network's workspace.  A later depth-limited call
    on the same network -- other boxes, a larger batch -- must not pick them up: kernels that apply a ReLU step from
    packed parameters may only run when this call has filled them.  (4, -1) and (2, -1) take the hidden layers'
    branch that does use them inside a depth limit, with parameters of this call."""
    net = wl.random_small_conv(17, (3, 10, 10), [(8, 3, 1, 1), (8, 4, 2, 1), (16, 3, 1, 1)], [12, 4])
    b = _binding()
    gnet = b.Network(net)
    x, lo, hi = wl.random_box(18, net.n_in, 2, 0.05)
    label = np.array([0, 1], np.int32)
    compare_with_oracle(net, lo, hi, gnet.certify(lo, hi, label), oracle.run(net, lo, hi, label=label), label)
    for B2, seed in ((2, 19), (5, 20)):
        x, lo, hi = wl.random_box(seed, net.n_in, B2, 0.03)
        label = (np.arange(B2) % 4).astype(np.int32)
        kw = dict(max_backsub_depth=depth) if final == -2 else dict(max_backsub_depth=depth, final_backsub_depth=final)
        g = gnet.certify(lo, hi, label, **kw)
        o = oracle.run(net, lo, hi, label=label, max_depth=depth, max_depth_last=None if final == -2 else final)
        compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


def test_edge_cases():
    b = _binding()
    net = wl.random_small_net(21, [6, 8, 4])
    gnet = b.Network(net)
    # empty batch
    r = gnet.certify(np.zeros((0, 6), np.float32), np.zeros((0, 6), np.float32), np.zeros((0,), np.int32))
    assert r.concrete(3)[0].shape == (0, 4)
    # degenerate box (eps = 0): bounds collapse to the forward pass
    x, _, _ = wl.random_box(3, 6, 2, 0.0)
    r = gnet.certify(x, x)
    acts = wl.forward(net, x.astype(np.float64))
    for k in (1, 3):
        l, u = r.concrete(k)
        np.testing.assert_allclose(l, acts[k], rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(u, acts[k], rtol=1e-5, atol=1e-6)
    # malformed inputs are rejected
    with pytest.raises(b.DpcError):
        gnet.certify(x + 1, x)
    with pytest.raises(b.DpcError):
        gnet.certify(x, x, np.array([0, 9], np.int32))
    bad = x.copy(); bad[0, 0] = np.nan
    with pytest.raises(b.DpcError):
        gnet.certify(bad, bad)
    # result reuse: no new allocation, same numbers
    r1 = gnet.certify(x, x + 0.1, np.array([0, 1], np.int32))
    l_a = r1.concrete(3)[0].copy()
    r2 = gnet.certify(x, x + 0.1, np.array([0, 1], np.int32), reuse=r1)
    assert r2 is r1
    np.testing.assert_array_equal(r1.concrete(3)[0], l_a)
    gnet.close()


def test_device_inputs_and_stream():
    import torch
    b = _binding()
    net = wl.random_small_net(22, [16, 40, 40, 5])
    x, lo, hi = wl.random_box(4, 16, 4, 0.1)
    label = np.array([0, 1, 2, 3], np.int32)
    gnet = b.Network(net)
    ref = gnet.certify(lo, hi, label)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        dlo, dhi, dlab = (torch.from_numpy(a).cuda() for a in (lo, hi, label))
    s.synchronize()
    got = gnet.certify(dlo, dhi, dlab, stream=s.cuda_stream, profile=1)
    for k in (1, 3, 5):
        np.testing.assert_array_equal(ref.concrete(k)[0], got.concrete(k)[0])
        np.testing.assert_array_equal(ref.concrete(k)[1], got.concrete(k)[1])
    np.testing.assert_array_equal(ref.verdict()[1], got.verdict()[1])
    p = got.profile()
    assert p["contract_launches"] == 1 + 2 and p["total_ms"] > 0 and p["contract_flop"] > 0   # layer 3: 1; output + margins (one pass): 2
    # malformed device-resident inputs: found by the kernel that ingests them, reported by the same call; the next
    # call starts from a clean flag
    bad_lab = torch.from_numpy(np.array([0, 1, 7, 3], np.int32)).cuda()
    with pytest.raises(b.DpcError):
        gnet.certify(dlo, dhi, bad_lab, stream=s.cuda_stream)
    with pytest.raises(b.DpcError):
        gnet.certify(dhi + 1.0, dlo, dlab, stream=s.cuda_stream)
    nan_lo = dlo.clone(); nan_lo[1, 3] = float("nan")
    with pytest.raises(b.DpcError):
        gnet.certify(nan_lo, dhi, dlab)
    again = gnet.certify(dlo, dhi, dlab, stream=s.cuda_stream)
    for k in (1, 3, 5):
        np.testing.assert_array_equal(ref.concrete(k)[0], again.concrete(k)[0])
    np.testing.assert_array_equal(ref.verdict()[0], again.verdict()[0])
    # a convolutional network takes device inputs in (C,H,W) order like host inputs
    cnet = wl.random_small_conv(7, (3, 8, 8), [(4, 3, 1, 1), (8, 4, 2, 1)], [6, 3])
    x, clo, chi = wl.random_box(8, cnet.n_in, 3, 0.05)
    clab = np.array([0, 1, 2], np.int32)
    g2 = b.Network(cnet)
    r_host = g2.certify(clo, chi, clab)
    r_dev = g2.certify(torch.from_numpy(clo).cuda(), torch.from_numpy(chi).cuda(), torch.from_numpy(clab).cuda())
    for k in (0, 1, len(cnet.layers)):
        np.testing.assert_array_equal(r_host.concrete(k)[0], r_dev.concrete(k)[0])
        np.testing.assert_array_equal(r_host.concrete(k)[1], r_dev.concrete(k)[1])
    np.testing.assert_array_equal(r_host.verdict()[1], r_dev.verdict()[1])
    g2.close()
    gnet.close()


@pytest.mark.parametrize("seed,dims,B", [(71, [24, 70, 70, 70, 6], 5),            # rows per group not a multiple of the row block
                                         (72, [50, 100, 257, 129, 10], 3),        # widths off every alignment
                                         (73, [1000, 64, 96, 4], 2),              # input wider than one chunk of the last step
                                         (74, [40, 600, 520, 5], 2),              # panels wider than 512: 32-row variant
                                         (75, [1100, 530, 40, 33, 3], 1),         # 32-row variant, two chunks at the input
                                         (76, [16, 32, 40, 7], 4)])               # a single step
@pytest.mark.parametrize("rows", [32, 64])
def test_resident_traversal_kernel(seed, dims, B, rows):
    """Traversal of a fully-connected layer's rows as one kernel (coefficients resident in LDS), forced on for
    shapes the default heuristic would leave to the per-layer kernels; against the oracle, and it must really
    have run (fewer contraction launches than the per-layer route)."""
    b = _binding()
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 1, dims[0], B, 0.05)
    label = np.arange(B, dtype=np.int32) % dims[-1]
    gnet = b.Network(net)
    o = oracle.run(net, lo, hi, label=label)
    launches = {}
    try:
        b.dpc_tuning_set("chain_rows", rows)          # row block of the variant for panels up to 512 columns
        for mode in (1, 0):
            b.dpc_tuning_set("chain", mode)
            g = gnet.certify(lo, hi, label, profile=1)
            compare_with_oracle(net, lo, hi, g, o, label)
            p = g.profile()
            launches[mode] = (p["contract_launches"] + p["chain_launches"], p["relax_launches"])
            assert p["chain_launches"] == (len(dims) - 3 if mode else 0)         # one per hidden layer after the first
    finally:
        b.dpc_tuning_set("chain", -1)
        b.dpc_tuning_set("chain_rows", 64)
    n_affine = len(dims) - 1
    assert launches[0][0] - launches[1][0] == sum(i - 2 for i in range(2, n_affine)), launches
    assert launches[0][1] - launches[1][1] == n_affine - 2, launches       # no separate first ReLU step either
    gnet.close()


def test_tuning_knobs_per_network():
    """dpc_network_tuning_set: a knob set on one network holds for that network only, whatever the process-wide value
    is, and DPC_TUNING_DEFAULT removes it.  Seen through the profile: the resident traversal kernel runs (or not)."""
    b = _binding()
    dims = [20, 33, 65, 40, 10]
    net = wl.random_small_net(91, dims)
    x, lo, hi = wl.random_box(92, dims[0], 4, 0.05)
    label = np.arange(4, dtype=np.int32) % dims[-1]
    o = oracle.run(net, lo, hi, label=label)
    forced, never, plain = b.Network(net), b.Network(net), b.Network(net)
    forced.tuning_set("chain", 1)
    never.tuning_set("chain", 0)

    def chain_launches(gnet):
        g = gnet.certify(lo, hi, label, profile=1)
        compare_with_oracle(net, lo, hi, g, o, label)
        return g.profile()["chain_launches"]

    try:
        for process_wide in (-1, 0, 1):
            b.dpc_tuning_set("chain", process_wide)
            assert chain_launches(forced) == len(dims) - 3
            assert chain_launches(never) == 0
            assert chain_launches(plain) == (len(dims) - 3 if process_wide == 1 else 0)      # by shape: too small for it
        forced.tuning_set("chain")                 # override removed: follows the process-wide value again
        b.dpc_tuning_set("chain", 0)
        assert chain_launches(forced) == 0
        with pytest.raises(b.DpcError):
            forced.tuning_set("no_such_key", 1)
    finally:
        b.dpc_tuning_set("chain", -1)
    for n in (forced, never, plain):
        n.close()


@pytest.mark.parametrize("seed,dims,B,eps", [(81, [5, 7, 6, 3], 3, 0.3), (82, [20, 33, 65, 40, 10], 4, 0.1), (83, [7, 130, 5], 2, 0.2),
                                             (84, [64, 257, 129, 70, 10], 5, 0.05), (85, [31, 40, 40, 40, 40, 2], 2, 0.1),
                                             (86, [1030, 48, 36, 4], 2, 0.02)])
def test_reusecert(seed, dims, B, eps):
    """ReuseCert (stored input-level bounds, one replacement step per layer) against the oracle's ReuseCert:
    concretised stored bounds of every affine layer, relaxations, margins, verdicts; with and without a property."""
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 10, dims[0], B, eps)
    label = np.arange(B, dtype=np.int32) % dims[-1]
    b = _binding()
    gnet = b.Network(net)
    o = oracle.run(net, lo, hi, label=label, certifier="reusecert")
    g = gnet.certify(lo, hi, label, certifier="reusecert")
    compare_with_oracle(net, lo, hi, g, o, label, relu_bounds=False)
    g2 = gnet.certify(lo, hi, None, certifier="reusecert")          # bounds only: the last layer is an ordinary step
    compare_with_oracle(net, lo, hi, g2, o, None, relu_bounds=False)
    # the certifier is a different one: on networks with at least three affine layers its output bounds differ from
    # DeepPoly's somewhere (they coincide up to two affine layers)
    d = gnet.certify(lo, hi, label)
    last = len(net.layers)
    same = np.allclose(d.concrete(last)[0], g.concrete(last)[0], rtol=1e-6, atol=1e-7)
    assert same == (len(dims) <= 3)
    gnet.close()


def test_reusecert_hand_example_and_errors():
    from tests.test_oracle_pins import read_golden, fc_net
    gd = read_golden("net_2_2_2_2.txt")
    e = read_golden("reusecert_2_2_2_2.txt")
    net = fc_net(2, [(gd["W1"].reshape(2, 2), gd["b1"]), (gd["W2"].reshape(2, 2), gd["b2"]), (gd["W3"].reshape(2, 2), gd["b3"])])
    b = _binding()
    gnet = b.Network(net)
    g = gnet.certify(gd["lo"][None].astype(np.float32), gd["hi"][None].astype(np.float32), gd["label"].astype(np.int32),
                     certifier="reusecert")
    np.testing.assert_allclose(g.concrete(3)[0][0], e["l3"], rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(g.concrete(3)[1][0], e["u3"], rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(g.concrete(5)[0][0], e["l5"], rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(g.concrete(5)[1][0], e["u5"], rtol=1e-6, atol=1e-6)
    v, m = g.verdict()
    np.testing.assert_allclose(m[0], e["margin"], rtol=1e-6)
    assert v[0] == 0
    with pytest.raises(b.DpcError):
        gnet.certify(gd["lo"][None].astype(np.float32), gd["hi"][None].astype(np.float32), None, certifier="reusecert",
                     max_backsub_depth=2)
    gnet.close()
    res = wl.random_small_res(7, 12, 16, 1, 4)
    rnet = b.Network(res)
    x, lo, hi = wl.random_box(8, res.n_in, 1, 0.05)
    with pytest.raises(b.DpcError):
        rnet.certify(lo, hi, None, certifier="reusecert")            # specified for chain networks only
    rnet.close()


@pytest.mark.parametrize("shape,convs,fcs", [((2, 6, 6), [(3, 3, 1, 1)], [6, 3]),
                                             ((3, 8, 8), [(4, 4, 2, 1), (8, 4, 2, 1)], [10, 4]),
                                             ((1, 9, 7), [(4, 3, 1, 0), (6, 3, 2, 1), (8, 2, 1, 0)], [5]),
                                             ((3, 10, 10), [(8, 3, 1, 1), (8, 4, 2, 1), (16, 3, 1, 1)], [12, 4]),
                                             ((3, 12, 12), [(8, 3, 1, 1), (16, 4, 2, 1), (16, 3, 1, 1)], [10, 4]),
                                             ((2, 13, 11), [(8, 5, 3, 2), (16, 3, 1, 1)], [7])])
@pytest.mark.parametrize("window,implicit,ck", [(1, 1, 0), (0, 1, 0), (1, 0, 0), (0, 0, 0), (1, 1, 8), (0, 1, 8), (1, 1, 100), (0, 1, 100), (1, 1, 101), (0, 1, 101)])
def test_reusecert_through_convolution_layers(shape, convs, fcs, window, implicit, ck):
    """ReuseCert on convolutional networks: the replacement step through a convolution layer is the contraction of its
    split kernel matrix with the input-level rows of the ReLU layer below, one output position at a time.
    window=1: the stored rows of the leading convolution layers cover their receptive field only (while that is smaller
    than the input -- the shapes mix both forms and every hand-over between them); window=0: rows over the whole input.
    implicit=1: layers whose channel count the implicit contraction takes (multiples of 8) read the rows in place, the
    others gather them first; implicit=0: all gather.  ck=8: the implicit contraction stages 8 channels at a time, so that layers with 16
    channels take more than one chunk per tap; ck=100 / 101: its tiles run over frame rows / over the flattened frame at
    every layer (by itself it picks one of the two per layer)."""
    net = wl.random_small_conv(171, shape, convs, fcs)
    B = 3
    x, lo, hi = wl.random_box(172, net.n_in, B, 0.04)
    label = (np.arange(B) % fcs[-1]).astype(np.int32)
    b = _binding()
    b.dpc_tuning_set("reuse_patch", window)
    b.dpc_tuning_set("reuse_window", implicit)
    b.dpc_tuning_set("reuse_window_ck", ck if ck < 100 else 0)
    b.dpc_tuning_set("reuse_window_tiles", ck - 100 if ck >= 100 else -1)
    try:
        gnet = b.Network(net)
        o = oracle.run(net, lo, hi, label=label, certifier="reusecert")
        g = gnet.certify(lo, hi, label, certifier="reusecert")
        compare_with_oracle(net, lo, hi, g, o, label, relu_bounds=False)
        compare_with_oracle(net, lo, hi, gnet.certify(lo, hi, None, certifier="reusecert"), o, None, relu_bounds=False)
        gnet.close()
    finally:
        b.dpc_tuning_set("reuse_patch", 1)
        b.dpc_tuning_set("reuse_window", 1)
        b.dpc_tuning_set("reuse_window_ck", 0)
        b.dpc_tuning_set("reuse_window_tiles", -1)


@pytest.mark.parametrize("cfg,idx", [("cfg2", [0, 17, 31]), ("cfg5", [5]), ("cfg3", [4, 29]), ("cfg4", [3])])
def test_reusecert_full_batch_gpu_sampled_oracle(cfg, idx):
    """ReuseCert at the benchmark's launch configuration (full batch); the oracle on a sample of the inputs."""
    w = wl.make_workload(cfg)
    b = _binding()
    gnet = b.Network(w.net)
    g = gnet.certify(w.lo, w.hi, w.label, certifier="reusecert")
    o = oracle.run(w.net, w.lo[idx], w.hi[idx], label=w.label[idx], certifier="reusecert")
    flipped, worst = compare_with_oracle(w.net, w.lo[idx], w.hi[idx], _Sub(g, idx), o, w.label[idx], max_flipped_inputs=1,
                                         check_samples=300, relu_bounds=False)
    print(cfg, "reusecert worst err/tol", worst)
    gnet.close()


@pytest.mark.parametrize("depth,final", [(0, -1), (1, -1), (2, 0), (0, 3)])
def test_separate_limit_for_the_last_layer(depth, final):
    """max_backsub_depth for the hidden layers, final_backsub_depth for the output layer and the margins;
    (0, -1) is CROWN-IBP."""
    net = wl.random_small_net(91, [14, 40, 36, 33, 6])
    x, lo, hi = wl.random_box(92, 14, 4, 0.1)
    label = np.array([0, 1, 2, 5], np.int32)
    b = _binding()
    gnet = b.Network(net)
    g = gnet.certify(lo, hi, label, max_backsub_depth=depth, final_backsub_depth=final)
    o = oracle.run(net, lo, hi, label=label, max_depth=depth, max_depth_last=final)
    compare_with_oracle(net, lo, hi, g, o, label)
    gnet.close()


def test_crownibp_hand_example_on_gpu():
    from tests.test_oracle_pins import read_golden, fc_net
    gd = read_golden("net_2_2_2_2.txt")
    e = read_golden("crownibp_2_2_2_2.txt")
    net = fc_net(2, [(gd["W1"].reshape(2, 2), gd["b1"]), (gd["W2"].reshape(2, 2), gd["b2"]), (gd["W3"].reshape(2, 2), gd["b3"])])
    b = _binding()
    gnet = b.Network(net)
    g = gnet.certify(gd["lo"][None].astype(np.float32), gd["hi"][None].astype(np.float32), gd["label"].astype(np.int32),
                     max_backsub_depth=0, final_backsub_depth=-1)
    for k, key in ((3, "3"), (5, "5")):
        np.testing.assert_allclose(g.concrete(k)[0][0], e["l" + key], rtol=1e-6, atol=1e-6)
        np.testing.assert_allclose(g.concrete(k)[1][0], e["u" + key], rtol=1e-6, atol=1e-6)
    v, m = g.verdict()
    np.testing.assert_allclose(m[0], e["margin"], rtol=1e-6)
    assert v[0] == 0
    gnet.close()


@pytest.mark.parametrize("kind", ["fc", "conv"])
def test_graph_replay_matches_eager(kind):
    """A reused result on a caller's stream replays the kernel sequence as one HIP graph.  Every replay
    (different boxes each time, eager library work and synchronisation between the replays, a batch change
    on the same network in the middle) must equal the eager launch sequence bit for bit."""
    import torch
    b = _binding()
    if kind == "fc":
        net, B = wl.random_small_net(31, [24, 70, 70, 70, 6]), 5
    else:
        net, B = wl.random_small_conv(32, (3, 8, 8), [(4, 3, 1, 1), (8, 4, 2, 1)], [16, 5]), 3
    n0 = net.n_in
    gnet = b.Network(net)
    s = torch.cuda.Stream()
    res = None
    last = len(net.layers)
    for it in range(6):
        x, lo, hi = wl.random_box(100 + it, n0, B, 0.02 * (1 + it % 3))
        label = np.argmax(wl.forward(net, x.astype(np.float64))[-1], axis=1).astype(np.int32)
        eager = gnet.certify(lo, hi, label, use_graph=0)
        res = gnet.certify(lo, hi, label, stream=s.cuda_stream, reuse=res)     # it = 0 eager, 1 captures, 2.. replay
        for k in range(1, last + 1):
            np.testing.assert_array_equal(eager.concrete(k)[0], res.concrete(k)[0])
            np.testing.assert_array_equal(eager.concrete(k)[1], res.concrete(k)[1])
        np.testing.assert_array_equal(eager.verdict()[1], res.verdict()[1])
        np.testing.assert_array_equal(eager.verdict()[0], res.verdict()[0])
        assert res.profile()["contract_launches"] == eager.profile()["contract_launches"]
        if it == 3:
            # a larger batch on the same network moves the shared workspace: the captured graph must not be replayed
            xb, lob, hib = wl.random_box(7, n0, 4 * B, 0.01)
            gnet.certify(lob, hib)
        torch.cuda.synchronize()
    gnet.close()


# ---- the five named configurations -------------------------------------------------------------
def test_cfg1_full():
    w = wl.make_workload("cfg1")
    gnet, g, o = _run_both(w.net, w.lo, w.hi, w.label)
    flipped, worst = compare_with_oracle(w.net, w.lo, w.hi, g, o, w.label)
    print("cfg1 worst err/tol", worst)
    gnet.close()


# Inputs on which the fp32 path decides lambda = [l + u >= 0] of some neuron the other way than the float64 oracle
# (a genuine near-tie, checked by compare_with_oracle; the input is then compared up to that layer and validated
# above it).  The workloads are seeded, so the count is a constant: {workload: number of such inputs}.
EXPECTED_LAMBDA_FLIPS = {"cfg2/0": 0, "cfg2/1": 0, "cfg2/2": 0, "cfg3": 0, "cfg4": 0, "cfg5": 0}


def _named_config(cfg, idx=None, eps_index=0, check_samples=200):
    """GPU on the full batch (the launch configuration the benchmark times) against the oracle on the inputs `idx`
    (None = all of them; inputs are independent, so the oracle on input b alone is the full-batch value)."""
    w = wl.make_workload(cfg, eps_index=eps_index)
    gnet = _binding().Network(w.net)
    g = gnet.certify(w.lo, w.hi, w.label)
    B = w.lo.shape[0]
    idx = list(range(B)) if idx is None else list(idx)
    o = oracle.run(w.net, w.lo[idx], w.hi[idx], label=w.label[idx])
    flipped, worst = compare_with_oracle(w.net, w.lo[idx], w.hi[idx], _Sub(g, idx), o, w.label[idx], max_flipped_inputs=len(idx),
                                         check_samples=check_samples)
    key = cfg + ("/%d" % eps_index if cfg == "cfg2" else "")
    print(key, "inputs compared", len(idx), "of", B, "worst err/tol", worst, "lambda flips {input: layer}", flipped,
          "verified", int(o.verdict.sum()))
    assert len(flipped) == EXPECTED_LAMBDA_FLIPS[key], f"{key}: lambda flips {flipped}"
    # verdicts of the whole batch exist and are 0/1
    v, m = g.verdict()
    assert v.shape == (B,) and set(np.unique(v)) <= {0, 1} and np.all(np.isfinite(m))
    gnet.close()


@pytest.mark.parametrize("eps_index", [0, 1, 2])
def test_cfg2_full_batch(eps_index):
    _named_config("cfg2", eps_index=eps_index)


def test_cfg2_network_at_a_perturbation_that_certifies():
    """The named settings certify nothing on untrained networks; at eps = 0.001 most inputs of the cfg2 network are
    certified and some are not: both verdicts, identical to the oracle's, on the full batch."""
    w = wl.make_workload("cfg2")
    lo = np.clip(w.x - 0.001, 0.0, 1.0).astype(np.float32)
    hi = np.clip(w.x + 0.001, 0.0, 1.0).astype(np.float32)
    gnet, g, o = _run_both(w.net, lo, hi, w.label)
    flipped, worst = compare_with_oracle(w.net, lo, hi, g, o, w.label, check_samples=100)
    v, m = g.verdict()
    assert np.array_equal(v, o.verdict) and 0 < int(v.sum()) < v.size
    print("cfg2 @ eps 0.001: verified", int(v.sum()), "of", v.size, "worst err/tol", worst)
    gnet.close()


def test_cfg3_full_batch():
    _named_config("cfg3")


def test_cfg5_full_batch():
    _named_config("cfg5", check_samples=100)


def test_cfg4_full_batch_gpu_half_batch_oracle():
    """The oracle needs about 5 s per input of this workload: the even-numbered half of the batch is compared."""
    _named_config("cfg4", idx=range(0, 16, 2), check_samples=50)


class _Sub:
    """View of a GPU result restricted to some inputs of the batch."""
    def __init__(self, res, idx):
        self.res, self.idx = res, list(idx)

    def concrete(self, k):
        l, u = self.res.concrete(k)
        return l[self.idx], u[self.idx]

    def relaxation(self, k):
        return tuple(a[self.idx] for a in self.res.relaxation(k))

    def verdict(self):
        v, m = self.res.verdict()
        return v[self.idx], m[self.idx]


@pytest.mark.parametrize("terms", [2, 3])
@pytest.mark.parametrize("seed,dims,B", [(71, [40, 64, 96, 36, 10], 3), (72, [100, 500, 500, 300, 40], 2), (73, [16, 32, 40, 7], 5),
                                         (74, [33, 130, 257, 64, 5], 4), (75, [784, 260, 132, 10], 33)])
def test_split_precision_contraction(terms, seed, dims, B):
    """Opt-in experiment: contractions on the bf16 MFMA units with operands split into 2 (bf16x3) or 3 (bf16x6) bf16
    terms, fp32 accumulation.  Same tolerance as the fp32 path; layers whose size is not a multiple of 4 stay on the
    fp32 kernel.  Both the fused-epilogue and the every-step-its-own-kernel routes."""
    net = wl.random_small_net(seed, dims)
    x, lo, hi = wl.random_box(seed + 1, dims[0], B, 0.03)
    label = np.arange(B, dtype=np.int32) % dims[-1]
    b = _binding()
    gnet = b.Network(net)
    o = oracle.run(net, lo, hi, label=label)
    b.dpc_tuning_set("contract_split", terms)
    try:
        for fuse in (1, 0):
            g = gnet.certify(lo, hi, label, fuse=fuse)
            compare_with_oracle(net, lo, hi, g, o, label)
        for wide in (0, 1):
            b.dpc_tuning_set("contract_split_wide", wide)
            compare_with_oracle(net, lo, hi, gnet.certify(lo, hi, label), o, label)
    finally:
        b.dpc_tuning_set("contract_split_wide", -1)
        b.dpc_tuning_set("contract_split", 0)
    gnet.close()


def test_split_precision_on_the_headline_workload_sample():
    b = _binding()
    w = wl.make_workload("cfg2", batch=6)
    o = oracle.run(w.net, w.lo, w.hi, label=w.label)
    gnet = b.Network(w.net)
    try:
        for terms in (2, 3):
            b.dpc_tuning_set("contract_split", terms)
            compare_with_oracle(w.net, w.lo, w.hi, gnet.certify(w.lo, w.hi, w.label), o, w.label)
    finally:
        b.dpc_tuning_set("contract_split", 0)
    gnet.close()
