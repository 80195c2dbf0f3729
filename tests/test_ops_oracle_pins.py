"""Pins for oracle/ops.py (the numpy definitions of the three hot operations): composing them
layer by layer must reproduce the independently written and pinned C oracle."""
import numpy as np

import oracle
from oracle import ops
from paper_2507_20055_amd import workloads as wl


def test_ops_compose_to_the_c_oracle():
    net = wl.random_small_net(3, [6, 9, 8, 7, 4])
    x, lo, hi = wl.random_box(5, 6, 3, 0.3)
    ref = oracle.run(net, lo, hi, sym_layer=7)
    B = 3
    aff = [(k, L) for k, L in enumerate(net.layers, start=1) if L.kind == "affine"]
    # bounds of the last layer (index 7): start from its weight rows, walk down
    k, L = aff[-1]
    R = L.W.shape[0]
    C = np.tile(L.W.astype(np.float64), (2 * B, 1))
    cst = np.tile(L.b.astype(np.float64), 2 * B)
    for (kj, Lj) in reversed(aff[:-1]):
        relu_idx = kj + 1
        C, cst = ops.relax_step(C, cst, 2, B, R, ref.lam[relu_idx], ref.mu[relu_idx], ref.nu[relu_idx], Lj.b)
        C = ops.contract(C, Lj.W)
    l, u = ops.concretise(C, cst, 2, B, R, lo, hi)
    np.testing.assert_allclose(l, ref.l[7], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(u, ref.u[7], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(C.reshape(2, B, R, 6)[0], ref.sym["cl"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(C.reshape(2, B, R, 6)[1], ref.sym["cu"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(cst.reshape(2, B, R)[1], ref.sym["ku"], rtol=1e-12, atol=1e-12)


def test_relax_step_hand_values():
    # one input, one row per side, three neurons: stable active, stable inactive, unstable
    lam = np.array([[1.0, 0.0, 0.0]]); mu = np.array([[1.0, 0.0, 0.25]]); nu = np.array([[0.0, 0.0, 0.75]])
    C = np.array([[2.0, -3.0, -4.0], [2.0, -3.0, 4.0]])
    out, k = ops.relax_step(C, np.array([1.0, 1.0]), 2, 1, 1, lam, mu, nu, np.array([10.0, 20.0, 30.0]))
    # lower row: +2 -> L (lam=1): 2 ; -3 -> U (mu=0): 0 ; -4 -> U: -1, const -4*0.75 = -3
    np.testing.assert_allclose(out[0], [2.0, 0.0, -1.0])
    np.testing.assert_allclose(k[0], 1.0 - 3.0 + 2.0 * 10 + 0.0 * 20 - 1.0 * 30)
    # upper row: +2 -> U: 2 ; -3 -> L (lam=0): 0 ; +4 -> U: 1, const +4*0.75 = 3
    np.testing.assert_allclose(out[1], [2.0, 0.0, 1.0])
    np.testing.assert_allclose(k[1], 1.0 + 3.0 + 2.0 * 10 + 1.0 * 30)


def test_concretise_hand_values():
    C = np.array([[1.0, -2.0], [1.0, -2.0]])
    l, u = ops.concretise(C, np.array([0.5, 0.5]), 2, 1, 1, np.array([[-1.0, 3.0]]), np.array([[2.0, 5.0]]))
    np.testing.assert_allclose(l, [[0.5 + 1 * -1 - 2 * 5]])
    np.testing.assert_allclose(u, [[0.5 + 1 * 2 - 2 * 3]])


def test_conv_transpose_rows_is_the_expanded_matrix():
    """ops.conv_transpose_rows applied to the identity gives the expanded convolution matrix; the
    same matrix obtained by pushing unit vectors through an ordinary convolution (independent code,
    (C,H,W) order) must agree after the channel-last permutation."""
    import pytest
    for (Ci, H, W, Co, k, s, p) in [(2, 5, 6, 3, 3, 1, 1), (3, 8, 8, 4, 4, 2, 1), (1, 7, 5, 2, 3, 2, 0)]:
        rng = np.random.default_rng(Ci + H)
        K = rng.normal(size=(Co, Ci, k, k)).astype(np.float32)
        L = wl.Layer("conv", K, np.zeros(Co, np.float32), stride=s, pad=p, in_shape=(Ci, H, W))
        _, Ho, Wo = L.out_shape
        n_in, n_out = Ci * H * W, Co * Ho * Wo
        D = wl.conv_forward(np.eye(n_in), L).T                         # [n_out, n_in], both (C,H,W)
        E = ops.conv_transpose_rows(np.eye(n_out), Ho, Wo, K, s, p, H, W)   # [n_out, n_in], both (H,W,C)
        perm_out = np.arange(n_out).reshape(Co, Ho, Wo).transpose(1, 2, 0).ravel()   # hwc position -> chw index
        perm_in = np.arange(n_in).reshape(Ci, H, W).transpose(1, 2, 0).ravel()
        np.testing.assert_allclose(E, D[np.ix_(perm_out, perm_in)], rtol=0, atol=1e-12)
