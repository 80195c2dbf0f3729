"""Float64 definitions of the three hot operations of one traverse iteration -- TEST
INFRASTRUCTURE ONLY.  Plain numpy, written from the paper's definitions; shares nothing with the
GPU library.

Row order everywhere: m = (side*batch + b)*R + r, side 0 = lower bound rows, 1 = upper.
"""
from __future__ import annotations

import numpy as np


def contract(A, W):
    """One traverse iteration through an affine layer (Section 3.2: repeat the value tensor, repeat
    the bound tensor, multiply, reduce; Section 4.3, Matmul rewrite: that is an inner product).
    A: [M, K] coefficients over the layer's outputs, W: [K, N] -> coefficients over its inputs."""
    return np.asarray(A, np.float64) @ np.asarray(W, np.float64)


def relax_step(C, cst, nsides, batch, R, lam, mu, nu, bias):
    """replace_lower / replace_upper through a ReLU layer (Appendix C: coeff >= 0 ? coeff*L :
    coeff*U, mirrored for upper) with L = lam*p, U = mu*p + nu, followed by the constant part of
    the affine layer below (each remaining term c*p picks up c*bias_p).
    C: [nsides*batch*R, n]; cst: [nsides*batch*R]; lam/mu/nu: [batch, n]; bias: [n] or None."""
    C = np.asarray(C, np.float64)
    n = C.shape[1]
    C3 = C.reshape(nsides, batch, R, n)
    k3 = np.asarray(cst, np.float64).reshape(nsides, batch, R).copy()
    out = np.empty_like(C3)
    lam, mu, nu = (np.asarray(a, np.float64)[:, None, :] for a in (lam, mu, nu))
    for side in range(nsides):
        X = C3[side]
        pos = X >= 0.0
        if side == 0:
            out[side] = np.where(pos, X * lam, X * mu)
            k3[side] += np.where(pos, 0.0, X * nu).sum(axis=-1)
        else:
            out[side] = np.where(pos, X * mu, X * lam)
            k3[side] += np.where(pos, X * nu, 0.0).sum(axis=-1)
        if bias is not None:
            k3[side] += (out[side] * np.asarray(bias, np.float64)[None, None, :]).sum(axis=-1)
    return out.reshape(-1, n), k3.reshape(-1)


def concretise(C, cst, nsides, batch, R, lo, hi):
    """simplify_lower / simplify_upper (Appendix C): coeff >= 0 ? coeff*l : coeff*u, mirrored.
    Returns (lower [batch, R], upper [batch, R] or None)."""
    C = np.asarray(C, np.float64)
    n = C.shape[1]
    C3 = C.reshape(nsides, batch, R, n)
    k3 = np.asarray(cst, np.float64).reshape(nsides, batch, R)
    lo, hi = np.asarray(lo, np.float64)[:, None, :], np.asarray(hi, np.float64)[:, None, :]
    res = []
    for side in range(nsides):
        X = C3[side]
        pos = X >= 0.0
        if side == 0:
            res.append(k3[side] + np.where(pos, X * lo, X * hi).sum(axis=-1))
        else:
            res.append(k3[side] + np.where(pos, X * hi, X * lo).sum(axis=-1))
    return res[0], (res[1] if nsides == 2 else None)


def conv_transpose_rows(rows, ih, iw, K, stride, off, oh, ow):
    """One traverse iteration through a convolution layer: coefficient rows over the layer's outputs
    times its expanded weight matrix (Section 3.3: the block of a convolutional layer "represents an
    expanded convolution kernel"; Appendix B.3: the product reduces to a transposed convolution).
    Written as the definition: the expanded matrix is built entry by entry and multiplied.
    rows: [M, ih*iw*Co] channel-last; K: [Co, Ci, kh, kw]; output window of oh x ow positions whose
    top-left corner is `off` inside the full transposed-convolution extent.  Returns [M, oh*ow*Ci]."""
    K = np.asarray(K, np.float64)
    Co, Ci, kh, kw = K.shape
    E = np.zeros((ih * iw * Co, oh * ow * Ci))
    for py in range(ih):
        for px in range(iw):
            for ky in range(kh):
                for kx in range(kw):
                    y, x = py * stride + ky - off, px * stride + kx - off
                    if 0 <= y < oh and 0 <= x < ow:
                        r0, c0 = (py * iw + px) * Co, (y * ow + x) * Ci
                        E[r0:r0 + Co, c0:c0 + Ci] += K[:, :, ky, kx]
    return np.asarray(rows, np.float64) @ E
