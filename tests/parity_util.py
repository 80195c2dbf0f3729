"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np

from paper_2507_20055_amd import workloads as wl

RTOL, ATOL = 1e-4, 1e-5       # tolerance stated for GPU bounds against the float64 oracle


def close(a, b, scale=1.0):
    return np.abs(a - b) <= scale * (ATOL + RTOL * np.abs(b))


def compare_with_oracle(net, lo, hi, gpu, ora, label=None, max_flipped_inputs=0, check_samples=2000, seed=0,
                        relu_bounds=True, min_flip_layer=0):
    """Element-by-element comparison of every layer's l,u (and lambda/mu/nu, margins, verdicts).

    lambda = [l+u >= 0] is a discontinuous decision taken on floating-point values: when the oracle's
    l+u is within rounding of 0 the fp32 path may legitimately decide the other way, after which the
    two runs bound *different* (both valid) relaxations for that input.  Such inputs are compared up to
    the flipped layer, the flip is checked to be a genuine near-tie, and everything after it is checked
    for validity instead (l <= u, sampled concrete activations contained).  At most
    `max_flipped_inputs` inputs may take that route, and none of them at a layer below `min_flip_layer`.
    mu, nu are compared with the oracle's wherever the oracle's u - l exceeds 1e-3 (tolerance: what the
    stated tolerance on l, u allows to first order, doubled), and everywhere with the transformer's formula
    evaluated on the bounds the kernel itself was given.
    relu_bounds=False: the certifier's specification leaves l, u of ReLU neurons unset (ReuseCert), so only affine
    layers are compared with the oracle (what the library returns for ReLU layers is still checked for soundness).
    Returns ({flipped input: layer of its first flip}, worst |gpu - oracle| / tolerance)."""
    B = lo.shape[0]
    nl = len(net.layers)
    flipped = {}
    worst = 0.0
    cache = {}

    def gpu_layer(k):
        if k not in cache:
            cache[k] = gpu.concrete(k)
        return cache[k]

    for k in range(1, nl + 1):
        L = net.layers[k - 1]
        gl, gu = gpu_layer(k)
        ok_rows = np.array([b not in flipped for b in range(B)])
        for g, o, name in ((gl, ora.l[k], "l"), (gu, ora.u[k], "u")):
            if L.kind == "relu" and not relu_bounds:
                break
            bad = ~close(g, o) & ok_rows[:, None]
            if bad.any():
                b, i = np.argwhere(bad)[0]
                raise AssertionError(f"layer {k} {name}[{b},{i}]: gpu {g[b, i]!r} oracle {o[b, i]!r}")
            err = np.abs(g - o) / (ATOL + RTOL * np.abs(o))
            if ok_rows.any():
                worst = max(worst, float(err[ok_rows].max()))
        if L.kind == "relu":
            glam, gmu, gnu = gpu.relaxation(k)
            diff = (glam != ora.lam[k]) & ok_rows[:, None]
            for b, i in np.argwhere(diff):
                pl, pu = ora.l[k - 1][b, i], ora.u[k - 1][b, i]
                assert abs(pl + pu) <= 2 * (ATOL + RTOL * max(abs(pl), abs(pu))), \
                    f"lambda differs at layer {k} [{b},{i}] but l+u = {pl + pu} is not a near-tie"
                flipped.setdefault(int(b), k)
            ok_rows = np.array([b not in flipped for b in range(B)])
            # mu, nu against the oracle's.  d(mu) = (-l du + u dl) / (u-l)^2, d(nu) = (l^2 du - u^2 dl) / (u-l)^2 with
            # |dl|, |du| up to the stated tolerance on the bounds (a neuron whose stability the two sides decide
            # differently has l or u within that tolerance of 0, which the same bound covers)
            ol, ou = ora.l[k - 1], ora.u[k - 1]
            wide = ((ou - ol) > 1e-3) & ok_rows[:, None]
            tl, tu = ATOL + RTOL * np.abs(ol), ATOL + RTOL * np.abs(ou)
            w2 = np.where(wide, (ou - ol) ** 2, 1.0)
            tol_mu = 2 * (np.abs(ol) * tu + np.abs(ou) * tl) / w2 + 1e-6
            tol_nu = 2 * (ol * ol * tu + ou * ou * tl) / w2 + 1e-6 * (1 + np.abs(ora.nu[k]))
            for g, o, t, name in ((gmu, ora.mu[k], tol_mu, "mu"), (gnu, ora.nu[k], tol_nu, "nu")):
                bad = wide & (np.abs(g - o) > t)
                assert not bad.any(), f"{name} differs from the oracle at layer {k} {np.argwhere(bad)[0]}: " \
                                      f"gpu {g[tuple(np.argwhere(bad)[0])]!r} oracle {o[tuple(np.argwhere(bad)[0])]!r}"
            # the ReLU transformer's formulas (Appendix C, compute_upper) evaluated in float64 on the bounds the
            # kernel was given
            pl, pu = (a.astype(np.float64) for a in gpu_layer(k - 1))
            unstable = (pl < 0) & (pu > 0)
            d = np.where(unstable, pu - pl, 1.0)
            emu = np.where(pl >= 0, 1.0, np.where(pu <= 0, 0.0, pu / d))
            enu = np.where(unstable, -(pu * pl) / d, 0.0)
            np.testing.assert_allclose(gmu, emu, rtol=1e-5, atol=1e-30)
            np.testing.assert_allclose(gnu, enu, rtol=1e-5, atol=1e-30)
            elam = (pl + pu >= 0).astype(np.float32)
            np.testing.assert_array_equal(glam, elam)
    if label is not None:
        gv, gm = gpu.verdict()
        ok_rows = np.array([b not in flipped for b in range(B)])
        bad = ~close(gm, ora.margin) & ok_rows[:, None]
        assert not bad.any(), f"margin mismatch at {np.argwhere(bad)[0]}"
        # verdicts must be identical unless a margin sits within tolerance of 0
        near0 = (np.abs(ora.margin) <= ATOL).any(axis=1)
        assert np.array_equal(gv[ok_rows & ~near0], ora.verdict[ok_rows & ~near0])
    assert len(flipped) <= max_flipped_inputs, f"lambda flipped on inputs {flipped}"
    assert all(k >= min_flip_layer for k in flipped.values()), f"lambda flipped below layer {min_flip_layer}: {flipped}"
    # validity of everything (also the flipped inputs): l <= u and sampled activations contained
    if check_samples:
        rng = np.random.default_rng(seed)
        for b in range(B):
            pts = lo[b].astype(np.float64) + (hi[b].astype(np.float64) - lo[b]) * rng.uniform(size=(check_samples, lo.shape[1]))
            acts = wl.forward(net, pts)
            for k in range(1, nl + 1):
                gl, gu = gpu_layer(k)
                slack = ATOL + RTOL * np.maximum(np.abs(gl[b]), np.abs(gu[b]))
                assert np.all(gl[b] <= gu[b] + slack)
                assert np.all(acts[k] >= gl[b] - slack) and np.all(acts[k] <= gu[b] + slack), f"unsound at layer {k}"
    return flipped, worst
