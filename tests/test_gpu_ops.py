"""Per-kernel parity: each hot kernel, called through the C ABI on device buffers, against the
float64 numpy definition in oracle/ops.py on the same seeded inputs.  Shapes span several tiles
and ragged tails in every dimension."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import ops                                   # noqa: E402


def _dev(a, dtype=None):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype=dtype)


def _rows(rng, M, n, ld, zero_frac=0.05):
    C = rng.normal(size=(M, n)).astype(np.float32)
    C[rng.uniform(size=C.shape) < zero_frac] = 0.0       # exact zeros take the ">=" branch
    full = np.zeros((M, ld), np.float32)
    full[:, :n] = C
    return C, full


@pytest.mark.parametrize("variant", [-1] + list(range(21)))
@pytest.mark.parametrize("M,K,N", [(1, 8, 8), (200, 100, 784), (333, 500, 500), (1000, 10, 100), (4100, 1024, 1024),
                                   (129, 36, 260), (64, 1, 5)])
def test_contract(M, K, N, variant):
    from paper_2507_20055_amd import binding as b
    b.dpc_tuning_set("contract_variant", variant)
    try:
        rng = np.random.default_rng(M * 7 + K)
        lda, ldw, ldc = (K + 31) // 32 * 32, (N + 31) // 32 * 32, (N + 31) // 32 * 32
        A, Af = _rows(rng, M, K, lda, 0.0)
        W, Wf = _rows(rng, K, N, ldw, 0.0)
        dA, dW = _dev(Af), _dev(Wf)
        dC = torch.full((M, ldc), float("nan"), device="cuda")
        b.dpc_op_contract(dA, K, dW, N, dC)
        torch.cuda.synchronize()
        got = dC.cpu().numpy()
        ref = ops.contract(A, W)
        # fp32 products accumulated in fp32 over K terms
        tol = 1e-5 * np.sqrt(K) * (np.abs(A).astype(np.float64) @ np.abs(W).astype(np.float64)) / np.sqrt(K) + 1e-6
        assert np.all(np.abs(got[:, :N] - ref) <= tol), np.abs(got[:, :N] - ref).max()
        assert np.all(got[:, N:] == 0.0)                 # padding columns are written as zeros
    finally:
        b.dpc_tuning_set("contract_variant", -1)


@pytest.mark.parametrize("nsides,B,R,n", [(2, 1, 10, 100), (2, 3, 37, 500), (1, 5, 9, 1024), (2, 2, 130, 784),
                                          (2, 2, 5, 4100), (2, 64, 3, 33)])
@pytest.mark.parametrize("shared", [False, True])
def test_relax_step(nsides, B, R, n, shared):
    from paper_2507_20055_amd import binding as b
    rng = np.random.default_rng(n + R)
    ld = (n + 31) // 32 * 32
    M = nsides * B * R
    l = rng.normal(size=(B, n)).astype(np.float32) - 0.3
    u = l + np.abs(rng.normal(size=(B, n))).astype(np.float32)
    lam = (l + u >= 0).astype(np.float32)
    uns = (l < 0) & (u > 0)
    mu = np.where(l >= 0, 1.0, np.where(u <= 0, 0.0, u / np.where(uns, u - l, 1))).astype(np.float32)
    nu = np.where(uns, -u * l / np.where(uns, u - l, 1), 0.0).astype(np.float32)
    bias = rng.normal(size=n).astype(np.float32)
    cst = rng.normal(size=M)
    if shared:
        src, srcf = _rows(rng, R, n, ld)
        C = np.tile(src, (nsides * B, 1))
        dC = torch.full((M, ld), float("nan"), device="cuda")
        dsrc = _dev(srcf)
    else:
        C, Cf = _rows(rng, M, n, ld)
        dC = _dev(Cf)
        dsrc = None
    dcst = _dev(cst)
    b.dpc_op_relax_step(dC, dcst, nsides, B, R, n, _dev(lam), _dev(mu), _dev(nu), _dev(bias), dsrc)
    torch.cuda.synchronize()
    ref_C, ref_k = ops.relax_step(C, cst, nsides, B, R, lam, mu, nu, bias)
    got = dC.cpu().numpy()
    np.testing.assert_allclose(got[:, :n], ref_C, rtol=2e-7, atol=0)          # one fp32 product each
    assert np.all(got[:, n:] == 0.0)
    mag = (np.abs(C).astype(np.float64) * (np.abs(nu)[None].repeat(nsides, 0).reshape(nsides * B, 1, n).repeat(R, 1).reshape(M, n)
                                           + np.abs(bias)[None])).sum(axis=1)
    assert np.all(np.abs(dcst.cpu().numpy() - ref_k) <= 1e-6 * mag + 1e-9)


@pytest.mark.parametrize("nsides,B,R,n", [(2, 1, 10, 784), (2, 3, 37, 1024), (1, 5, 9, 100), (2, 2, 130, 3072), (2, 64, 3, 33)])
def test_concretise(nsides, B, R, n):
    from paper_2507_20055_amd import binding as b
    rng = np.random.default_rng(n * 3 + R)
    ld = (n + 31) // 32 * 32
    M = nsides * B * R
    C, Cf = _rows(rng, M, n, ld)
    cst = rng.normal(size=M)
    lo = rng.uniform(size=(B, n)).astype(np.float32)
    hi = lo + rng.uniform(size=(B, n)).astype(np.float32) * 0.1
    out_l = torch.full((B, R), float("nan"), device="cuda")
    out_u = torch.full((B, R), float("nan"), device="cuda")
    b.dpc_op_concretise(_dev(Cf), _dev(cst), nsides, B, R, n, _dev(lo), _dev(hi), out_l, out_u if nsides == 2 else None)
    torch.cuda.synchronize()
    rl, ru = ops.concretise(C, cst, nsides, B, R, lo, hi)
    mag = (np.abs(C).astype(np.float64).reshape(nsides, B, R, n) * np.abs(hi)[None, :, None, :]).sum(-1) + np.abs(cst).reshape(nsides, B, R)
    np.testing.assert_array_less(np.abs(out_l.cpu().numpy() - rl), 2e-7 * mag[0] + 1e-7)
    if nsides == 2:
        np.testing.assert_array_less(np.abs(out_u.cpu().numpy() - ru), 2e-7 * mag[1] + 1e-7)


def test_ops_reject_bad_shapes():
    from paper_2507_20055_amd import binding as b
    A = torch.zeros((4, 32), device="cuda")
    with pytest.raises(b.DpcError):
        b.dpc_op_contract(A, 40, A, 32, A)                # K larger than lda
    with pytest.raises(b.DpcError):
        b.dpc_op_contract(A[:, 1:], 8, A, 8, A)           # misaligned / odd leading dimension


CONV_CASES = [
    # ih, iw, Co, Ci, k, stride, off, dense?   (dense rows: whole map, off = pad; patch rows: off = 0)
    (4, 4, 16, 3, 4, 2, 0, False),      # cfg3 conv2 rows through conv1
    (8, 8, 32, 16, 4, 2, 1, True),      # cfg3 FC rows through conv2
    (16, 16, 16, 3, 4, 2, 1, True),     # cfg3 FC rows through conv1
    (4, 4, 32, 3, 3, 1, 0, False),      # cfg4 conv2 rows through conv1
    (3, 3, 32, 32, 4, 2, 0, False),     # cfg4 conv3 rows through conv2
    (8, 8, 32, 3, 3, 1, 0, False),
    (4, 4, 64, 32, 3, 1, 0, False),     # cfg4 conv4 rows through conv3
    (6, 6, 32, 32, 4, 2, 0, False),
    (14, 14, 32, 3, 3, 1, 0, False),
    (8, 8, 64, 64, 4, 2, 1, True),      # cfg4 FC rows through conv4
    (16, 16, 64, 32, 3, 1, 1, True),
    (16, 16, 32, 32, 4, 2, 1, True),
    (32, 32, 32, 3, 3, 1, 1, True),
    (5, 7, 8, 12, 3, 2, 0, False),      # odd sizes, stride 2 with a 3x3 kernel (a class without taps)
    (3, 3, 6, 5, 2, 1, 0, False),       # channels not multiples of 8 / 4: generic kernel
    (20, 20, 16, 8, 3, 1, 1, True),     # more than 256 positions per class: chunked
    (6, 6, 8, 1, 3, 1, 1, True),        # few input channels: 1, 2 and 4 of them, 8 and 64 output channels
    (10, 9, 16, 2, 3, 2, 0, False),
    (7, 5, 64, 4, 4, 2, 0, False),
    (40, 24, 16, 3, 4, 2, 1, True),     # strips of output rows, stride 2
    (33, 31, 32, 4, 3, 1, 1, True),     # strips, ragged widths, 36 of 64 product columns
    (5, 7, 16, 12, 3, 2, 0, False),     # at most 16 input channels, reduction channels in groups of 16: 16 x 16 tiles
    (4, 4, 48, 16, 3, 1, 0, False),
    (28, 28, 16, 16, 3, 1, 1, True),    # several entry blocks per row
    (9, 9, 32, 9, 4, 2, 1, True),
    (20, 20, 16, 16, 4, 2, 1, True),    # stride 2 with several entry blocks per row: each block stages a band of input rows
    (18, 18, 16, 32, 3, 1, 1, True),
]


@pytest.mark.parametrize("algo", [0, 1, 2])
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_transpose(case, algo):
    from paper_2507_20055_amd import binding as b
    ih, iw, Co, Ci, k, s, off, dense = case
    if dense:
        oh = (ih - 1) * s + k - 2 * off
        ow = (iw - 1) * s + k - 2 * off
        if s == 2 and k == 4:
            oh, ow = 2 * ih, 2 * iw
    else:
        oh, ow = (ih - 1) * s + k, (iw - 1) * s + k
    rng = np.random.default_rng(ih * 100 + Co + Ci)
    for M in (1, 37, 300) + ((1500,) if (ih, Ci, algo) == (32, 3, 0) else ()):     # 1500: several panels per workgroup
        n_in, n_out = ih * iw * Co, oh * ow * Ci
        ld_in, ld_out = (n_in + 3) // 4 * 4, (n_out + 31) // 32 * 32
        rows, rows_f = _rows(rng, M, n_in, ld_in)
        K = rng.normal(size=(Co, Ci, k, k)).astype(np.float32)
        out = torch.full((M, ld_out), float("nan"), device="cuda")
        b.dpc_tuning_set("conv_algo", algo)
        try:
            b.dpc_op_conv_transpose(_dev(rows_f), ih, iw, Co, K, s, off, out, oh, ow)
        finally:
            b.dpc_tuning_set("conv_algo", 0)
        got = out.cpu().numpy()
        ref = ops.conv_transpose_rows(rows, ih, iw, K, s, off, oh, ow)
        mag = ops.conv_transpose_rows(np.abs(rows), ih, iw, np.abs(K), s, off, oh, ow)
        assert np.all(np.abs(got[:, :n_out] - ref) <= 2e-6 * mag + 1e-6), np.abs(got[:, :n_out] - ref).max()
        assert np.all(got[:, n_out:] == 0.0)


@pytest.mark.parametrize("block", range(6))
def test_conv_transpose_random_shapes(block):
    """Seeded sweep of shapes for the transposed convolution (strides 1-3, kernels 1-5, odd extents, channel counts on
    and off the MFMA kernels' multiples, patch and dense windows) against the expanded-matrix definition."""
    from paper_2507_20055_amd import binding as b
    done = 0
    for t in range(40):
        rng = np.random.default_rng(7000 + 40 * block + t)
        s = int(rng.choice([1, 1, 2, 2, 3])); k = int(rng.integers(1, 6))
        ih = int(rng.integers(1, 24)); iw = int(rng.integers(1, 24))
        Co = int(rng.choice([4, 8, 16, 24, 32, 48, 64, 6])); Ci = int(rng.choice([1, 3, 4, 5, 8, 12, 16, 24, 32, 40, 64]))
        if rng.random() < 0.5:                       # dense window: `off` rows / columns of the full extent cut off all round
            off = int(rng.integers(0, k))
            oh, ow = (ih - 1) * s + k - 2 * off, (iw - 1) * s + k - 2 * off
            if rng.random() < 0.3:
                oh += min(off, int(rng.integers(0, s))); ow += min(off, int(rng.integers(0, s)))
        else:
            off = 0
            oh, ow = (ih - 1) * s + k, (iw - 1) * s + k
        if oh < 1 or ow < 1 or oh * ow * Ci > 40000 or ih * iw * Co > 40000:
            continue
        M = int(rng.choice([1, 2, 3, 5, 17, 37, 64, 129, 300]))
        n_in, n_out = ih * iw * Co, oh * ow * Ci
        ld_in, ld_out = (n_in + 3) // 4 * 4, (n_out + 31) // 32 * 32
        rows, rows_f = _rows(rng, M, n_in, ld_in)
        K = rng.normal(size=(Co, Ci, k, k)).astype(np.float32)
        out = torch.full((M, ld_out), float("nan"), device="cuda")
        b.dpc_op_conv_transpose(_dev(rows_f), ih, iw, Co, K, s, off, out, oh, ow)
        got = out.cpu().numpy()
        ref = ops.conv_transpose_rows(rows, ih, iw, K, s, off, oh, ow)
        mag = ops.conv_transpose_rows(np.abs(rows), ih, iw, np.abs(K), s, off, oh, ow)
        case = (ih, iw, Co, Ci, k, s, off, oh, ow, M)
        assert np.all(np.abs(got[:, :n_out] - ref) <= 2e-6 * mag + 1e-6), case
        assert np.all(got[:, n_out:] == 0.0), case
        done += 1
    assert done >= 20
