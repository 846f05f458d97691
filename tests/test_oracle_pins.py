"""Pins for the CPU oracle: every routine in oracle/xconv_oracle.c is checked
against something other than itself -- published generator outputs, library
routines (numpy float16, torch bfloat16, torch conv2d and its autograd), brute
force written independently here, closed forms and the statistical statements
of the paper (Sec. 3 Eq. (2), (3), (5), (6); Proposition 1; Algorithm 1).
CPU only.
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import xconv_oracle as xo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_numbers(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(t) for t in line.split()])
    return rows


# --------------------------------------------------------------------------
# generator
# --------------------------------------------------------------------------
def test_splitmix64_published_vector():
    want = [row[0] for row in _read_numbers("splitmix64_seed1234567.txt")]
    assert xo.splitmix64_stream(1234567, len(want)) == want


def test_stream_word_is_the_counter_form_of_splitmix64():
    # word ctr of seed's stream == (ctr+1)-th output of SplitMix64 started at
    # the first output of SplitMix64(seed)
    for seed in (0, 1, 3001, 2**63 + 12345):
        key = xo.splitmix64_stream(seed, 1)[0]
        stream = xo.splitmix64_stream(key, 6)
        assert [xo.stream_word(seed, c) for c in range(6)] == stream


def test_rademacher_entries_and_balance():
    Z = xo.probe_matrix(xo.RADEMACHER, 3001, 256, 64)
    assert set(np.unique(Z)) == {-1.0, 1.0}
    n = Z.size
    assert abs(Z.sum()) < 4.0 * np.sqrt(n)
    assert np.all(np.abs(Z.sum(axis=0)) < 4.5 * np.sqrt(Z.shape[0]))
    assert np.all(np.abs(Z.sum(axis=1)) < 4.5 * np.sqrt(Z.shape[1]))
    # entry number i = c*r + j is bit i mod 64 of stream word i div 64, a set bit meaning -1
    for (c, j) in [(0, 0), (3, 5), (255, 63)]:
        i = c * 64 + j
        w = xo.stream_word(3001, i // 64)
        assert Z[c, j] == (-1.0 if ((w >> (i % 64)) & 1) else 1.0)
    # a probe count that is not a multiple of 64: words run across the rows
    Z2 = xo.probe_matrix(xo.RADEMACHER, 77, 9, 24)
    for i in (0, 23, 24, 63, 64, 100, 215):
        w = xo.stream_word(77, i // 64)
        assert Z2.reshape(-1)[i] == (-1.0 if ((w >> (i % 64)) & 1) else 1.0)
    # no correlation between neighbouring entries, which now share a word: the lag-1 product averages to 0
    flat = Z.reshape(-1).astype(np.float64)
    assert abs(np.mean(flat[:-1] * flat[1:])) < 4.0 / np.sqrt(flat.size)


def test_gaussian_moments():
    Z = xo.probe_matrix(xo.GAUSSIAN, 3002, 512, 256).astype(np.float64)
    n = Z.size
    assert abs(Z.mean()) < 4.0 / np.sqrt(n)
    assert abs(Z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    kurt = np.mean(Z ** 4)
    assert abs(kurt - 3.0) < 4.0 * np.sqrt(96.0 / n)
    assert abs(np.mean(Z ** 3)) < 4.0 * np.sqrt(15.0 / n)
    # Box-Muller from the two stream words, redone here in numpy double
    for (c, j) in [(0, 0), (17, 3), (511, 255)]:
        idx = c * 256 + j
        u1 = ((xo.stream_word(3002, 2 * idx) >> 11) + 1) * 2.0 ** -53
        u2 = (xo.stream_word(3002, 2 * idx + 1) >> 11) * 2.0 ** -53
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        assert abs(Z[c, j] - g) <= 2e-7 * max(1.0, abs(g))


@pytest.mark.parametrize("dist", [xo.RADEMACHER, xo.GAUSSIAN])
def test_probe_second_moment_is_identity(dist):
    # E[z z^T] = I (Eq. (3)): Z Z^T / r -> I as r grows, off-diagonals ~ 1/sqrt(r)
    C = 16
    for r, tol in ((1024, 0.2), (16384, 0.05)):
        Z = xo.probe_matrix(dist, 77, C, r).astype(np.float64)
        G = Z @ Z.T / r
        assert np.max(np.abs(G - np.eye(C))) < tol


def test_probe_matrix_seed_behaviour():
    a = xo.probe_matrix(xo.GAUSSIAN, 5, 32, 8)
    b = xo.probe_matrix(xo.GAUSSIAN, 5, 32, 8)
    c = xo.probe_matrix(xo.GAUSSIAN, 6, 32, 8)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, c)
    assert abs(np.corrcoef(a.ravel(), c.ravel())[0, 1]) < 0.3
    with pytest.raises(ValueError):
        xo.probe_matrix(9, 5, 4, 4)


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def test_round_storage_matches_library_conversions():
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(2000) * 10.0 ** rng.integers(-9, 5, 2000),
        np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65504.0, 65519.9, 65520.0,
                  6e-8, 2.98e-8, 2.99e-8, 5.96e-8, 1e-40, 3.3895e38, 3.4e38, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]),
    ])
    for v in vals:
        f32 = np.float32(v)
        # the oracle rounds double sums directly; use doubles that are floats so
        # the library conversion (float -> 16 bit) rounds the same number
        v = float(f32)
        got16 = xo.round_storage(v, xo.F16)
        with np.errstate(over="ignore"):
            want16 = float(np.float32(v).astype(np.float16))
        assert got16 == want16 or (np.isnan(got16) and np.isnan(want16)), (v, got16, want16)
        gotb = xo.round_storage(v, xo.BF16)
        wantb = float(torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).to(torch.float32))
        assert gotb == wantb, (v, gotb, wantb)
        assert xo.round_storage(v, xo.F32) == v


# --------------------------------------------------------------------------
# exact gradient, Eq. (2)/(5)
# --------------------------------------------------------------------------
def _brute_conv(X, Wt, stride, pad):
    """Textbook direct convolution (gather form), written here independently."""
    B, C_in, H, W = X.shape
    C_out, _, kH, kW = Wt.shape
    Ho = (H + 2 * pad[0] - kH) // stride[0] + 1
    Wo = (W + 2 * pad[1] - kW) // stride[1] + 1
    Xp = np.zeros((B, C_in, H + 2 * pad[0], W + 2 * pad[1]))
    Xp[:, :, pad[0]:pad[0] + H, pad[1]:pad[1] + W] = X
    Y = np.zeros((B, C_out, Ho, Wo))
    for b, m, oy, ox in itertools.product(range(B), range(C_out), range(Ho), range(Wo)):
        patch = Xp[b, :, oy * stride[0]:oy * stride[0] + kH, ox * stride[1]:ox * stride[1] + kW]
        Y[b, m, oy, ox] = np.sum(patch * Wt[m])
    return Y


TINY = [
    # B, C_in, C_out, H, W, kH, kW, stride, pad
    (2, 3, 2, 6, 5, 3, 3, (1, 1), (1, 1)),
    (2, 2, 3, 6, 6, 3, 3, (2, 2), (1, 1)),
    (1, 3, 3, 5, 6, 1, 1, (1, 1), (0, 0)),
    (2, 2, 2, 6, 6, 3, 3, (1, 1), (0, 0)),
    (1, 2, 2, 7, 6, 3, 2, (2, 1), (1, 0)),
    (2, 1, 2, 5, 5, 5, 5, (1, 1), (2, 2)),
]


@pytest.mark.parametrize("case", TINY)
def test_conv_fwd_against_brute_force_and_torch(case):
    B, C_in, C_out, H, W, kH, kW, stride, pad = case
    rng = np.random.default_rng(1)
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    Wt = rng.standard_normal((C_out, C_in, kH, kW))
    Y = xo.conv_fwd(X, Wt, stride, pad)
    assert np.allclose(Y, _brute_conv(X.astype(np.float64), Wt, stride, pad), atol=1e-12)
    Yt = F.conv2d(torch.from_numpy(X).double(), torch.from_numpy(Wt), stride=stride, padding=pad).numpy()
    assert np.allclose(Y, Yt, atol=1e-12)


@pytest.mark.parametrize("case", TINY)
def test_dw_exact_unit_weight_brute_force(case):
    # dW[m,n,ky,kx] = <dY, conv(X, E_{m,n,ky,kx})> for every unit weight
    B, C_in, C_out, H, W, kH, kW, stride, pad = case
    rng = np.random.default_rng(2)
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    Ho, Wo = xo.out_extent(H, kH, stride[0], pad[0]), xo.out_extent(W, kW, stride[1], pad[1])
    dY = rng.standard_normal((B, C_out, Ho, Wo)).astype(np.float32)
    dW = xo.dw_exact(dY, X, kH, kW, stride, pad)
    for m, n, ky, kx in itertools.product(range(C_out), range(C_in), range(kH), range(kW)):
        E = np.zeros((C_out, C_in, kH, kW))
        E[m, n, ky, kx] = 1.0
        want = np.sum(dY.astype(np.float64) * _brute_conv(X.astype(np.float64), E, stride, pad))
        assert abs(dW[m, n, ky, kx] - want) < 1e-10


@pytest.mark.parametrize("case", TINY + [(3, 5, 4, 9, 11, 3, 3, (2, 2), (1, 1)), (2, 4, 6, 12, 12, 3, 3, (1, 1), (1, 1))])
def test_dw_exact_against_torch_autograd(case):
    B, C_in, C_out, H, W, kH, kW, stride, pad = case
    rng = np.random.default_rng(3)
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    Ho, Wo = xo.out_extent(H, kH, stride[0], pad[0]), xo.out_extent(W, kW, stride[1], pad[1])
    dY = rng.standard_normal((B, C_out, Ho, Wo)).astype(np.float32)
    w = torch.zeros((C_out, C_in, kH, kW), dtype=torch.float64, requires_grad=True)
    y = F.conv2d(torch.from_numpy(X).double(), w, stride=stride, padding=pad)
    y.backward(torch.from_numpy(dY).double())
    assert np.allclose(xo.dw_exact(dY, X, kH, kW, stride, pad), w.grad.numpy(), atol=1e-10)


def test_dw_exact_adjoint_identity():
    rng = np.random.default_rng(4)
    B, C_in, C_out, H, W, k = 3, 4, 5, 10, 9, 3
    for stride, pad in (((1, 1), (1, 1)), ((2, 2), (1, 1)), ((1, 2), (0, 1))):
        X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
        Wt = rng.standard_normal((C_out, C_in, k, k))
        Y = xo.conv_fwd(X, Wt, stride, pad)
        dY = rng.standard_normal(Y.shape).astype(np.float32)
        lhs = np.sum(dY.astype(np.float64) * Y)
        rhs = np.sum(xo.dw_exact(dY, X, k, k, stride, pad) * Wt)
        assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))


# ---------------------------------------------------------------------------
# input gradient (Sec. 2: backpropagation through the layer stays exact; only dW is estimated)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", TINY + [(3, 5, 4, 9, 11, 3, 3, (2, 2), (1, 1)), (2, 4, 6, 12, 12, 3, 3, (1, 1), (1, 1)),
                                         (2, 3, 4, 10, 9, 3, 3, (3, 2), (0, 1))])
def test_dx_against_torch_autograd(case):
    B, C_in, C_out, H, W, kH, kW, stride, pad = case
    rng = np.random.default_rng(31)
    Ho, Wo = xo.out_extent(H, kH, stride[0], pad[0]), xo.out_extent(W, kW, stride[1], pad[1])
    dY = rng.standard_normal((B, C_out, Ho, Wo)).astype(np.float32)
    Wt = rng.standard_normal((C_out, C_in, kH, kW))
    x = torch.zeros((B, C_in, H, W), dtype=torch.float64, requires_grad=True)
    y = F.conv2d(x, torch.from_numpy(Wt), stride=stride, padding=pad)
    y.backward(torch.from_numpy(dY).double())
    assert np.allclose(xo.dx(dY, Wt, H, W, stride, pad), x.grad.numpy(), atol=1e-11)


def test_dx_adjoint_identity_with_the_forward_convolution():
    # <dX, V> = <dY, conv(V, W)> for any V: the transposed convolution is the adjoint of the forward one, which is
    # written as a scatter over the inputs and pinned by brute force above
    rng = np.random.default_rng(32)
    B, C_in, C_out, H, W, k = 3, 4, 5, 10, 9, 3
    for stride, pad in (((1, 1), (1, 1)), ((2, 2), (1, 1)), ((1, 2), (0, 1)), ((3, 3), (2, 2))):
        V = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
        Wt = rng.standard_normal((C_out, C_in, k, k))
        Y = xo.conv_fwd(V, Wt, stride, pad)
        dY = rng.standard_normal(Y.shape).astype(np.float32)
        lhs = np.sum(xo.dx(dY, Wt, H, W, stride, pad) * V.astype(np.float64))
        rhs = np.sum(dY.astype(np.float64) * Y)
        assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(rhs))


def test_dx_special_cases():
    rng = np.random.default_rng(33)
    # k = 1, stride 1: dX[b,n,p] = sum_m W[m,n] dY[b,m,p]
    B, C_in, C_out, H, W = 2, 3, 4, 5, 6
    dY = rng.standard_normal((B, C_out, H, W)).astype(np.float32)
    Wt = rng.standard_normal((C_out, C_in, 1, 1))
    want = np.einsum("mn,bmyx->bnyx", Wt[:, :, 0, 0], dY.astype(np.float64))
    assert np.allclose(xo.dx(dY, Wt, H, W), want, atol=1e-12)
    # a single non-zero residual at (oy, ox) with stride 2: dX is the kernel stamped at (oy*2 - p, ox*2 - p)
    dY = np.zeros((1, 1, 4, 4), dtype=np.float32)
    dY[0, 0, 1, 2] = 2.0
    Wt = rng.standard_normal((1, 2, 3, 3))
    got = xo.dx(dY, Wt, 8, 8, (2, 2), (1, 1))
    want = np.zeros((1, 2, 8, 8))
    want[0, :, 1:4, 3:6] = 2.0 * Wt[0]
    assert np.allclose(got, want, atol=1e-12)


def test_dw_exact_special_cases():
    rng = np.random.default_rng(5)
    # k = 1: the gradient is the plain matrix product  sum_{b,p} dY[b,m,p] X[b,n,p]
    B, C_in, C_out, H, W = 3, 5, 4, 6, 7
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    dY = rng.standard_normal((B, C_out, H, W)).astype(np.float32)
    want = np.einsum("bmp,bnp->mn", dY.reshape(B, C_out, -1).astype(np.float64), X.reshape(B, C_in, -1).astype(np.float64))
    assert np.allclose(xo.dw_exact(dY, X, 1, 1)[:, :, 0, 0], want, atol=1e-10)
    # a single bright input pixel: dW is a flipped, shifted copy of dY around it
    X = np.zeros((1, 1, 7, 7), dtype=np.float32)
    X[0, 0, 3, 4] = 2.0
    dY = rng.standard_normal((1, 1, 7, 7)).astype(np.float32)
    dW = xo.dw_exact(dY, X, 3, 3, (1, 1), (1, 1))
    for ky, kx in itertools.product(range(3), range(3)):
        # input pixel (3,4) is seen by output pixel (3 - ky + 1, 4 - kx + 1)
        assert abs(dW[0, 0, ky, kx] - 2.0 * dY[0, 0, 3 - ky + 1, 4 - kx + 1]) < 1e-12


# --------------------------------------------------------------------------
# probe, correlation, expansion: Algorithm 1 / Eq. (6)
# --------------------------------------------------------------------------
def test_probe_fwd_is_a_channel_contraction():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((3, 7, 5, 6)).astype(np.float32)
    Z = rng.standard_normal((7, 4)).astype(np.float32)
    Xt = xo.probe_fwd(X, Z, xo.F32)
    want = np.einsum("nj,bnyx->bjyx", Z.astype(np.float64), X.astype(np.float64))
    assert Xt.shape == (3, 4, 5, 6)
    assert np.array_equal(Xt, want.astype(np.float32))
    # 16-bit storage: one rounding of the exact sum
    Xh = xo.probe_fwd(X, Z, xo.F16)
    assert np.array_equal(Xh, want.astype(np.float32).astype(np.float16).astype(np.float32)) or \
        np.max(np.abs(Xh - want)) <= 2.0 ** -11 * np.max(np.abs(want)) * 1.0001
    Xb = xo.probe_fwd(X, Z, xo.BF16)
    assert np.max(np.abs(Xb - want) / np.maximum(np.abs(want), 1e-30)) <= 2.0 ** -8
    assert np.array_equal(Xb.view(np.uint32) & 0xFFFF, np.zeros(Xb.shape, dtype=np.uint32))


CLOSED_FORM_CASES = [
    # B, C_in, C_out, H, W, k, stride, pad, r, dist
    (3, 8, 5, 9, 10, 3, 1, 1, 4, xo.GAUSSIAN),
    (2, 6, 7, 11, 9, 3, 2, 1, 3, xo.RADEMACHER),
    (2, 5, 3, 8, 8, 1, 1, 0, 2, xo.GAUSSIAN),
    (2, 4, 4, 9, 9, 5, 1, 2, 6, xo.RADEMACHER),
    (2, 4, 3, 10, 7, 3, 1, 0, 5, xo.GAUSSIAN),
]


@pytest.mark.parametrize("case", CLOSED_FORM_CASES)
def test_estimate_closed_form(case):
    # For a fixed Z the estimator is linear in X, so
    #   dW_est[m,n,:,:] = sum_n' (Z Z^T / r)[n,n'] dW_exact[m,n',:,:]
    # (Eq. (6) with the probes restricted to channels).  The right-hand side is
    # built from the torch-pinned exact gradient and numpy alone.
    B, C_in, C_out, H, W, k, st, p, r, dist = case
    rng = np.random.default_rng(7)
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    Ho, Wo = xo.out_extent(H, k, st, p), xo.out_extent(W, k, st, p)
    dY = rng.standard_normal((B, C_out, Ho, Wo)).astype(np.float32)
    Z = xo.probe_matrix(dist, 11, C_in, r)
    est = xo.dw_estimate(dY, X, Z, k, k, (st, st), (p, p), xo.F32)
    w = torch.zeros((C_out, C_in, k, k), dtype=torch.float64, requires_grad=True)
    F.conv2d(torch.from_numpy(X).double(), w, stride=st, padding=p).backward(torch.from_numpy(dY).double())
    G = Z.astype(np.float64) @ Z.astype(np.float64).T / r
    want = np.einsum("nq,mqyx->mnyx", G, w.grad.numpy())
    # fp32 storage of the probed activations is the only rounding
    assert np.max(np.abs(est - want)) <= 2e-6 * np.max(np.abs(want))


def test_estimate_steps_compose():
    rng = np.random.default_rng(8)
    B, C_in, C_out, H, W, k, r = 2, 6, 4, 8, 8, 3, 3
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    dY = rng.standard_normal((B, C_out, H, W)).astype(np.float32)
    Z = xo.probe_matrix(xo.GAUSSIAN, 1, C_in, r)
    Xt = xo.probe_fwd(X, Z, xo.F32)
    G = xo.correlate(dY, Xt, k, k, (1, 1), (1, 1))
    # correlation pinned by torch: it is the exact gradient w.r.t. an r-channel input
    w = torch.zeros((C_out, r, k, k), dtype=torch.float64, requires_grad=True)
    F.conv2d(torch.from_numpy(Xt).double(), w, padding=1).backward(torch.from_numpy(dY).double())
    assert np.allclose(G, w.grad.numpy(), atol=1e-10)
    # expansion pinned by einsum
    want = np.einsum("nj,mjyx->mnyx", Z.astype(np.float64), G) / r
    assert np.allclose(xo.expand(G, Z), want, atol=1e-12)
    assert np.allclose(xo.dw_from_xt(dY, Xt, Z, k, k, (1, 1), (1, 1)), want, atol=1e-12)
    assert np.allclose(xo.dw_estimate(dY, X, Z, k, k, (1, 1), (1, 1), xo.F32), want, atol=1e-12)
    # sampled entries are the same numbers
    idx = np.array([[0, 0, 0, 0], [3, 5, 2, 1], [1, 2, 1, 1], [2, 4, 0, 2]], dtype=np.int32)
    got = xo.dw_from_xt_at(dY, Xt, Z, idx, k, k, (1, 1), (1, 1))
    assert np.allclose(got, [want[tuple(i)] for i in idx], atol=1e-12)
    ex = xo.dw_exact(dY, X, k, k, (1, 1), (1, 1))
    got = xo.dw_exact_at(dY, X, idx, k, k, (1, 1), (1, 1))
    assert np.allclose(got, [ex[tuple(i)] for i in idx], atol=1e-12)


def _sylvester_hadamard(n):
    Hm = np.array([[1.0]])
    while Hm.shape[0] < n:
        Hm = np.block([[Hm, Hm], [Hm, -Hm]])
    return Hm


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1)])
def test_full_rank_orthogonal_probe_recovers_exact_gradient(stride, pad):
    # r = C_in with Z Z^T = r I: the estimate is the exact gradient (Sec. 2:
    # raising the probing rank recovers the exact gradient).
    rng = np.random.default_rng(9)
    B, C_in, C_out, H, W, k = 2, 8, 5, 10, 10, 3
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    Ho = xo.out_extent(H, k, stride, pad)
    dY = rng.standard_normal((B, C_out, Ho, Ho)).astype(np.float32)
    exact = xo.dw_exact(dY, X, k, k, (stride, stride), (pad, pad))
    for Z in (_sylvester_hadamard(C_in), np.sqrt(C_in) * np.eye(C_in)):
        Z = Z.astype(np.float32)
        est = xo.dw_estimate(dY, X, Z, k, k, (stride, stride), (pad, pad), xo.F32)
        assert np.max(np.abs(est - exact)) <= 3e-6 * np.max(np.abs(exact))
    # a random full-rank Rademacher probe is NOT exact
    Zr = xo.probe_matrix(xo.RADEMACHER, 1, C_in, C_in)
    est = xo.dw_estimate(dY, X, Zr, k, k, (stride, stride), (pad, pad), xo.F32)
    assert np.max(np.abs(est - exact)) > 1e-2 * np.max(np.abs(exact))


def _layer(seed, B=2, C_in=8, C_out=4, H=8, W=8):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    dY = rng.standard_normal((B, C_out, H, W)).astype(np.float32)
    return X, dY


@pytest.mark.parametrize("dist", [xo.RADEMACHER, xo.GAUSSIAN])
def test_unbiasedness_rate(dist):
    # Eq. (3): the estimator is unbiased, so the mean over S independent seeds
    # approaches the exact gradient like 1/sqrt(S).
    X, dY = _layer(10)
    C_in, r = X.shape[1], 2
    exact = xo.dw_exact(dY, X, 3, 3, (1, 1), (1, 1))
    Xc = X  # the probe output is linear in X; fp32 storage rounding is far below the noise
    S_list = [16, 64, 256, 1024]
    errs = []
    acc = np.zeros_like(exact)
    done = 0
    for S in S_list:
        while done < S:
            Z = xo.probe_matrix(dist, 100000 + done, C_in, r)
            acc += xo.dw_estimate(dY, Xc, Z, 3, 3, (1, 1), (1, 1), xo.F32)
            done += 1
        errs.append(np.linalg.norm(acc / S - exact) / np.linalg.norm(exact))
    slope = np.polyfit(np.log(S_list), np.log(errs), 1)[0]
    assert -0.65 < slope < -0.35, (slope, errs)
    assert errs[-1] < 0.12, errs


@pytest.mark.parametrize("dist", [xo.RADEMACHER, xo.GAUSSIAN])
def test_estimator_variance_formula(dist):
    # From Eq. (3) with unit-variance entries: per entry, with w = dW_exact[m,:,ky,kx],
    #   Var = (|w|^2 + w_n^2)/r  (Gaussian),   (|w|^2 - w_n^2)/r  (Rademacher).
    X, dY = _layer(11, C_in=6, C_out=3, H=6, W=6)
    C_in, r, S = 6, 3, 3000
    exact = xo.dw_exact(dY, X, 3, 3, (1, 1), (1, 1))
    sq = np.zeros_like(exact)
    for s in range(S):
        Z = xo.probe_matrix(dist, 500000 + s, C_in, r)
        d = xo.dw_estimate(dY, X, Z, 3, 3, (1, 1), (1, 1), xo.F32) - exact
        sq += d * d
    var = sq / S
    norm2 = np.sum(exact ** 2, axis=1, keepdims=True)
    sign = 1.0 if dist == xo.GAUSSIAN else -1.0
    want = (norm2 + sign * exact ** 2) / r
    ratio = var.sum() / want.sum()
    assert 0.93 < ratio < 1.07, ratio
    # entrywise within Monte-Carlo scatter
    assert np.all(var < 1.35 * want + 1e-12) and np.all(var > 0.7 * want - 1e-12)


def test_error_decays_like_inverse_sqrt_r():
    # Proposition 1, large-r regime: error ~ |A|_F / sqrt(r)
    X, dY = _layer(12, C_in=64, C_out=4, H=6, W=6)
    exact = xo.dw_exact(dY, X, 3, 3, (1, 1), (1, 1))
    rs = [2, 4, 8, 16, 32]
    errs = []
    for r in rs:
        e = 0.0
        for s in range(24):
            Z = xo.probe_matrix(xo.GAUSSIAN, 900000 + 100 * r + s, 64, r)
            e += np.linalg.norm(xo.dw_estimate(dY, X, Z, 3, 3, (1, 1), (1, 1), xo.F32) - exact) ** 2
        errs.append(np.sqrt(e / 24))
    slope = np.polyfit(np.log(rs), np.log(errs), 1)[0]
    assert -0.6 < slope < -0.4, (slope, errs)


def test_sixteen_bit_storage_effect_is_small():
    # Storing the probed activations in 16 bits perturbs the estimate far less
    # than the 2e-2 parity budget of the 16-bit paths.
    rng = np.random.default_rng(13)
    B, C_in, C_out, H, W, r = 4, 16, 8, 12, 12, 4
    X = np.maximum(rng.standard_normal((B, C_in, H, W)), 0).astype(np.float16).astype(np.float32)
    dY = (0.1 * rng.standard_normal((B, C_out, H, W))).astype(np.float16).astype(np.float32)
    Z = xo.probe_matrix(xo.RADEMACHER, 3, C_in, r)
    e32 = xo.dw_estimate(dY, X, Z, 3, 3, (1, 1), (1, 1), xo.F32)
    e16 = xo.dw_estimate(dY, X, Z, 3, 3, (1, 1), (1, 1), xo.F16)
    eb = xo.dw_estimate(dY, X, Z, 3, 3, (1, 1), (1, 1), xo.BF16)
    scale = np.max(np.abs(e32))
    assert 0 < np.max(np.abs(e16 - e32)) < 2e-3 * scale
    assert 0 < np.max(np.abs(eb - e32)) < 1e-2 * scale


def test_paper_memory_ratio_table():
    # Sec. 4.1: N*C_in/r = 2^(14-gamma) for N = 1024, C_in = 16, r = 2^gamma
    for gamma, ratio in _read_numbers("paper_memory_ratio.txt"):
        assert 1024 * 16 // (2 ** gamma) == ratio == 2 ** (14 - gamma)


# ---------------------------------------------------------------------------
# Block-sparse probing vectors and the 1/nnz scaling (Sec. 3, Eq. (7), Eq. (8))
# ---------------------------------------------------------------------------
def test_sparse_probe_matrix_is_the_dense_one_with_entries_dropped():
    C_in, r = 64, 48
    for dist in (xo.RADEMACHER, xo.GAUSSIAN):
        dense = xo.probe_matrix(dist, 77, C_in, r)
        assert np.array_equal(xo.probe_matrix(dist, 77, C_in, r, 0), dense)
        for keep in (4096, 16384, 24576):
            Z = xo.probe_matrix(dist, 77, C_in, r, keep)
            kept = Z != 0
            assert np.array_equal(Z[kept], dense[kept])                # kept entries are the dense values
            p = keep / 32768.0
            n = C_in * r
            assert abs(kept.mean() - p) < 4.0 * np.sqrt(p * (1 - p) / n)   # Bernoulli(p) per entry (Eq. (7))
            # the keep decision does not depend on the value: +1 and -1 are dropped alike
            if dist == xo.RADEMACHER:
                assert abs(Z.sum()) < 4.0 * np.sqrt(n * p)
        # the mask is its own stream: it is the same for both distributions of one seed
    assert np.array_equal(xo.probe_matrix(xo.RADEMACHER, 77, C_in, r, 16384) != 0,
                          xo.probe_matrix(xo.GAUSSIAN, 77, C_in, r, 16384) != 0)
    assert not np.array_equal(xo.probe_matrix(xo.RADEMACHER, 77, C_in, r, 16384) != 0,
                              xo.probe_matrix(xo.RADEMACHER, 78, C_in, r, 16384) != 0)


@pytest.mark.parametrize("case", CLOSED_FORM_CASES)
def test_sparse_estimate_closed_form(case):
    # With the scaling of Eq. (8) the estimator is still linear in X:
    #   dW_est[m,n] = sum_n' (D Z Z^T)[n,n'] dW_exact[m,n'],  D = diag(1 / nnz(Z_n)).
    B, C_in, C_out, H, W, k, st, p, r, dist = case
    rng = np.random.default_rng(17)
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    Ho, Wo = xo.out_extent(H, k, st, p), xo.out_extent(W, k, st, p)
    dY = rng.standard_normal((B, C_out, Ho, Wo)).astype(np.float32)
    Z = xo.probe_matrix(dist, 12, C_in, r, 20000)
    Z[0, :] = 0.0                                  # a block without any probe: nothing to estimate from
    Xt = xo.probe_fwd(X, Z, xo.F32)
    est = xo.dw_from_xt(dY, Xt, Z, k, k, (st, st), (p, p), nnz_norm=True)
    w = torch.zeros((C_out, C_in, k, k), dtype=torch.float64, requires_grad=True)
    F.conv2d(torch.from_numpy(X).double(), w, stride=st, padding=p).backward(torch.from_numpy(dY).double())
    Zd = Z.astype(np.float64)
    nnz = (Zd != 0).sum(axis=1)
    D = np.where(nnz > 0, 1.0 / np.maximum(nnz, 1), 0.0)
    want = np.einsum("nq,mqyx->mnyx", D[:, None] * (Zd @ Zd.T), w.grad.numpy())
    assert np.max(np.abs(est - want)) <= 2e-6 * np.max(np.abs(want))
    assert np.all(est[:, 0] == 0.0)
    # dense Z: nnz = r, the two scalings coincide
    Zf = xo.probe_matrix(dist, 12, C_in, r)
    Xtf = xo.probe_fwd(X, Zf, xo.F32)
    assert np.allclose(xo.dw_from_xt(dY, Xtf, Zf, k, k, (st, st), (p, p), nnz_norm=True),
                       xo.dw_from_xt(dY, Xtf, Zf, k, k, (st, st), (p, p)), rtol=1e-12, atol=0)


def test_sparse_estimator_is_unbiased_with_the_nnz_scaling_only():
    # Eq. (8): dividing by nnz(Z_n) keeps the estimator unbiased; dividing by r
    # (Eq. (6)) would shrink it by the keep probability.
    X, dY = _layer(14)
    C_in, r, keep = X.shape[1], 16, 16384          # p = 1/2; a block is empty with probability 2^-16
    exact = xo.dw_exact(dY, X, 3, 3, (1, 1), (1, 1))
    S_list = [16, 64, 256, 1024]
    errs, acc, acc_r, done = [], np.zeros_like(exact), np.zeros_like(exact), 0
    for S in S_list:
        while done < S:
            Z = xo.probe_matrix(xo.RADEMACHER, 300000 + done, C_in, r, keep)
            Xt = xo.probe_fwd(X, Z, xo.F32)
            G = xo.correlate(dY, Xt, 3, 3, (1, 1), (1, 1))
            acc += xo.expand(G, Z, nnz_norm=True)
            acc_r += xo.expand(G, Z)
            done += 1
        errs.append(np.linalg.norm(acc / S - exact) / np.linalg.norm(exact))
    slope = np.polyfit(np.log(S_list), np.log(errs), 1)[0]
    assert -0.65 < slope < -0.35, (slope, errs)
    shrink = np.sum(acc_r / done * exact) / np.sum(exact * exact)
    assert abs(shrink - 0.5) < 0.05, shrink


# ---------------------------------------------------------------------------
# volumetric layers (one more spatial axis)
# ---------------------------------------------------------------------------
VOL_SHAPES = [
    # B, C_in, C_out, (D, H, W), k, stride, pad
    (2, 3, 4, (5, 6, 7), (3, 3, 3), (1, 1, 1), (1, 1, 1)),
    (1, 2, 3, (6, 5, 8), (3, 1, 2), (2, 1, 2), (1, 0, 1)),
    (2, 2, 2, (4, 7, 5), (1, 3, 3), (1, 2, 1), (0, 2, 0)),
    (1, 3, 2, (7, 4, 4), (5, 3, 1), (1, 1, 1), (2, 1, 0)),
]


def _vol(seed, B, C_in, C_out, dims, k, stride, pad):
    rng = np.random.default_rng(seed)
    D, H, W = dims
    out = tuple(xo.out_extent(n, kk, s, p) for n, kk, s, p in zip(dims, k, stride, pad))
    X = rng.standard_normal((B, C_in, D, H, W)).astype(np.float32)
    dY = rng.standard_normal((B, C_out) + out).astype(np.float32)
    return X, dY


@pytest.mark.parametrize("shape", VOL_SHAPES, ids=[str(i) for i in range(len(VOL_SHAPES))])
def test_exact_3d_gradient_matches_autograd_of_conv3d(shape):
    # Eq. (2)/(5) with kD*kH*kW offsets is the weight gradient of the library's 3-D convolution
    B, C_in, C_out, dims, k, stride, pad = shape
    X, dY = _vol(31, *shape)
    got = xo.dw_exact3d(dY, X, k, stride, pad)
    w = torch.zeros((C_out, C_in) + k, dtype=torch.float64, requires_grad=True)
    F.conv3d(torch.from_numpy(X).double(), w, stride=stride, padding=pad).backward(torch.from_numpy(dY).double())
    want = w.grad.numpy()
    assert got.shape == want.shape
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


def test_3d_routines_reduce_to_the_2d_ones_for_a_single_slice():
    rng = np.random.default_rng(32)
    B, C_in, C_out, H, W, r = 2, 3, 4, 6, 5, 4
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    dY = rng.standard_normal((B, C_out, 3, 5)).astype(np.float32)      # 3x3, stride (2,1), pad (1,1)
    Z = xo.probe_matrix(xo.GAUSSIAN, 5, C_in, r)
    Xt2 = xo.probe_fwd(X, Z, xo.BF16)
    Xt3 = xo.probe_fwd3d(X[:, :, None], Z, xo.BF16)
    assert np.array_equal(Xt3[:, :, 0], Xt2)
    want = xo.dw_from_xt(dY, Xt2, Z, 3, 3, (2, 1), (1, 1))
    got = xo.dw_from_xt3d(dY[:, :, None], Xt3, Z, (1, 3, 3), (1, 2, 1), (0, 1, 1))
    assert np.allclose(got[:, :, 0], want, rtol=1e-13, atol=0)


def test_3d_estimate_with_a_full_rank_orthogonal_probe_is_exact():
    # Z Z^T = r I (Hadamard rows): the estimator of Eq. (6) returns the exact gradient
    shape = VOL_SHAPES[0][:1] + (4, 3) + VOL_SHAPES[0][3:]
    X, dY = _vol(33, *shape)
    Zh = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]], dtype=np.float32)
    k, stride, pad = shape[4:]
    Xt = xo.probe_fwd3d(X, Zh, xo.F32)
    est = xo.dw_from_xt3d(dY, Xt, Zh, k, stride, pad)
    exact = xo.dw_exact3d(dY, X, k, stride, pad)
    assert np.max(np.abs(est - exact)) <= 1e-5 * np.max(np.abs(exact))


def test_sampled_3d_entries_match_the_full_routines():
    shape = VOL_SHAPES[1]
    B, C_in, C_out, dims, k, stride, pad = shape
    X, dY = _vol(34, *shape)
    r = 3
    Z = xo.probe_matrix(xo.GAUSSIAN, 9, C_in, r)
    Xt = xo.probe_fwd3d(X, Z, xo.F32)
    full_x = xo.dw_exact3d(dY, X, k, stride, pad)
    full_e = xo.dw_from_xt3d(dY, Xt, Z, k, stride, pad)
    idx = np.array([(m, n, kz, ky, kx) for m in range(C_out) for n in range(C_in)
                    for kz in range(k[0]) for ky in range(k[1]) for kx in range(k[2])], dtype=np.int32)
    assert np.allclose(xo.dw_exact3d_at(dY, X, idx, k, stride, pad), full_x.reshape(-1), rtol=1e-13, atol=0)
    assert np.allclose(xo.dw_from_xt3d_at(dY, Xt, Z, idx, k, stride, pad), full_e.reshape(-1), rtol=1e-12, atol=1e-300)


# ---------------------------------------------------------------------------
# the estimator with probing vectors over pixels and channels (Eq. (6) as stated)
# ---------------------------------------------------------------------------
def _pixel_case(seed, B=3, C_in=2, C_out=3, H=5, W=4, k=(3, 2), stride=(1, 2), pad=(1, 1)):
    rng = np.random.default_rng(seed)
    Ho, Wo = xo.out_extent(H, k[0], stride[0], pad[0]), xo.out_extent(W, k[1], stride[1], pad[1])
    X = rng.standard_normal((B, C_in, H, W)).astype(np.float32)
    dY = rng.standard_normal((B, C_out, Ho, Wo)).astype(np.float32)
    return X, dY, k, stride, pad


def test_pixel_probe_estimator_matches_its_matrix_form():
    # Eq. (6) written with explicit shift matrices: dw_i^{m,n} = (1/r) tr(L^m T_{-k(i)} Z_n),
    # L^m = Xbar^T dY^m, the shift as a 0/1 matrix with zero padding
    X, dY, k, stride, pad = _pixel_case(41)
    B, C_in, H, W = X.shape
    C_out, Ho, Wo = dY.shape[1:]
    r, N, Np = 5, H * W, Ho * Wo
    Z = xo.pixel_probe_matrix(xo.GAUSSIAN, 17, C_in, H, W, r)
    Xbar = xo.pixel_probe_fwd(X, Z)
    assert np.allclose(Xbar, X.reshape(B, -1).astype(np.float64) @ Z.astype(np.float64), rtol=1e-6, atol=1e-6)
    got = xo.pixel_dw_estimate(dY, Xbar, Z, C_in, H, W, k[0], k[1], stride, pad)
    Zb = Z.astype(np.float64).reshape(C_in, N, r)
    for m in range(C_out):
        L = Xbar.astype(np.float64).T @ dY[:, m].reshape(B, Np).astype(np.float64)     # r x N' (Alg. 1 bwd step 3)
        for n in range(C_in):
            for ky in range(k[0]):
                for kx in range(k[1]):
                    T = np.zeros((Np, N))                                      # T[p', q] = 1 if output pixel p' reads input pixel q
                    for oy in range(Ho):
                        for ox in range(Wo):
                            iy, ix = oy * stride[0] + ky - pad[0], ox * stride[1] + kx - pad[1]
                            if 0 <= iy < H and 0 <= ix < W:
                                T[oy * Wo + ox, iy * W + ix] = 1.0
                    want = np.trace(L @ T @ Zb[n]) / r                         # the factor 1/r once, at the end (bwd step 4)
                    assert abs(got[m, n, ky, kx] - want) <= 1e-12 * max(1.0, abs(want))    # nothing between the two is rounded


def test_pixel_probe_with_an_orthogonal_full_rank_probe_is_exact():
    # r = C_in*N probing vectors with Z Z^T = r I: every trace is probed exactly
    X, dY, k, stride, pad = _pixel_case(42, B=2, C_in=2, C_out=2, H=4, W=4)
    B, C_in, H, W = X.shape
    K = C_in * H * W                                                         # 32: a Sylvester Hadamard matrix exists
    Hd = np.array([[1.0]])
    while Hd.shape[0] < K:
        Hd = np.block([[Hd, Hd], [Hd, -Hd]])
    Z = Hd.astype(np.float32)
    est = xo.pixel_dw_estimate(dY, xo.pixel_probe_fwd(X, Z), Z, C_in, H, W, k[0], k[1], stride, pad)
    exact = xo.dw_exact(dY, X, k[0], k[1], stride, pad)
    assert np.max(np.abs(est - exact)) <= 1e-5 * np.max(np.abs(exact))


def test_pixel_probe_estimator_is_unbiased():
    X, dY, k, stride, pad = _pixel_case(43, B=4, C_in=2, C_out=2, H=6, W=6, k=(3, 3), stride=(1, 1), pad=(1, 1))
    C_in, H, W = X.shape[1:]
    exact = xo.dw_exact(dY, X, 3, 3, stride, pad)
    S_list, errs, acc, done = [8, 32, 128, 512], [], np.zeros_like(exact), 0
    for S in S_list:
        while done < S:
            Z = xo.pixel_probe_matrix(xo.RADEMACHER, 500000 + done, C_in, H, W, 8)
            acc += xo.pixel_dw_estimate(dY, xo.pixel_probe_fwd(X, Z), Z, C_in, H, W, 3, 3, stride, pad)
            done += 1
        errs.append(np.linalg.norm(acc / S - exact) / np.linalg.norm(exact))
    slope = np.polyfit(np.log(S_list), np.log(errs), 1)[0]
    assert -0.65 < slope < -0.35, (slope, errs)


def test_pixel_probe_rounds_only_what_algorithm_1_saves():
    # Algorithm 1 saves Xbar and the seed.  Z is drawn in the storage type and Xbar is kept in fp32; the outer product
    # L = Xbar^T dY of backward step 3 is a transient: with 16-bit probing vectors the estimate still equals the
    # matrix form evaluated in double from the saved Xbar, to summation order
    X, dY, k, stride, pad = _pixel_case(44)
    B, C_in, H, W = X.shape
    C_out, Ho, Wo = dY.shape[1:]
    r = 4
    Z = xo.pixel_probe_matrix(xo.GAUSSIAN, 3, C_in, H, W, r, xo.BF16)
    assert np.array_equal(Z, np.array([xo.round_storage(v, xo.BF16) for v in Z.reshape(-1)], dtype=np.float32).reshape(Z.shape))
    Xbar = xo.pixel_probe_fwd(X, Z)
    assert Xbar.dtype == np.float32
    got = xo.pixel_dw_estimate(dY, Xbar, Z, C_in, H, W, k[0], k[1], stride, pad)
    # the same through the library routines for the channel-probe case: the probing vectors as an r-image batch of
    # activations, L as its residual: dW = (1/r) * exact gradient of that batch
    L = np.einsum("bj,bmyx->jmyx", Xbar.astype(np.float64), dY.astype(np.float64))
    Zimg = Z.astype(np.float64).reshape(C_in, H, W, r).transpose(3, 0, 1, 2)
    want = np.zeros_like(got)
    for ky in range(k[0]):
        for kx in range(k[1]):
            for oy in range(Ho):
                iy = oy * stride[0] + ky - pad[0]
                if not 0 <= iy < H:
                    continue
                for ox in range(Wo):
                    ix = ox * stride[1] + kx - pad[1]
                    if 0 <= ix < W:
                        want[:, :, ky, kx] += L[:, :, oy, ox].T @ Zimg[:, :, iy, ix]
    want /= r
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


def test_block_sparse_pixel_probes_keep_whole_blocks_and_match_the_matrix_form():
    # Eq. (7): a block z_{n,j} (all pixels of channel n in vector j) is kept or zeroed as a whole, the kept ones equal
    # the dense matrix; Eq. (8): dw^{m,n} = (1/nnz(Z_n)) sum_j tr(L_j T Z_{n,j})
    X, dY, k, stride, pad = _pixel_case(45, B=3, C_in=4, C_out=2, H=4, W=5)
    B, C_in, H, W = X.shape
    C_out, Ho, Wo = dY.shape[1:]
    r, N, Np, keep = 12, H * W, Ho * Wo, 16384
    Zd = xo.pixel_probe_matrix(xo.GAUSSIAN, 23, C_in, H, W, r)
    Z = xo.pixel_probe_matrix(xo.GAUSSIAN, 23, C_in, H, W, r, keep_q15=keep)
    Zb, Zdb = Z.reshape(C_in, N, r), Zd.reshape(C_in, N, r)
    kept = np.any(Zb != 0, axis=1)                                            # [C_in, r]
    assert 0.25 < kept.mean() < 0.75
    assert np.array_equal(Zb, Zdb * kept[:, None, :])
    assert np.array_equal(kept.reshape(-1), xo.keep_mask(23, keep, C_in * r) != 0)
    assert np.array_equal(xo.pixel_block_counts(Z, C_in), kept.sum(axis=1))
    frac = (xo.keep_mask(7, 8192, 200000) != 0).mean()
    assert abs(frac - 0.25) < 0.005
    Xbar = xo.pixel_probe_fwd(X, Z)
    got = xo.pixel_dw_estimate(dY, Xbar, Z, C_in, H, W, k[0], k[1], stride, pad, nnz_norm=True)
    coef = (Xbar * np.float32(1.0 / r)).astype(np.float64) * r                # the oracle forms Xbar / r in fp32
    for m in range(C_out):
        L = coef.T @ dY[:, m].reshape(B, Np).astype(np.float64)
        for n in range(C_in):
            nnz = int(kept[n].sum())
            for ky in range(k[0]):
                for kx in range(k[1]):
                    T = np.zeros((Np, N))
                    for oy in range(Ho):
                        for ox in range(Wo):
                            iy, ix = oy * stride[0] + ky - pad[0], ox * stride[1] + kx - pad[1]
                            if 0 <= iy < H and 0 <= ix < W:
                                T[oy * Wo + ox, iy * W + ix] = 1.0
                    want = np.trace(L @ T @ Zb[n].astype(np.float64)) / nnz if nnz else 0.0
                    assert abs(got[m, n, ky, kx] - want) <= 1e-6 * max(1.0, abs(want))


def test_block_sparse_pixel_probe_estimator_is_unbiased_with_the_nnz_scaling_only():
    X, dY, k, stride, pad = _pixel_case(46, B=4, C_in=3, C_out=2, H=6, W=6, k=(3, 3), stride=(1, 1), pad=(1, 1))
    C_in, H, W = X.shape[1:]
    exact = xo.dw_exact(dY, X, 3, 3, stride, pad)
    S_list, errs, acc, acc_r, done = [16, 64, 256, 1024], [], np.zeros_like(exact), np.zeros_like(exact), 0
    for S in S_list:
        while done < S:
            Z = xo.pixel_probe_matrix(xo.RADEMACHER, 700000 + done, C_in, H, W, 16, keep_q15=16384)
            Xbar = xo.pixel_probe_fwd(X, Z)
            acc += xo.pixel_dw_estimate(dY, Xbar, Z, C_in, H, W, 3, 3, stride, pad, nnz_norm=True)
            acc_r += xo.pixel_dw_estimate(dY, Xbar, Z, C_in, H, W, 3, 3, stride, pad)
            done += 1
        errs.append(np.linalg.norm(acc / S - exact) / np.linalg.norm(exact))
    slope = np.polyfit(np.log(S_list), np.log(errs), 1)[0]
    assert -0.65 < slope < -0.35, (slope, errs)
    shrink = np.sum(acc_r / done * exact) / np.sum(exact * exact)
    assert abs(shrink - 0.5) < 0.05, shrink


# ---------------------------------------------------------------------------
# independent probing: every input channel with probes of its own (Sec. 3, the alternative to Eq. (6))
# ---------------------------------------------------------------------------
def _hadamard(n):
    Hd = np.array([[1.0]])
    while Hd.shape[0] < n:
        Hd = np.block([[Hd, Hd], [Hd, -Hd]])
    return Hd


def test_independent_probing_with_orthogonal_probes_per_channel_is_exact():
    # r = N probes per channel with Z_n Z_n^T = r I probe every channel pair exactly, although r < C_in*N; the
    # channels get different orthogonal matrices, so a probe taken from the wrong channel fails
    X, dY, k, stride, pad = _pixel_case(47, B=3, C_in=3, C_out=2, H=4, W=4)
    B, C_in, H, W = X.shape
    N = H * W
    rng = np.random.default_rng(5)
    Z = np.concatenate([(_hadamard(N) * rng.choice([-1.0, 1.0], size=(1, N)))[rng.permutation(N)] for _ in range(C_in)])
    Z = Z.astype(np.float32)
    Xbar = xo.pixel_indep_probe_fwd(X, Z)
    assert Xbar.shape == (B, C_in, N)
    est = xo.pixel_indep_dw_estimate(dY, Xbar, Z, C_in, H, W, k[0], k[1], stride, pad)
    exact = xo.dw_exact(dY, X, k[0], k[1], stride, pad)
    assert np.max(np.abs(est - exact)) <= 1e-5 * np.max(np.abs(exact))
    # the same probes used for all channels at once (Eq. (6)) are not exact: the test separates the two modes
    sim = xo.pixel_dw_estimate(dY, xo.pixel_probe_fwd(X, Z), Z, C_in, H, W, k[0], k[1], stride, pad)
    assert np.max(np.abs(sim - exact)) > 0.05 * np.max(np.abs(exact))


def test_independent_probing_state_sums_to_the_multi_channel_state_and_has_no_crosstalk():
    X, dY, k, stride, pad = _pixel_case(48, B=4, C_in=3, C_out=2, H=5, W=4)
    B, C_in, H, W = X.shape
    r = 6
    Z = xo.pixel_probe_matrix(xo.GAUSSIAN, 29, C_in, H, W, r)
    Xbar = xo.pixel_indep_probe_fwd(X, Z)
    # Eq. (6) probes the stacked matrix: its state is the sum of the per-channel states
    np.testing.assert_allclose(Xbar.astype(np.float64).sum(axis=1), xo.pixel_probe_fwd(X, Z), rtol=0, atol=2e-5)
    # an input that lives on one channel gives no gradient on the others, whatever the probes (the multi-channel
    # estimate does: that is its crosstalk)
    X1 = X.copy()
    X1[:, 1:] = 0
    est = xo.pixel_indep_dw_estimate(dY, xo.pixel_indep_probe_fwd(X1, Z), Z, C_in, H, W, k[0], k[1], stride, pad)
    assert np.all(est[:, 1:] == 0) and np.any(est[:, 0] != 0)
    sim = xo.pixel_dw_estimate(dY, xo.pixel_probe_fwd(X1, Z), Z, C_in, H, W, k[0], k[1], stride, pad)
    assert np.any(sim[:, 1:] != 0)


def test_independent_probing_equals_multi_channel_probing_with_block_diagonal_vectors():
    # C_in*r vectors, vector (n, j) non-zero on channel n only where it equals Z_n[:, j]: Eq. (6) with these vectors
    # and the factor 1/r is the independent estimate
    X, dY, k, stride, pad = _pixel_case(49, B=3, C_in=3, C_out=2, H=4, W=5)
    B, C_in, H, W = X.shape
    N, r = H * W, 4
    Z = xo.pixel_probe_matrix(xo.RADEMACHER, 31, C_in, H, W, r)
    Zd = np.zeros((C_in * N, C_in * r), dtype=np.float32)
    for n in range(C_in):
        Zd[n * N:(n + 1) * N, n * r:(n + 1) * r] = Z[n * N:(n + 1) * N]
    Xbar = xo.pixel_indep_probe_fwd(X, Z)
    np.testing.assert_allclose(xo.pixel_probe_fwd(X, Zd), Xbar.reshape(B, C_in * r), rtol=0, atol=1e-6)
    want = xo.pixel_dw_estimate(dY, Xbar.reshape(B, C_in * r), Zd, C_in, H, W, k[0], k[1], stride, pad) * C_in
    got = xo.pixel_indep_dw_estimate(dY, Xbar, Z, C_in, H, W, k[0], k[1], stride, pad)
    assert np.max(np.abs(got - want)) <= 2e-6 * np.max(np.abs(want))


def test_independent_probing_is_unbiased_and_closer_than_multi_channel_probing():
    X, dY, k, stride, pad = _pixel_case(50, B=4, C_in=4, C_out=2, H=6, W=6, k=(3, 3), stride=(1, 1), pad=(1, 1))
    C_in, H, W = X.shape[1:]
    exact = xo.dw_exact(dY, X, 3, 3, stride, pad)
    acc, e_ind, e_sim, S = np.zeros_like(exact), 0.0, 0.0, 256
    for t in range(S):
        Z = xo.pixel_probe_matrix(xo.RADEMACHER, 900000 + t, C_in, H, W, 8)
        ind = xo.pixel_indep_dw_estimate(dY, xo.pixel_indep_probe_fwd(X, Z), Z, C_in, H, W, 3, 3, stride, pad)
        sim = xo.pixel_dw_estimate(dY, xo.pixel_probe_fwd(X, Z), Z, C_in, H, W, 3, 3, stride, pad)
        acc += ind
        e_ind += np.sum((ind - exact) ** 2)
        e_sim += np.sum((sim - exact) ** 2)
    one = np.sqrt(e_ind / S) / np.linalg.norm(exact)
    mean = np.linalg.norm(acc / S - exact) / np.linalg.norm(exact)
    assert mean < 3.0 * one / np.sqrt(S), (mean, one)                       # the mean of S draws shrinks like 1/sqrt(S)
    assert e_ind < 0.6 * e_sim, (e_ind, e_sim)                               # C_in = 4 channels of crosstalk removed


# ---------------------------------------------------------------------------
# ReLU that keeps signs only (Sec. 5, overall effective memory savings: layers that relied on the convolution's stored input)
# ---------------------------------------------------------------------------
def test_sign_relu_bit_layout_and_values():
    x = -np.ones(130, dtype=np.float32)
    x[[0, 63, 64, 129]] = [2.0, 0.5, 3.0, 1.0]
    x[5] = 0.0                                            # zero is not positive: no gradient through it
    y, words = xo.relu_sign_fwd(x)
    assert words.dtype == np.uint64 and words.tolist() == [1 | (1 << 63), 1, 2]
    assert np.array_equal(y, np.where(x > 0, x, 0))
    dy = np.arange(1, 131, dtype=np.float32)
    dx = xo.relu_sign_bwd(dy, words)
    assert np.array_equal(np.nonzero(dx)[0], [0, 63, 64, 129]) and dx[129] == 130.0


def test_sign_relu_matches_autograd():
    import torch
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 5, 7, 6)).astype(np.float32)
    x[0, 0, 0, :3] = 0.0
    dy = rng.standard_normal(x.shape).astype(np.float32)
    t = torch.from_numpy(x).requires_grad_(True)
    out = torch.relu(t)
    out.backward(torch.from_numpy(dy))
    y, words = xo.relu_sign_fwd(x)
    assert np.array_equal(y, out.detach().numpy())
    assert words.size == (x.size + 63) // 64
    assert np.array_equal(xo.relu_sign_bwd(dy, words), t.grad.numpy())
