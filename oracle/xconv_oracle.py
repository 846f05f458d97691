"""ctypes front end of the CPU oracle (oracle/xconv_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this module.  The functions marshal
numpy arrays into the C routine of the same name, where the paper's formulas
are written out (Sec. 3 Eq. (2), (3), (5), (6); Algorithm 1); what is stated
here in numpy is the block mask and 1/nnz scaling of Eq. (7)/(8) and the
independent probing mode, a loop of single-channel calls.

Array conventions: float32 inputs whose values are already representable in
the storage type; gradients come back as float64.
dtype codes: 0 fp32, 1 bf16, 2 fp16.  dist codes: 0 Rademacher, 1 Gaussian.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

F32, BF16, F16 = 0, 1, 2
RADEMACHER, GAUSSIAN = 0, 1

_c_f32p = ctypes.POINTER(ctypes.c_float)
_c_f64p = ctypes.POINTER(ctypes.c_double)
_c_i32p = ctypes.POINTER(ctypes.c_int32)


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build(force=True)
        L = ctypes.CDLL(path)
        L.xo_splitmix64.restype = ctypes.c_uint64
        L.xo_splitmix64.argtypes = [ctypes.POINTER(ctypes.c_uint64)]
        L.xo_stream_word.restype = ctypes.c_uint64
        L.xo_stream_word.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        L.xo_probe_matrix.restype = ctypes.c_int
        L.xo_probe_matrix.argtypes = [ctypes.c_int, ctypes.c_uint64, ctypes.c_int, ctypes.c_int, _c_f32p]
        L.xo_round_storage.restype = ctypes.c_double
        L.xo_round_storage.argtypes = [ctypes.c_double, ctypes.c_int]
        L.xo_probe_fwd.restype = None
        L.xo_probe_fwd.argtypes = [_c_f32p, _c_f32p, _c_f32p] + [ctypes.c_int] * 6
        L.xo_correlate.restype = None
        L.xo_correlate.argtypes = [_c_f32p, _c_f32p, _c_f64p] + [ctypes.c_int] * 11
        L.xo_dw_exact.restype = None
        L.xo_dw_exact.argtypes = [_c_f32p, _c_f32p, _c_f64p] + [ctypes.c_int] * 11
        L.xo_probe_matrix_sparse.restype = ctypes.c_int
        L.xo_probe_matrix_sparse.argtypes = [ctypes.c_int, ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int, _c_f32p]
        L.xo_expand_nnz.restype = None
        L.xo_expand_nnz.argtypes = [_c_f64p, _c_f32p, _c_f64p] + [ctypes.c_int] * 5
        L.xo_expand.restype = None
        L.xo_expand.argtypes = [_c_f64p, _c_f32p, _c_f64p] + [ctypes.c_int] * 5
        L.xo_dw_from_xt.restype = None
        L.xo_dw_from_xt.argtypes = [_c_f32p, _c_f32p, _c_f32p, _c_f64p] + [ctypes.c_int] * 12
        L.xo_dw_estimate.restype = None
        L.xo_dw_estimate.argtypes = [_c_f32p, _c_f32p, _c_f32p, _c_f64p] + [ctypes.c_int] * 13
        L.xo_dw_from_xt_at.restype = None
        L.xo_dw_from_xt_at.argtypes = [_c_f32p, _c_f32p, _c_f32p, _c_i32p, ctypes.c_int, _c_f64p] + [ctypes.c_int] * 12
        L.xo_dw_exact_at.restype = None
        L.xo_dw_exact_at.argtypes = [_c_f32p, _c_f32p, _c_i32p, ctypes.c_int, _c_f64p] + [ctypes.c_int] * 11
        L.xo_conv_fwd.restype = None
        L.xo_correlate3d.restype = None
        L.xo_correlate3d.argtypes = [_c_f32p, _c_f32p, _c_f64p] + [ctypes.c_int] * 15
        L.xo_correlate3d_at.restype = None
        L.xo_correlate3d_at.argtypes = [_c_f32p, _c_f32p, _c_i32p, ctypes.c_int, _c_f64p] + [ctypes.c_int] * 15
        L.xo_keep_mask.restype = None
        L.xo_keep_mask.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_size_t, _c_f32p]
        L.xo_round_array.restype = None
        L.xo_round_array.argtypes = [_c_f32p, ctypes.c_size_t, ctypes.c_int]
        L.xo_pixel_probe_fwd.restype = None
        L.xo_pixel_probe_fwd.argtypes = [_c_f32p, _c_f32p, _c_f32p] + [ctypes.c_int] * 5
        L.xo_pixel_dw_estimate.restype = None
        L.xo_pixel_dw_estimate.argtypes = [_c_f32p, _c_f32p, _c_f32p, _c_f64p] + [ctypes.c_int] * 12
        L.xo_conv_fwd.argtypes = [_c_f32p, _c_f64p, _c_f64p] + [ctypes.c_int] * 11
        L.xo_dx.restype = None
        L.xo_dx.argtypes = [_c_f32p, _c_f64p, _c_f64p] + [ctypes.c_int] * 11
        _LIB = L
    return _LIB


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_c_f32p)


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_c_f64p)


def out_extent(n, k, stride, pad):
    span = n + 2 * pad - k
    return 0 if span < 0 else span // stride + 1


def splitmix64_stream(state, count):
    st = ctypes.c_uint64(state)
    return [int(lib().xo_splitmix64(ctypes.byref(st))) for _ in range(count)]


def stream_word(seed, ctr):
    return int(lib().xo_stream_word(ctypes.c_uint64(seed), ctypes.c_uint64(ctr)))


def probe_matrix(dist, seed, C_in, r, keep_q15=0):
    """Z[C_in, r]; keep_q15 > 0: block-sparse probes (Eq. (7)), entries kept with probability keep_q15 / 32768."""
    Z = np.empty((C_in, r), dtype=np.float32)
    rc = lib().xo_probe_matrix_sparse(dist, ctypes.c_uint64(seed), keep_q15, C_in, r, Z.ctypes.data_as(_c_f32p))
    if rc != 0:
        raise ValueError("unknown probe distribution %r" % (dist,))
    return Z


def round_storage(v, dtype):
    return float(lib().xo_round_storage(float(v), dtype))


def probe_fwd(X, Z, dtype=F32):
    X, Xp = _f32(X)
    Z, Zp = _f32(Z)
    B, C_in, H, W = X.shape
    r = Z.shape[1]
    assert Z.shape[0] == C_in
    Xt = np.empty((B, r, H, W), dtype=np.float32)
    lib().xo_probe_fwd(Xp, Zp, Xt.ctypes.data_as(_c_f32p), B, C_in, H, W, r, dtype)
    return Xt


def correlate(dY, A, kH, kW, stride=(1, 1), pad=(0, 0)):
    dY, dYp = _f32(dY)
    A, Ap = _f32(A)
    B, C_out, Ho, Wo = dY.shape
    _, Q, H, W = A.shape
    assert Ho == out_extent(H, kH, stride[0], pad[0]) and Wo == out_extent(W, kW, stride[1], pad[1])
    G = np.empty((C_out, Q, kH, kW), dtype=np.float64)
    lib().xo_correlate(dYp, Ap, G.ctypes.data_as(_c_f64p), B, C_out, Q, H, W,
                       kH, kW, stride[0], stride[1], pad[0], pad[1])
    return G


def dw_exact(dY, X, kH, kW, stride=(1, 1), pad=(0, 0)):
    dY, dYp = _f32(dY)
    X, Xp = _f32(X)
    B, C_out, Ho, Wo = dY.shape
    _, C_in, H, W = X.shape
    assert Ho == out_extent(H, kH, stride[0], pad[0]) and Wo == out_extent(W, kW, stride[1], pad[1])
    dW = np.empty((C_out, C_in, kH, kW), dtype=np.float64)
    lib().xo_dw_exact(dYp, Xp, dW.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W,
                      kH, kW, stride[0], stride[1], pad[0], pad[1])
    return dW


def expand(G, Z, nnz_norm=False):
    """dW = Z G / r (Eq. (6) step (iii)), or with nnz_norm rows scaled by 1 / nnz(Z_n) (Eq. (8))."""
    G, Gp = _f64(G)
    Z, Zp = _f32(Z)
    C_out, r, kH, kW = G.shape
    C_in = Z.shape[0]
    assert Z.shape[1] == r
    dW = np.empty((C_out, C_in, kH, kW), dtype=np.float64)
    (lib().xo_expand_nnz if nnz_norm else lib().xo_expand)(Gp, Zp, dW.ctypes.data_as(_c_f64p), C_out, C_in, r, kH, kW)
    return dW


def dw_from_xt(dY, Xt, Z, kH, kW, stride=(1, 1), pad=(0, 0), nnz_norm=False):
    if nnz_norm:    # the two steps one after the other, the second with the scaling of Eq. (8)
        return expand(correlate(dY, Xt, kH, kW, stride, pad), Z, nnz_norm=True)
    dY, dYp = _f32(dY)
    Xt, Xtp = _f32(Xt)
    Z, Zp = _f32(Z)
    B, C_out, Ho, Wo = dY.shape
    _, r, H, W = Xt.shape
    C_in = Z.shape[0]
    assert Z.shape[1] == r
    assert Ho == out_extent(H, kH, stride[0], pad[0]) and Wo == out_extent(W, kW, stride[1], pad[1])
    dW = np.empty((C_out, C_in, kH, kW), dtype=np.float64)
    lib().xo_dw_from_xt(dYp, Xtp, Zp, dW.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W, r,
                        kH, kW, stride[0], stride[1], pad[0], pad[1])
    return dW


def dw_estimate(dY, X, Z, kH, kW, stride=(1, 1), pad=(0, 0), dtype=F32):
    dY, dYp = _f32(dY)
    X, Xp = _f32(X)
    Z, Zp = _f32(Z)
    B, C_out, Ho, Wo = dY.shape
    _, C_in, H, W = X.shape
    r = Z.shape[1]
    assert Z.shape[0] == C_in
    assert Ho == out_extent(H, kH, stride[0], pad[0]) and Wo == out_extent(W, kW, stride[1], pad[1])
    dW = np.empty((C_out, C_in, kH, kW), dtype=np.float64)
    lib().xo_dw_estimate(dYp, Xp, Zp, dW.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W, r,
                         kH, kW, stride[0], stride[1], pad[0], pad[1], dtype)
    return dW


def dw_from_xt_at(dY, Xt, Z, idx, kH, kW, stride=(1, 1), pad=(0, 0)):
    dY, dYp = _f32(dY)
    Xt, Xtp = _f32(Xt)
    Z, Zp = _f32(Z)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    B, C_out, Ho, Wo = dY.shape
    _, r, H, W = Xt.shape
    C_in = Z.shape[0]
    out = np.empty(idx.shape[0], dtype=np.float64)
    lib().xo_dw_from_xt_at(dYp, Xtp, Zp, idx.ctypes.data_as(_c_i32p), idx.shape[0],
                           out.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W, r,
                           kH, kW, stride[0], stride[1], pad[0], pad[1])
    return out


def dw_exact_at(dY, X, idx, kH, kW, stride=(1, 1), pad=(0, 0)):
    dY, dYp = _f32(dY)
    X, Xp = _f32(X)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    B, C_out, Ho, Wo = dY.shape
    _, C_in, H, W = X.shape
    out = np.empty(idx.shape[0], dtype=np.float64)
    lib().xo_dw_exact_at(dYp, Xp, idx.ctypes.data_as(_c_i32p), idx.shape[0],
                         out.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W,
                         kH, kW, stride[0], stride[1], pad[0], pad[1])
    return out


def dx(dY, Wt, H, W, stride=(1, 1), pad=(0, 0)):
    """Exact input gradient dX [B, C_in, H, W] of the layer (transposed convolution of dY with the weights)."""
    dY, dYp = _f32(dY)
    Wt, Wp = _f64(Wt)
    B, C_out, Ho, Wo = dY.shape
    _, C_in, kH, kW = Wt.shape
    assert Wt.shape[0] == C_out and Ho == out_extent(H, kH, stride[0], pad[0]) and Wo == out_extent(W, kW, stride[1], pad[1])
    dX = np.empty((B, C_in, H, W), dtype=np.float64)
    lib().xo_dx(dYp, Wp, dX.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W, kH, kW, stride[0], stride[1], pad[0], pad[1])
    return dX


def conv_fwd(X, Wt, stride=(1, 1), pad=(0, 0)):
    X, Xp = _f32(X)
    Wt, Wp = _f64(Wt)
    B, C_in, H, W = X.shape
    C_out, _, kH, kW = Wt.shape
    Ho = out_extent(H, kH, stride[0], pad[0])
    Wo = out_extent(W, kW, stride[1], pad[1])
    Y = np.empty((B, C_out, Ho, Wo), dtype=np.float64)
    lib().xo_conv_fwd(Xp, Wp, Y.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W,
                      kH, kW, stride[0], stride[1], pad[0], pad[1])
    return Y


# ---- volumetric layers (one more spatial axis) ------------------------------------
def probe_fwd3d(X, Z, dtype=F32):
    """Xt[b,j,z,y,x] = sum_n Z[n,j] X[b,n,z,y,x]: the probe acts voxel by voxel, so the depth
    axis is folded into the rows of the 2-D routine."""
    X = np.asarray(X)
    B, C_in, D, H, W = X.shape
    return probe_fwd(X.reshape(B, C_in, D * H, W), Z, dtype).reshape(B, -1, D, H, W)


def correlate3d(dY, A, k, stride=(1, 1, 1), pad=(0, 0, 0)):
    dY, dYp = _f32(dY)
    A, Ap = _f32(A)
    B, C_out, Do, Ho, Wo = dY.shape
    _, Q, D, H, W = A.shape
    kD, kH, kW = k
    assert (Do, Ho, Wo) == tuple(out_extent(n, kk, s, p) for n, kk, s, p in zip((D, H, W), k, stride, pad))
    G = np.empty((C_out, Q, kD, kH, kW), dtype=np.float64)
    lib().xo_correlate3d(dYp, Ap, G.ctypes.data_as(_c_f64p), B, C_out, Q, D, H, W, kD, kH, kW,
                         stride[0], stride[1], stride[2], pad[0], pad[1], pad[2])
    return G


def dw_exact3d(dY, X, k, stride=(1, 1, 1), pad=(0, 0, 0)):
    """Exact gradient of a 3-D layer (Eq. (2)/(5) with kD*kH*kW offsets), [C_out,C_in,kD,kH,kW]."""
    return correlate3d(dY, X, k, stride, pad)


def dw_from_xt3d(dY, Xt, Z, k, stride=(1, 1, 1), pad=(0, 0, 0), nnz_norm=False):
    """Backward of Algorithm 1 for a 3-D layer from the stored probe output."""
    G = correlate3d(dY, Xt, k, stride, pad)
    C_out, r, kD, kH, kW = G.shape
    return expand(G.reshape(C_out, r, kD * kH, kW), Z, nnz_norm).reshape(C_out, -1, kD, kH, kW)


def correlate3d_at(dY, A, idx, k, stride=(1, 1, 1), pad=(0, 0, 0)):
    """Entries idx[i] = (m, q, kz, ky, kx) of correlate3d's result."""
    dY, dYp = _f32(dY)
    A, Ap = _f32(A)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 5)
    B, C_out = dY.shape[:2]
    _, Q, D, H, W = A.shape
    out = np.empty(idx.shape[0], dtype=np.float64)
    lib().xo_correlate3d_at(dYp, Ap, idx.ctypes.data_as(_c_i32p), idx.shape[0], out.ctypes.data_as(_c_f64p),
                            B, C_out, Q, D, H, W, k[0], k[1], k[2], stride[0], stride[1], stride[2], pad[0], pad[1], pad[2])
    return out


def dw_exact3d_at(dY, X, idx, k, stride=(1, 1, 1), pad=(0, 0, 0)):
    """Entries idx[i] = (m, n, kz, ky, kx) of the exact 3-D gradient."""
    return correlate3d_at(dY, X, idx, k, stride, pad)


def dw_from_xt3d_at(dY, Xt, Z, idx, k, stride=(1, 1, 1), pad=(0, 0, 0)):
    """Entries idx[i] = (m, n, kz, ky, kx) of dw_from_xt3d: (1/r) sum_j Z[n,j] G[m,j,kz,ky,kx]
    (Eq. (6) step (iii)) with the r entries of G each sample needs."""
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 5)
    Z = np.asarray(Z, dtype=np.float64)
    r = Z.shape[1]
    gi = np.repeat(idx, r, axis=0)
    gi[:, 1] = np.tile(np.arange(r, dtype=np.int32), idx.shape[0])
    G = correlate3d_at(dY, Xt, gi, k, stride, pad).reshape(idx.shape[0], r)
    return np.einsum("ij,ij->i", Z[idx[:, 1]], G) / r


# ---- the estimator with probing vectors over pixels and channels (Eq. (6), Algorithm 1 as stated) ----
def keep_mask(seed, keep_q15, n):
    """Keep decisions 0/1 of n blocks (Eq. (7)); block i is kept with probability keep_q15 / 32768."""
    m = np.empty(n, dtype=np.float32)
    lib().xo_keep_mask(int(seed), int(keep_q15), n, m.ctypes.data_as(_c_f32p))
    return m


def pixel_probe_matrix(dist, seed, C_in, H, W, r, dtype=F32, keep_q15=0):
    """Z [C_in*H*W, r], row (n, q) = n*H*W + q, from the same generator as the channel probes
    (entry index = row * r + j), rounded to the storage type the products run in.  keep_q15 != 0:
    block-sparse probing vectors (Eq. (7)): block (n, j), the N entries of vector j on channel n, is
    zero unless keep decision n*r + j says keep."""
    Z = np.ascontiguousarray(probe_matrix(dist, seed, C_in * H * W, r), dtype=np.float32)
    if dtype != F32:
        lib().xo_round_array(Z.ctypes.data_as(_c_f32p), Z.size, dtype)
    if keep_q15:
        keep = keep_mask(seed, keep_q15, C_in * r).reshape(C_in, 1, r)
        Z = np.ascontiguousarray((Z.reshape(C_in, H * W, r) * keep).reshape(C_in * H * W, r))
    return Z


def pixel_block_counts(Z, C_in):
    """nnz(Z_n) of Eq. (8): the number of probing vectors with a non-zero block on channel n."""
    Zb = np.asarray(Z).reshape(C_in, -1, Z.shape[1])
    return np.count_nonzero(np.any(Zb != 0, axis=1), axis=1)


def pixel_probe_fwd(X, Z):
    """Xbar [B, r] = Z^T X over the stacked pixel x channel axis (Alg. 1 forward step 3), fp32."""
    X, Xp = _f32(X)
    Z, Zp = _f32(Z)
    B, C_in, H, W = X.shape
    r = Z.shape[1]
    assert Z.shape[0] == C_in * H * W
    Xbar = np.empty((B, r), dtype=np.float32)
    lib().xo_pixel_probe_fwd(Xp, Zp, Xbar.ctypes.data_as(_c_f32p), B, C_in, H, W, r)
    return Xbar


def pixel_dw_estimate(dY, Xbar, Z, C_in, H, W, kH, kW, stride=(1, 1), pad=(0, 0), nnz_norm=False):
    """dw_i = (1/r) tr(L T_{-k(i)} Z), L = Xbar^T dY (Alg. 1 backward steps 3 and 4; nothing but the saved Xbar is rounded).
    nnz_norm: the estimate of input channel n is scaled by 1 / nnz(Z_n) instead of 1 / r (Eq. (8)); a channel
    without any block gives zeros."""
    dY, dYp = _f32(dY)
    Xbar, Xbp = _f32(Xbar)
    Z, Zp = _f32(Z)
    B, C_out, Ho, Wo = dY.shape
    r = Z.shape[1]
    assert Xbar.shape == (B, r) and Z.shape[0] == C_in * H * W
    assert Ho == out_extent(H, kH, stride[0], pad[0]) and Wo == out_extent(W, kW, stride[1], pad[1])
    dW = np.empty((C_out, C_in, kH, kW), dtype=np.float64)
    lib().xo_pixel_dw_estimate(dYp, Xbp, Zp, dW.ctypes.data_as(_c_f64p), B, C_in, C_out, H, W, r,
                               kH, kW, stride[0], stride[1], pad[0], pad[1])
    if nnz_norm:
        nnz = pixel_block_counts(Z, C_in)
        dW *= np.where(nnz > 0, r / np.maximum(nnz, 1), 0.0).reshape(1, C_in, 1, 1)
    return dW


def pixel_indep_probe_fwd(X, Z):
    """Independent probing (Sec. 3, the per-channel alternative to Eq. (6)): every input channel n is
    probed on its own with Z_n [H*W, r], the rows of channel n of Z [C_in*H*W, r].  Xbar [B, C_in, r]:
    channel n is the single-channel forward product of X[:, n] with Z_n."""
    X = np.asarray(X, dtype=np.float32)
    Z = np.asarray(Z, dtype=np.float32)
    B, C_in, H, W = X.shape
    N = H * W
    assert Z.shape[0] == C_in * N
    Xbar = np.empty((B, C_in, Z.shape[1]), dtype=np.float32)
    for n in range(C_in):
        Xbar[:, n, :] = pixel_probe_fwd(X[:, n:n + 1], Z[n * N:(n + 1) * N])
    return Xbar


def pixel_indep_dw_estimate(dY, Xbar, Z, C_in, H, W, kH, kW, stride=(1, 1), pad=(0, 0)):
    """Independent probing, backward: the trace estimate of every (input, output) channel pair uses the
    probes of its own input channel only, so column n of dW is the single-channel estimate (Alg. 1
    backward with C_in = 1) from Xbar[:, n] and Z_n; no term mixes two input channels."""
    Xbar = np.asarray(Xbar, dtype=np.float32)
    Z = np.asarray(Z, dtype=np.float32)
    N = H * W
    C_out = np.asarray(dY).shape[1]
    assert Xbar.shape[1] == C_in and Z.shape[0] == C_in * N
    dW = np.empty((C_out, C_in, kH, kW), dtype=np.float64)
    for n in range(C_in):
        dW[:, n:n + 1] = pixel_dw_estimate(dY, Xbar[:, n, :], Z[n * N:(n + 1) * N], 1, H, W, kH, kW, stride, pad)
    return dW


def relu_sign_fwd(X):
    """ReLU that keeps only the signs of its input for the backward pass (Sec. 5, "Overall effective memory
    savings": layers that relied on the convolution to store their state): Y = max(X, 0) and one bit per
    element, bit i%64 of 64-bit word i//64 set iff element i (row-major) is positive."""
    X = np.asarray(X)
    pos = (X.reshape(-1) > 0)
    n = pos.size
    padded = np.zeros((n + 63) // 64 * 64, dtype=np.uint8)
    padded[:n] = pos
    words = np.packbits(padded.reshape(-1, 64), axis=1, bitorder="little").view("<u8").reshape(-1)
    return np.maximum(X, 0), words


def relu_sign_bwd(dY, words):
    """dX = dY where the stored sign bit is set, else 0."""
    dY = np.asarray(dY)
    bits = np.unpackbits(np.ascontiguousarray(words, dtype="<u8").view(np.uint8), bitorder="little")[:dY.size]
    return np.where(bits.reshape(dY.shape) != 0, dY, 0).astype(dY.dtype)
