"""GPU parity of the estimator with probing vectors over pixels and channels (xconv_pixel_*)
against the CPU oracle: the stored projections Xbar to 1e-5 of their largest magnitude (an fp32
sum against the oracle's fp64 sum over C_in*H*W terms), the gradient to the tolerances of the
other parity tests (fp32 1e-4, 16-bit storage 2e-2 of the largest magnitude)."""
import numpy as np
import pytest
import torch

from oracle import xconv_oracle as xo
from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth
from test_gpu_parity import DEV, GRAD_TOL, ODT, OPROBE, rel_max, say

pytestmark = pytest.mark.gpu

# name, dtype, B, C_in, C_out, H, W, k, stride, pad, r, probe[, keep_q15]
PIX = [
    ("f32-3x3", "f32", 8, 8, 16, 16, 16, 3, 1, 1, 16, "gaussian"),
    ("f32-rademacher-r5", "f32", 6, 4, 8, 12, 12, 3, 1, 1, 5, "rademacher"),
    ("bf16-3x3", "bf16", 16, 16, 32, 12, 12, 3, 1, 1, 32, "rademacher"),
    ("f16-gaussian", "f16", 12, 8, 16, 10, 12, 3, 1, 1, 16, "gaussian"),
    ("f32-stride2-5x5", "f32", 5, 6, 10, 13, 11, 5, 2, 2, 8, "gaussian"),
    ("bf16-odd-planes", "bf16", 9, 5, 7, 7, 9, 3, 1, 0, 12, "rademacher"),
    ("f16-1x1", "f16", 4, 16, 16, 8, 8, 1, 1, 0, 16, "rademacher"),
    ("f32-one-image", "f32", 1, 4, 4, 8, 8, 3, 1, 1, 4, "rademacher"),
    ("f16-image-and-vector-blocks", "f16", 300, 4, 8, 8, 8, 3, 1, 1, 80, "rademacher"),
    ("f32-ragged-blocks", "f32", 70, 4, 4, 8, 12, 3, 1, 1, 20, "gaussian"),
    ("bf16-batch-520", "bf16", 520, 2, 4, 8, 8, 3, 1, 1, 8, "rademacher"),
    ("f32-block-sparse", "f32", 8, 8, 16, 16, 16, 3, 1, 1, 16, "gaussian", 16384),
    ("bf16-block-sparse", "bf16", 16, 16, 32, 12, 12, 3, 1, 1, 32, "rademacher", 12000),
    ("f16-block-sparse-empty-channels", "f16", 6, 12, 8, 8, 8, 3, 1, 1, 2, "rademacher", 9000),
    ("f32-batch-40", "f32", 40, 8, 8, 8, 8, 3, 1, 1, 64, "rademacher"),
]


def run_pixel(e, nhwc=False):
    name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = e[:12]
    keep = e[12] if len(e) > 12 else 0
    say("pixel probe %s%s" % (e, " channels-last" if nhwc else ""))
    cfg = synth.LayerConfig(name=name, B=B, C_in=C_in, C_out=C_out, H=H, W=W, k=k, stride=st, pad=pad, r=r, dtype=dtype,
                            probe=probe, x_dist="relu_normal", dy_var=1e-2, seeds=(8101 + len(name), 8202 + len(name), 8303 + len(name)))
    X, dY = synth.make_layer(cfg)
    d = xb.desc_from_config(cfg)
    d.keep_q15 = keep
    if nhwc:
        d.layout = xb.XCONV_NHWC
    Z = xo.pixel_probe_matrix(OPROBE[probe], cfg.seeds[2], C_in, H, W, r, ODT[dtype], keep)
    if name.endswith("empty-channels"):
        assert (xo.pixel_block_counts(Z, C_in) == 0).any()      # some channel has no block: its estimate is zero
    want_xbar = xo.pixel_probe_fwd(X, Z)
    if nhwc:   # the same values handed over as [B, H, W, C]
        Xd = xb.to_device(np.ascontiguousarray(X.transpose(0, 2, 3, 1)), dtype, DEV)
        dYd = xb.to_device(np.ascontiguousarray(dY.transpose(0, 2, 3, 1)), dtype, DEV)
    else:
        Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    assert xb.xconv_pixel_xbar_bytes(d) == B * r * 4
    xbar = torch.full((B, r), float("nan"), dtype=torch.float32, device=DEV)
    ws = xb.alloc_bytes(xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_PROBE), DEV)
    ws.fill_(0x7f)
    xb.xconv_pixel_probe_fwd(d, Xd, xbar, ws)
    torch.cuda.synchronize()
    got_xbar = xbar.cpu().numpy()
    assert np.max(np.abs(got_xbar - want_xbar)) <= 1e-5 * np.max(np.abs(want_xbar)), rel_max(got_xbar, want_xbar)
    # backward from the oracle's projections, so that both sides start from the same stored state
    want = xo.pixel_dw_estimate(dY, want_xbar, Z, C_in, H, W, k, k, (st, st), (pad, pad), nnz_norm=keep != 0)
    dW = torch.full((C_out, C_in, k, k), float("nan"), dtype=torch.float32, device=DEV)
    ws2 = xb.alloc_bytes(xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), DEV)
    ws2.fill_(0x7f)
    xb.xconv_pixel_dw_estimate(d, dYd, torch.from_numpy(want_xbar).to(DEV), dW, ws2)
    torch.cuda.synchronize()
    got = dW.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    err = rel_max(got, want)
    assert err <= GRAD_TOL[dtype], err
    # and end to end, from the projections the library stored
    xb.xconv_pixel_dw_estimate(d, dYd, xbar, dW, ws2)
    torch.cuda.synchronize()
    assert rel_max(dW.cpu().numpy().astype(np.float64), want) <= GRAD_TOL[dtype]
    return got


@pytest.mark.parametrize("e", PIX, ids=[e[0] for e in PIX])
def test_pixel_probe_layers(e):
    run_pixel(e)


NHWC_PIX = [PIX[0], PIX[2], PIX[3], PIX[4], PIX[5], PIX[6], PIX[9], PIX[12]]


@pytest.mark.parametrize("e", NHWC_PIX, ids=[e[0] for e in NHWC_PIX])
def test_pixel_probe_channels_last(e):
    # the oracle's NCHW result: the estimator does not depend on the order the tensors are stored in
    run_pixel(e, nhwc=True)


def test_pixel_probe_is_deterministic():
    assert np.array_equal(run_pixel(PIX[2]), run_pixel(PIX[2]))


def test_pixel_probe_full_size_C2():
    # the benchmark layer bench.py --pixel-probe times by default, every entry against the oracle
    cfg = synth.CONFIGS["C2"]
    run_pixel(("C2", cfg.dtype, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.probe))


def test_pixel_probe_full_size_C5():
    # the largest 16-bit benchmark layer (K = 200704 values per image, r = 64, B = 256), every entry against the
    # oracle, which takes about half a minute for it
    cfg = synth.CONFIGS["C5"]
    run_pixel(("C5", cfg.dtype, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.probe))

