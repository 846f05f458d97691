"""GPU parity of the forward convolution and the exact input gradient (xconv_conv_fwd, xconv_dx_exact) against the
oracle (xo.conv_fwd, xo.dx) on identical seeded inputs: element by element on layers with ragged channel and pixel
tiles, strides 1..3, paddings 0..2, 1x1 to 5x5 kernels, both layouts and the three storage types; the benchmark layers
C1 and C2 at full size, C5 on sampled images.  Tolerance: fp32 sums against fp64 sums, one rounding to the storage type
(the gradients' bar: 1e-4 of the largest value for fp32; for 16-bit storage one unit in the last place of the result,
2^-8 / 2^-11 relative, plus the fp32 summation error)."""
import numpy as np
import pytest
import torch

from oracle import xconv_oracle as xo
from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TD = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def say(msg):
    print("[gpu-case] " + msg, flush=True)


def check(got, want, dtype):
    scale = np.max(np.abs(want))
    if dtype == "f32":
        assert np.max(np.abs(got - want)) <= 1e-4 * scale, np.max(np.abs(got - want)) / scale
    else:
        ulp = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}[dtype]
        tol = 1.01 * ulp * np.abs(want) + 1e-4 * scale        # one rounding of a sum that is off by the fp32 summation error
        bad = np.abs(got - want) > tol
        assert not bad.any(), (int(bad.sum()), float(np.max(np.abs(got - want)) / scale))


def run_case(B, C_in, C_out, H, W, k, stride, pad, dtype, nhwc=False, seed=900, images=None):
    kH, kW = (k, k) if isinstance(k, int) else k
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    say("conv fwd + dX: B%d C%d->%d %dx%d k%dx%d s%d,%d p%d,%d %s %s" % (B, C_in, C_out, H, W, kH, kW, sh, sw, ph, pw, dtype, "NHWC" if nhwc else "NCHW"))
    Ho, Wo = xo.out_extent(H, kH, sh, ph), xo.out_extent(W, kW, sw, pw)
    X = synth.draw((B, C_in, H, W), seed, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, Ho, Wo), seed + 1, "normal", 1e-2, dtype)
    Wt = synth.draw((C_out, C_in, kH, kW), seed + 2, "normal", 1.0 / (C_in * kH * kW), dtype)
    d = xb.make_desc(B, C_in, C_out, H, W, (kH, kW), (sh, sw), (ph, pw), 1, dtype, "rademacher", 1,
                     layout=xb.XCONV_NHWC if nhwc else xb.XCONV_NCHW)
    perm, back = ((0, 2, 3, 1), (0, 3, 1, 2)) if nhwc else ((0, 1, 2, 3), (0, 1, 2, 3))
    Xd = xb.to_device(np.ascontiguousarray(X.transpose(perm)), dtype, DEV)
    dYd = xb.to_device(np.ascontiguousarray(dY.transpose(perm)), dtype, DEV)
    Wd = xb.to_device(Wt, dtype, DEV)
    Y = torch.full(tuple(np.array((B, C_out, Ho, Wo))[list(perm)]), float("nan"), dtype=TD[dtype], device=DEV)
    dX = torch.full(tuple(np.array((B, C_in, H, W))[list(perm)]), float("nan"), dtype=TD[dtype], device=DEV)
    xb.xconv_conv_fwd(d, Xd, Wd, Y)
    xb.xconv_dx_exact(d, dYd, Wd, dX)
    torch.cuda.synchronize()
    Yg = Y.float().cpu().numpy().transpose(back).astype(np.float64)
    dXg = dX.float().cpu().numpy().transpose(back).astype(np.float64)
    assert np.all(np.isfinite(Yg)) and np.all(np.isfinite(dXg))
    sel = slice(None) if images is None else images
    check(Yg[sel], xo.conv_fwd(X[sel], Wt.astype(np.float64), (sh, sw), (ph, pw)), dtype)
    check(dXg[sel], xo.dx(dY[sel], Wt.astype(np.float64), H, W, (sh, sw), (ph, pw)), dtype)


CASES = [
    # B, C_in, C_out, H, W, k, stride, pad, dtype
    (2, 3, 5, 7, 9, 3, 1, 1, "f32"),
    (3, 20, 40, 12, 13, 3, 1, 1, "f32"),
    (2, 17, 70, 11, 10, 3, 2, 1, "f32"),
    (2, 33, 130, 9, 9, 1, 1, 0, "f32"),
    (1, 8, 8, 16, 16, 5, 1, 2, "f32"),
    (2, 12, 24, 15, 14, (3, 2), (2, 3), (1, 0), "f32"),
    (3, 40, 36, 12, 12, 3, 1, 1, "f16"),
    (2, 70, 33, 13, 9, 3, 2, 1, "bf16"),
    (2, 6, 150, 8, 8, 3, 3, 2, "f16"),
    (1, 64, 64, 10, 10, 1, 2, 0, "bf16"),
    (2, 31, 31, 9, 11, (2, 4), 1, (1, 2), "f16"),
]


@pytest.mark.parametrize("case", CASES, ids=["%s-c%d-%d-k%s-s%s" % (c[8], c[1], c[2], c[5], c[6]) for c in CASES])
@pytest.mark.parametrize("nhwc", [False, True], ids=["nchw", "nhwc"])
def test_conv_fwd_and_dx_against_the_oracle(case, nhwc):
    run_case(*case, nhwc=nhwc)


def test_conv_fwd_and_dx_on_the_benchmark_layers():
    for name, images in (("C1", None), ("C2", slice(0, 8)), ("C5", slice(250, 252))):
        cfg = synth.CONFIGS[name]
        run_case(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.k, cfg.stride, cfg.pad, cfg.dtype, seed=cfg.seeds[0], images=images)


def test_conv_entry_points_reject_bad_arguments():
    d = xb.make_desc(2, 4, 4, 8, 8, 3, 1, 1, 1, "f32", "rademacher", 1)
    t = torch.zeros(1024, dtype=torch.float32, device=DEV)
    L = xb.lib()
    assert L.xconv_conv_fwd(xb.ctypes.byref(d), None, t.data_ptr(), t.data_ptr(), None) == xb.XCONV_EINVAL
    assert L.xconv_dx_exact(xb.ctypes.byref(d), t.data_ptr(), None, t.data_ptr(), None) == xb.XCONV_EINVAL
    assert L.xconv_conv_fwd(xb.ctypes.byref(d), t.data_ptr() + 2, t.data_ptr(), t.data_ptr(), None) == xb.XCONV_EINVAL
    d.H = 0
    assert L.xconv_conv_fwd(xb.ctypes.byref(d), t.data_ptr(), t.data_ptr(), t.data_ptr(), None) == xb.XCONV_EINVAL
