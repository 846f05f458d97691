"""xconv_dw_estimate_static, the entry point for callers that cannot allocate device memory: through the C ABI its
output equals xconv_dw_estimate's bit for bit, on two calls in a row (the second on a smaller layer, so that what the
first call left in the library's scratch array lies beyond what the second one writes), and a layer whose scratch
exceeds the array is refused before anything is launched."""
import numpy as np
import pytest
import torch

from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layer(B, C_in, C_out, H, W, r, dtype, seed):
    d = xb.make_desc(B, C_in, C_out, H, W, 3, 1, 1, r, dtype, "rademacher", seed)
    X = synth.draw((B, C_in, H, W), seed + 1, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, H, W), seed + 2, "normal", 1e-2, dtype)
    Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    Xt = xb.alloc_xt(d, DEV)
    xb.xconv_probe_fwd(d, Xd, Xt, None, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))
    return d, dYd, Xt


def _both(d, dYd, Xt):
    shape = (d.C_out, d.C_in, 3, 3)
    want = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_estimate(d, dYd, Xt, None, want, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
    got = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_estimate_static(d, dYd, Xt, None, got)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_static_scratch_estimate_equals_the_workspace_one_twice_in_a_row(dtype):
    print("[gpu-case] xconv_dw_estimate_static %s: B=24 C=32->48 20x20 r=32, then B=5 C=16->24 12x12 r=8" % dtype, flush=True)
    big = _layer(24, 32, 48, 20, 20, 32, dtype, 501)
    small = _layer(5, 16, 24, 12, 12, 8 if dtype == "f32" else 32, dtype, 601)
    for layer in (big, small):
        assert 0 < xb.xconv_workspace_bytes(layer[0], xb.XCONV_OP_ESTIMATE) <= xb.xconv_static_scratch_bytes()
        got, want = _both(*layer)
        assert np.all(np.isfinite(want))
        assert np.array_equal(got, want)


def test_static_scratch_estimate_refuses_what_does_not_fit():
    d = xb.make_desc(64, 256, 512, 28, 28, 3, 1, 1, 256, "f16", "rademacher", 1)
    assert xb.xconv_workspace_bytes(d, xb.XCONV_OP_ESTIMATE) > xb.xconv_static_scratch_bytes()
    one = torch.zeros(64, dtype=torch.float32, device=DEV)
    st = xb.lib().xconv_dw_estimate_static(xb.ctypes.byref(d), one.data_ptr(), one.data_ptr(), None, one.data_ptr(), None)
    assert st == xb.XCONV_EWORKSPACE
