"""GPU parity of independent probing (xconv_pixel_indep_*: every input channel with probing
vectors of its own) against the CPU oracle, to the tolerances of the other pixel-probe tests:
the stored projections to 1e-5 of their largest magnitude, the gradient to 1e-4 (fp32) and 2e-2
(16-bit storage) of its largest magnitude."""
import numpy as np
import pytest
import torch

from oracle import xconv_oracle as xo
from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth
from test_gpu_parity import DEV, GRAD_TOL, ODT, OPROBE, rel_max, say

pytestmark = pytest.mark.gpu

# name, dtype, B, C_in, C_out, H, W, k, stride, pad, r, probe
IND = [
    ("f32-3x3", "f32", 8, 8, 16, 16, 16, 3, 1, 1, 8, "gaussian"),
    ("bf16-3x3", "bf16", 16, 16, 32, 12, 12, 3, 1, 1, 4, "rademacher"),
    ("f16-stride2-5x5", "f16", 6, 6, 10, 13, 11, 5, 2, 2, 8, "gaussian"),
    ("f32-ragged-vectors", "f32", 5, 3, 4, 7, 9, 3, 1, 0, 5, "rademacher"),
    ("f32-one-channel", "f32", 7, 1, 6, 12, 12, 3, 1, 1, 16, "gaussian"),
    ("f16-1024-vectors", "f16", 40, 32, 16, 8, 8, 3, 1, 1, 32, "rademacher"),
    ("bf16-1x1", "bf16", 12, 8, 8, 8, 8, 1, 1, 0, 16, "rademacher"),
    ("f32-2048-vectors", "f32", 6, 64, 8, 8, 8, 3, 1, 1, 32, "rademacher"),        # four groups of 16 channels
    ("f16-ragged-groups", "f16", 5, 40, 12, 8, 8, 3, 1, 1, 4, "gaussian"),         # groups of 16, 16 and 8 channels
    ("f32-wide-r-groups", "f32", 4, 20, 6, 6, 8, 3, 1, 1, 128, "rademacher"),       # r = 128: groups of 8, 8 and 4 channels
    ("bf16-one-channel-groups", "bf16", 3, 3, 4, 8, 8, 3, 1, 1, 1024, "rademacher"),  # r = 1024: one channel per pass
    ("f16-few-vectors-wide-groups", "f16", 4, 80, 8, 8, 8, 3, 1, 1, 4, "rademacher"),  # r = 4: groups of 64 and 16 channels
    ("f32-two-vectors", "f32", 3, 150, 6, 6, 6, 3, 1, 1, 2, "gaussian"),               # r = 2: groups of 128 and 22 channels
]


def setup(e):
    name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = e
    cfg = synth.LayerConfig(name=name, B=B, C_in=C_in, C_out=C_out, H=H, W=W, k=k, stride=st, pad=pad, r=r, dtype=dtype,
                            probe=probe, x_dist="relu_normal", dy_var=1e-2, seeds=(9101 + len(name), 9202 + len(name), 9303 + len(name)))
    X, dY = synth.make_layer(cfg)
    d = xb.desc_from_config(cfg)
    Z = xo.pixel_probe_matrix(OPROBE[probe], cfg.seeds[2], C_in, H, W, r, ODT[dtype])
    return cfg, d, X, dY, Z


def gpu_fwd(d, Xd, B, C_in, r):
    assert xb.xconv_pixel_indep_xbar_bytes(d) == B * C_in * r * 4
    xbar = torch.full((B, C_in, r), float("nan"), dtype=torch.float32, device=DEV)
    ws = xb.alloc_bytes(xb.xconv_pixel_indep_workspace_bytes(d, xb.XCONV_OP_PROBE), DEV)
    ws.fill_(0x7f)
    xb.xconv_pixel_indep_probe_fwd(d, Xd, xbar, ws)
    torch.cuda.synchronize()
    return xbar


def gpu_bwd(d, dYd, xbar, shape):
    dW = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    ws = xb.alloc_bytes(xb.xconv_pixel_indep_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), DEV)
    ws.fill_(0x7f)
    xb.xconv_pixel_indep_dw_estimate(d, dYd, xbar, dW, ws)
    torch.cuda.synchronize()
    return dW.cpu().numpy().astype(np.float64)


def run_indep(e, nhwc=False):
    name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = e
    say("independent probing %s%s" % (e, " channels-last" if nhwc else ""))
    cfg, d, X, dY, Z = setup(e)
    want_xbar = xo.pixel_indep_probe_fwd(X, Z)
    if nhwc:   # the same values handed over as [B, H, W, C]
        d.layout = xb.XCONV_NHWC
        Xd = xb.to_device(np.ascontiguousarray(X.transpose(0, 2, 3, 1)), dtype, DEV)
        dYd = xb.to_device(np.ascontiguousarray(dY.transpose(0, 2, 3, 1)), dtype, DEV)
    else:
        Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    xbar = gpu_fwd(d, Xd, B, C_in, r)
    got_xbar = xbar.cpu().numpy()
    assert np.max(np.abs(got_xbar - want_xbar)) <= 1e-5 * np.max(np.abs(want_xbar)), rel_max(got_xbar, want_xbar)
    # backward from the oracle's projections, so that both sides start from the same stored state
    want = xo.pixel_indep_dw_estimate(dY, want_xbar, Z, C_in, H, W, k, k, (st, st), (pad, pad))
    got = gpu_bwd(d, dYd, torch.from_numpy(want_xbar).to(DEV), (C_out, C_in, k, k))
    assert np.all(np.isfinite(got))
    err = rel_max(got, want)
    assert err <= GRAD_TOL[dtype], err
    # and end to end, from the projections the library stored
    assert rel_max(gpu_bwd(d, dYd, xbar, (C_out, C_in, k, k)), want) <= GRAD_TOL[dtype]
    return got


@pytest.mark.parametrize("e", IND, ids=[e[0] for e in IND])
def test_independent_probing_layers(e):
    run_indep(e)


@pytest.mark.parametrize("e", [IND[0], IND[1], IND[2], IND[3], IND[8]], ids=[e[0] for e in IND[:4]] + [IND[8][0]])
def test_independent_probing_channels_last(e):
    run_indep(e, nhwc=True)


def test_independent_probing_is_deterministic():
    assert np.array_equal(run_indep(IND[1]), run_indep(IND[1]))


def test_independent_state_sums_to_the_multi_channel_state_and_one_channel_is_the_same_estimator():
    e = IND[0]
    name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = e
    say("independent vs multi-channel %s" % (e,))
    cfg, d, X, dY, Z = setup(e)
    Xd = xb.to_device(X, dtype, DEV)
    ind = gpu_fwd(d, Xd, B, C_in, r).cpu().numpy().astype(np.float64)
    sim = torch.empty((B, r), dtype=torch.float32, device=DEV)
    xb.xconv_pixel_probe_fwd(d, Xd, sim, xb.alloc_bytes(xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_PROBE), DEV))
    torch.cuda.synchronize()
    sim = sim.cpu().numpy()
    assert np.max(np.abs(ind.sum(axis=1) - sim)) <= 2e-5 * np.max(np.abs(sim))
    # with a single input channel the two modes are one estimator
    e1 = IND[4]
    cfg, d, X, dY, Z = setup(e1)
    Xd, dYd = xb.to_device(X, "f32", DEV), xb.to_device(dY, "f32", DEV)
    xbar = gpu_fwd(d, Xd, e1[2], 1, e1[10])
    a = gpu_bwd(d, dYd, xbar, (e1[4], 1, 3, 3))
    dW = torch.empty((e1[4], 1, 3, 3), dtype=torch.float32, device=DEV)
    xb.xconv_pixel_dw_estimate(d, dYd, xbar.reshape(e1[2], e1[10]).contiguous(), dW,
                               xb.alloc_bytes(xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), DEV))
    torch.cuda.synchronize()
    assert np.array_equal(a, dW.cpu().numpy().astype(np.float64))


def test_independent_probing_has_no_crosstalk():
    # an input that lives on one channel gives exact zeros on every other channel's gradient
    e = IND[0]
    name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = e
    say("independent probing, single live channel %s" % (e,))
    cfg, d, X, dY, Z = setup(e)
    X[:, 1:] = 0
    Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    got = gpu_bwd(d, dYd, gpu_fwd(d, Xd, B, C_in, r), (C_out, C_in, k, k))
    assert np.all(got[:, 1:] == 0) and np.any(got[:, 0] != 0)
    want = xo.pixel_indep_dw_estimate(dY, xo.pixel_indep_probe_fwd(X, Z), Z, C_in, H, W, k, k, (st, st), (pad, pad))
    assert rel_max(got, want) <= GRAD_TOL[dtype]


def test_independent_probing_full_size_C2():
    # the layer bench.py --pixel-probe --independent times by default (64 channels x 16 vectors, four passes over groups of 16 channels),
    # every entry against the oracle
    cfg = synth.CONFIGS["C2"]
    run_indep(("C2", cfg.dtype, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.probe))

