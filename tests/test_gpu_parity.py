"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on identical seeded inputs and the same Z.

Tolerances (relative to the largest magnitude of the oracle's result):
fp32 storage 1e-4, bf16/fp16 storage 2e-2 for the gradients.  The stored probe
output is compared element by element: fp32 to 2e-6 of the largest value,
16-bit storage to one unit in the last place of the storage type (the oracle
rounds the exact sum once, the kernel rounds an fp32 sum once).
"""
import sys

import numpy as np
import pytest
import torch

from oracle import xconv_oracle as xo
from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ODT = {"f32": xo.F32, "bf16": xo.BF16, "f16": xo.F16}
OPROBE = {"rademacher": xo.RADEMACHER, "gaussian": xo.GAUSSIAN}
GRAD_TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2e-2}
ULP = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}     # half a unit in the last place, relative


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def rel_max(got, want):
    return float(np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-300))


def run_probe(cfg, X, Z=None, seed_path=False):
    """Returns (Xt buffer, unpacked Xt as numpy [B,r,H,W])."""
    d = xb.desc_from_config(cfg)
    Xd = xb.to_device(X, cfg.dtype, DEV)
    Xt = xb.alloc_xt(d, DEV)
    Xt.fill_(0x7f)                                  # poison: every byte must be overwritten
    if seed_path:
        ws = xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV)
        xb.xconv_probe_fwd(d, Xd, Xt, None, ws)
    else:
        Zd = torch.from_numpy(np.ascontiguousarray(Z, dtype=np.float32)).to(DEV)
        xb.xconv_probe_fwd(d, Xd, Xt, Zd, None)
        # the same Z through the scratch-backed route (fragments packed once per call)
        Xt2 = xb.alloc_xt(d, DEV)
        Xt2.fill_(0x7f)
        xb.xconv_probe_fwd(d, Xd, Xt2, Zd, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))
        assert torch.equal(Xt, Xt2)
    out = torch.empty((cfg.B, cfg.r, cfg.H, cfg.W), dtype=torch.float32, device=DEV)
    xb.xconv_xt_unpack(d, Xt, out)
    torch.cuda.synchronize()
    return d, Xt, out.cpu().numpy()


def run_estimate(cfg, d, dY, Xt, Z=None):
    dYd = xb.to_device(dY, cfg.dtype, DEV)
    ws = xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV)
    dW = torch.full((cfg.C_out, cfg.C_in, cfg.k, cfg.k), float("nan"), dtype=torch.float32, device=DEV)
    Zd = None if Z is None else torch.from_numpy(np.ascontiguousarray(Z, dtype=np.float32)).to(DEV)
    xb.xconv_dw_estimate(d, dYd, Xt, Zd, dW, ws)
    torch.cuda.synchronize()
    return dW.cpu().numpy().astype(np.float64)


def run_exact(cfg, d, dY, X):
    dYd = xb.to_device(dY, cfg.dtype, DEV)
    Xd = xb.to_device(X, cfg.dtype, DEV)
    ws = xb.alloc_ws(d, xb.XCONV_OP_EXACT, DEV)
    dW = torch.full((cfg.C_out, cfg.C_in, cfg.k, cfg.k), float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_exact(d, dYd, Xd, dW, ws)
    torch.cuda.synchronize()
    return dW.cpu().numpy().astype(np.float64)


def check_probe_output(cfg, got, want, z_exact=True):
    assert got.shape == want.shape
    scale = np.max(np.abs(want))
    if cfg.dtype == "f32":
        assert np.max(np.abs(got - want)) <= 2e-6 * scale, rel_max(got, want)
    else:
        # One rounding each of sums that differ by the fp32 accumulation error: allow a unit in the
        # last place.  A Z that is not representable in the storage type enters the 16-bit MFMA as
        # hi + lo, which for bf16 leaves 2^-16 of each product; sums that cancel to almost nothing
        # can then be off by more than their own last place, hence the larger absolute floor.
        floor = 1e-6 if (z_exact or cfg.dtype == "f16") else 1e-4
        tol = 2.0 * ULP[cfg.dtype] * np.maximum(np.abs(want), 2.0 ** -14) + floor * scale
        bad = np.abs(got - want) > tol
        assert not bad.any(), (int(bad.sum()), float(np.max((np.abs(got - want) - tol)[bad])), rel_max(got, want))
        assert np.mean(got == want) > 0.97


def full_parity(cfg, seed_path=False, check_exact=True):
    say("%s %s B%d C%d->%d %dx%d k%d s%d p%d r%d %s seed_path=%s" % (
        cfg.name, cfg.dtype, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.probe, seed_path))
    X, dY = synth.make_layer(cfg)
    Z = xo.probe_matrix(OPROBE[cfg.probe], cfg.seeds[2], cfg.C_in, cfg.r)
    st, pd = (cfg.stride, cfg.stride), (cfg.pad, cfg.pad)
    Xt_o = xo.probe_fwd(X, Z, ODT[cfg.dtype])
    d, Xt, Xt_g = run_probe(cfg, X, Z, seed_path)
    check_probe_output(cfg, Xt_g, Xt_o, z_exact=(cfg.probe == "rademacher"))
    want = xo.dw_from_xt(dY, Xt_o, Z, cfg.k, cfg.k, st, pd)
    got = run_estimate(cfg, d, dY, Xt, None if seed_path else Z)
    assert np.all(np.isfinite(got))
    err = rel_max(got, want)
    assert err <= GRAD_TOL[cfg.dtype], err
    if check_exact:
        want_x = xo.dw_exact(dY, X, cfg.k, cfg.k, st, pd)
        got_x = run_exact(cfg, d, dY, X)
        errx = rel_max(got_x, want_x)
        assert errx <= GRAD_TOL[cfg.dtype], errx
    return err


# ---------------------------------------------------------------------------
# generator on the device
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("probe", ["rademacher", "gaussian"])
def test_device_probe_matrix_matches_host_and_oracle(probe):
    for seed, C_in, r in ((3001, 16, 8), (3005, 256, 64), (77, 33, 5)):
        say("probe_matrix_dev %s seed=%d %dx%d" % (probe, seed, C_in, r))
        d = xb.make_desc(1, C_in, 1, 8, 8, 3, 1, 1, r, "f32", probe, seed)
        Zd = torch.empty((C_in, r), dtype=torch.float32, device=DEV)
        xb.xconv_probe_matrix_dev(d, Zd)
        torch.cuda.synchronize()
        Zg = Zd.cpu().numpy()
        Zh = xb.xconv_probe_matrix(d)
        Zo = xo.probe_matrix(OPROBE[probe], seed, C_in, r)
        if probe == "rademacher":
            assert np.array_equal(Zg, Zo) and np.array_equal(Zh, Zo)
        else:
            assert np.max(np.abs(Zg - Zo)) <= 2.4e-7 * np.max(np.abs(Zo))
            assert np.mean(Zg == Zo) > 0.98


# ---------------------------------------------------------------------------
# reduced copies of the five benchmark layers: several tiles and ragged tails
# ---------------------------------------------------------------------------
SMALL = [
    synth.CONFIGS["C1"],
    synth.small_variant(synth.CONFIGS["C2"], B=5, H=20, W=24, name="C2-small"),
    synth.small_variant(synth.CONFIGS["C3"], B=11, H=22, W=26, C_in=72, C_out=136, name="C3-small"),
    synth.small_variant(synth.CONFIGS["C4"], B=2, H=40, W=300, name="C4-small"),
    synth.small_variant(synth.CONFIGS["C5"], B=18, H=12, W=12, C_in=96, C_out=80, name="C5-small"),
]


@pytest.mark.parametrize("cfg", SMALL, ids=[c.name for c in SMALL])
def test_small_layers_explicit_z(cfg):
    full_parity(cfg, seed_path=False)


@pytest.mark.parametrize("cfg", [SMALL[1], SMALL[4]], ids=["C2-small", "C5-small"])
def test_small_layers_seed_path(cfg):
    # Z regenerated on the device from the seed in forward and backward (Algorithm 1)
    full_parity(cfg, seed_path=True, check_exact=False)


EDGE = [
    # name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype
    ("odd-plane-f32", 3, 5, 7, 9, 11, 3, 1, 1, 3, "gaussian", "f32"),          # planes not a multiple of the vector width
    ("odd-plane-f16", 9, 5, 7, 9, 11, 3, 1, 1, 3, "rademacher", "f16"),
    ("odd-plane-bf16", 3, 20, 18, 7, 9, 3, 2, 1, 20, "rademacher", "bf16"),
    ("k1-f32", 4, 24, 40, 12, 12, 1, 1, 0, 8, "gaussian", "f32"),
    ("k1-s2-f16", 8, 32, 32, 12, 12, 1, 2, 0, 16, "rademacher", "f16"),
    ("k5-f32", 2, 8, 20, 16, 16, 5, 1, 2, 4, "rademacher", "f32"),             # 25 offsets: three offset groups
    ("k5-bf16", 8, 16, 16, 12, 12, 5, 1, 2, 16, "rademacher", "bf16"),
    ("nopad-f32", 2, 16, 16, 14, 18, 3, 1, 0, 8, "gaussian", "f32"),
    ("rect-k-f16", 8, 16, 24, 13, 16, (3, 2), (2, 1), (1, 0), 8, "rademacher", "f16"),
    ("gauss-f16", 8, 64, 32, 8, 8, 3, 1, 1, 24, "gaussian", "f16"),            # Z not representable in 16 bits: hi+lo probe
    ("gauss-bf16", 16, 40, 32, 8, 8, 3, 1, 1, 48, "gaussian", "bf16"),
    ("r-wide-f32", 2, 96, 16, 8, 8, 3, 1, 1, 80, "rademacher", "f32"),         # r > 64: two probe column blocks
    ("r-wide-f16", 8, 96, 16, 8, 8, 3, 1, 1, 80, "rademacher", "f16"),
    ("b1-f16", 1, 16, 16, 8, 8, 3, 1, 1, 4, "rademacher", "f16"),              # a single image in a group of 8
    ("one-pixel-out", 2, 4, 4, 3, 3, 3, 1, 0, 2, "gaussian", "f32"),
    ("wide-f32", 1, 8, 8, 6, 700, 3, 1, 1, 4, "rademacher", "f32"),            # several column strips
    ("wide-f16", 8, 16, 16, 4, 260, 3, 1, 1, 16, "rademacher", "f16"),
    ("big-cout-f32", 1, 8, 300, 8, 8, 3, 1, 1, 8, "rademacher", "f32"),
    ("cin-512-f32", 2, 512, 16, 8, 8, 3, 1, 1, 64, "gaussian", "f32"),           # the probe's Z fragments fill its LDS budget (128 KB)
    ("cin-512-f16-split", 8, 512, 16, 8, 8, 3, 1, 1, 64, "gaussian", "f16"),
    ("cin-528-f16", 8, 528, 16, 8, 8, 3, 1, 1, 32, "rademacher", "f16"),         # one channel block more: the generic probe takes it
    ("r-1024-f16", 2, 1040, 16, 6, 6, 3, 1, 1, 1024, "rademacher", "f16"),       # the largest r the library takes
    ("r-1000-f32", 1, 1030, 8, 5, 5, 3, 1, 1, 1000, "gaussian", "f32"),
    ("batch-65541-f32", 65541, 8, 8, 4, 4, 3, 1, 1, 4, "rademacher", "f32"),     # more images than one grid extent holds
]


def _edge_cfg(e):
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = e
    return name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype


@pytest.mark.parametrize("e", EDGE, ids=[e[0] for e in EDGE])
def test_edge_shapes(e):
    run_edge(e)


# Shapes that the producer/consumer correlation kernel takes (16-bit storage, probe columns a
# multiple of 32, even output width): partial groups of 8 images, output channels that do not
# fill a 32-row tile, strides, paddings, 4 / 3 / 25 kernel offsets, column strips with a ragged
# last strip, several workgroup tiles along the probe columns, and a split of the reduction
# whose ranges cross from one group of images into the next.
WS_EDGE = [
    ("ws-partial-group-f16", 11, 16, 40, 12, 12, 3, 1, 1, 32, "rademacher", "f16"),
    ("ws-r64-bf16", 9, 24, 70, 10, 14, 3, 1, 1, 64, "rademacher", "bf16"),
    ("ws-stride2-bf16", 8, 16, 48, 14, 20, 3, 2, 1, 32, "rademacher", "bf16"),
    ("ws-k2x2-f16", 8, 16, 32, 9, 13, (2, 2), 1, 0, 32, "gaussian", "f16"),
    ("ws-k5-f16", 8, 16, 32, 12, 12, 5, 1, 2, 32, "rademacher", "f16"),
    ("ws-k1x3-f16", 16, 16, 64, 6, 16, (1, 3), 1, (0, 1), 64, "rademacher", "f16"),
    ("ws-strips-f16", 8, 16, 32, 4, 260, 3, 1, 1, 32, "rademacher", "f16"),
    ("ws-r128-f16", 8, 16, 32, 8, 8, 3, 1, 1, 128, "rademacher", "f16"),
    ("ws-pad2-s2-bf16", 8, 16, 32, 13, 17, 3, 2, 2, 32, "rademacher", "bf16"),
    ("ws-exact-cin64-f16", 8, 64, 32, 8, 8, 3, 1, 1, 16, "rademacher", "f16"),   # the exact gradient takes it (64 channels)
    ("ws-runs-f16", 40, 16, 32, 6, 6, 3, 1, 1, 32, "rademacher", "f16"),         # 4 ranges over 5 groups x 6 rows
]


@pytest.mark.parametrize("e", WS_EDGE, ids=[e[0] for e in WS_EDGE])
def test_producer_consumer_kernel_shapes(e, monkeypatch):
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = e
    d = xb.make_desc(B, C_in, C_out, H, W, k, stride, pad, r, dtype, probe, 13)
    monkeypatch.setenv("XCONV_CORR_ROW", "0")        # (the row-sweep kernel would take some of these shapes: see below)
    if name.startswith("ws-runs"):
        monkeypatch.setenv("XCONV_WS_SPLITS", "4")   # the overrides in force are part of the key of the plan cache
    op = xb.XCONV_OP_EXACT if name.startswith("ws-exact") else xb.XCONV_OP_ESTIMATE
    plan = xb.xconv_plan_info(d, op)
    assert plan["ws"] == 1, plan
    if name.startswith("ws-runs"):
        assert plan["S"] == 4 and plan["NS"] == 30, plan
    run_edge(e)


# Shapes that the row-sweep kernel takes (16-bit storage, 3x3 kernels at unit stride, output rows of 4..28 columns, a
# multiple of 4, probe columns a multiple of 32): rows of 2..16 k-steps in one or two sub-steps with every position
# the sliding window can have at the end of a row, partial groups of 8 images, output channels that do not fill a
# tile, paddings 0 and 2, two tiles along the probe columns, the exact gradient, and a split of the reduction whose
# ranges cross from one group of images into the next.
ROW_EDGE = [
    ("row-w4-f16", 8, 16, 32, 6, 4, 3, 1, 1, 32, "rademacher", "f16"),
    ("row-w8-nopad-f16", 8, 16, 32, 10, 10, 3, 1, 0, 32, "gaussian", "f16"),
    ("row-w12-partial-group-f16", 11, 16, 40, 12, 12, 3, 1, 1, 32, "rademacher", "f16"),
    ("row-w12-pad2-bf16", 8, 16, 32, 8, 10, 3, 1, 2, 32, "rademacher", "bf16"),
    ("row-w16-r64-bf16", 9, 24, 70, 10, 16, 3, 1, 1, 64, "rademacher", "bf16"),
    ("row-w20-f16", 8, 16, 64, 7, 20, 3, 1, 1, 64, "rademacher", "f16"),
    ("row-w24-bf16", 10, 16, 33, 9, 24, 3, 1, 1, 64, "gaussian", "bf16"),
    ("row-w28-f16", 16, 32, 96, 28, 28, 3, 1, 1, 64, "rademacher", "f16"),
    ("row-r128-f16", 8, 16, 32, 8, 8, 3, 1, 1, 128, "rademacher", "f16"),
    ("row-exact-cin64-f16", 8, 64, 32, 8, 8, 3, 1, 1, 16, "rademacher", "f16"),
    ("row-runs-f16", 40, 16, 32, 6, 8, 3, 1, 1, 32, "rademacher", "f16"),        # 4 ranges over 5 groups x 6 rows
    ("row-runs-two-tiles-bf16", 20, 16, 48, 5, 28, 3, 1, 1, 64, "rademacher", "bf16"),
]


@pytest.mark.parametrize("e", ROW_EDGE, ids=[e[0] for e in ROW_EDGE])
def test_row_sweep_kernel_shapes(e, monkeypatch):
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = e
    d = xb.make_desc(B, C_in, C_out, H, W, k, stride, pad, r, dtype, probe, 13)
    if "runs" in name:
        monkeypatch.setenv("XCONV_ROW_SPLITS", "4" if name == "row-runs-f16" else "3")
    op = xb.XCONV_OP_EXACT if name.startswith("row-exact") else xb.XCONV_OP_ESTIMATE
    plan = xb.xconv_plan_info(d, op)
    assert plan["ws"] == 3, plan
    if name == "row-runs-f16":
        assert plan["S"] == 4 and plan["NS"] == 30, plan
    run_edge(e)


# fp32 producer/consumer kernel: plans with one and with two workgroups per compute unit, strips
# with a narrower last strip, several image groups with a partial last one, strides, 5x5 (three
# offset groups), output channels beyond the tile, wide A (the exact path), several steps per
# workgroup across image-group boundaries.
WS32_EDGE = [
    ("ws32-b5-c24", 5, 24, 24, 16, 16, 3, 1, 1, 8, "rademacher", "f32"),
    ("ws32-strips", 3, 16, 40, 12, 40, 3, 1, 1, 16, "gaussian", "f32"),
    ("ws32-stride2", 6, 32, 48, 17, 15, 3, 2, 1, 16, "rademacher", "f32"),
    ("ws32-k5", 4, 16, 16, 12, 12, 5, 1, 2, 8, "gaussian", "f32"),
    ("ws32-r40", 9, 48, 72, 10, 12, 3, 1, 1, 40, "rademacher", "f32"),
    ("ws32-k1x3", 4, 16, 32, 9, 12, (1, 3), 1, (0, 1), 16, "rademacher", "f32"),
    ("ws32-k3-s3", 5, 16, 16, 24, 24, 3, 3, 0, 8, "rademacher", "f32"),
]


@pytest.mark.parametrize("e", WS32_EDGE, ids=[e[0] for e in WS32_EDGE])
@pytest.mark.parametrize("occ", ["1", "2"], ids=["one-wg-per-cu", "two-wg-per-cu"])
def test_fp32_producer_consumer_kernel_shapes(e, occ, monkeypatch):
    monkeypatch.setenv("XCONV_WS32_OCC", occ)
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = e
    d = xb.make_desc(B, C_in, C_out, H, W, k, stride, pad, r, dtype, probe, 13)
    assert xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)["ws"] == 2
    run_edge(e)


def test_fp32_producer_consumer_kernel_runs_across_image_groups(monkeypatch):
    # few workgroups: each walks through many steps, whole runs and image-group boundaries
    monkeypatch.setenv("XCONV_WS32_SPLITS", "3")
    run_edge(("ws32-runs", 11, 16, 16, 8, 8, 3, 1, 1, 8, "rademacher", "f32"))


def test_producer_consumer_kernel_is_deterministic():
    say("determinism, producer/consumer kernel")
    e = WS_EDGE[1]
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = e
    X = synth.draw((B, C_in, H, W), 31, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, H, W), 32, "normal", 1e-2, dtype)
    d = xb.make_desc(B, C_in, C_out, H, W, k, stride, pad, r, dtype, probe, 33)
    assert xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)["ws"] == 1
    _three_runs_agree(d, X, dY, dtype, C_out, C_in)


def test_row_sweep_kernel_is_deterministic():
    say("determinism, row-sweep kernel")
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = ROW_EDGE[7]
    X = synth.draw((B, C_in, H, W), 31, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, H, W), 32, "normal", 1e-2, dtype)
    d = xb.make_desc(B, C_in, C_out, H, W, k, stride, pad, r, dtype, probe, 33)
    assert xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)["ws"] == 3
    _three_runs_agree(d, X, dY, dtype, C_out, C_in)


def _three_runs_agree(d, X, dY, dtype, C_out, C_in):
    Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    Xt = xb.alloc_xt(d, DEV)
    xb.xconv_probe_fwd(d, Xd, Xt, None, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))
    outs = []
    for _ in range(3):
        dW = torch.full((C_out, C_in, 3, 3), float("nan"), dtype=torch.float32, device=DEV)
        xb.xconv_dw_estimate(d, dYd, Xt, None, dW, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
        torch.cuda.synchronize()
        outs.append(dW.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# The second pass (sum of the split partial tiles, then Z / r or 1/nnz, Alg. 1 backward step 4) runs as one launch on
# small layers and as two on large ones: both routes on the same layers, whatever their size.
@pytest.mark.parametrize("fused", ["0", "1"], ids=["two-launches", "one-launch"])
def test_second_pass_routes(fused, monkeypatch):
    monkeypatch.setenv("XCONV_FUSED_PASS2", fused)
    for e in (EDGE[0], WS_EDGE[1], ROW_EDGE[7], WS32_EDGE[4], ("c2-like", 16, 64, 64, 32, 32, 3, 1, 1, 16, "gaussian", "f32"),
              ("wide-cin-exact", 4, 300, 40, 8, 8, 3, 1, 1, 24, "rademacher", "f16")):
        run_edge(e)
    for e in SPARSE[:2]:
        test_block_sparse_probes(e, False)
        test_block_sparse_probes(e, True)


# Reference measurement of the benchmark (not part of the method): the launch runs, counts its operations as documented
# and leaves one finite value per wave.
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_matrix_rate_diagnostic_runs(dtype):
    say("mfma rate %s" % dtype)
    out = torch.full((xb.XCONV_DIAG_OUT_BYTES // 4,), float("nan"), dtype=torch.float32, device=DEV)
    flops = xb.xconv_diag_mfma_rate(dtype, 8, out)
    torch.cuda.synchronize()
    per = 2 * 32 * 32 * (2 if dtype == "f32" else 16)
    assert flops == 512 * 4 * 8 * 4 * per
    assert bool(torch.isfinite(out).all())


# The one-launch second pass gives a workgroup 1, 2 or 4 quads of output channels (chosen by the layer's size) and takes Z
# in blocks of rows: every width, a probe count that is not a multiple of 4 and more input channels than one block holds.
@pytest.mark.parametrize("quads", ["1", "2", "4"])
def test_second_pass_quad_widths(quads, monkeypatch):
    monkeypatch.setenv("XCONV_FUSED_PASS2", "1")
    monkeypatch.setenv("XCONV_PASS2_QW", quads)
    for e in (("p2-blocks", 3, 136, 24, 8, 8, 3, 1, 1, 250, "gaussian", "f32"),
              ("p2-odd-r", 5, 40, 72, 9, 12, 3, 1, 1, 13, "rademacher", "f32"),
              WS_EDGE[1], ROW_EDGE[7]):
        run_edge(e)
    for e in (SPARSE[1], SPARSE[4]):
        test_block_sparse_probes(e, False)
        test_block_sparse_probes(e, True)


# ---------------------------------------------------------------------------
# block-sparse probing vectors with the 1/nnz scaling (Eq. (7), Eq. (8))
# ---------------------------------------------------------------------------
SPARSE = [
    # name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype, keep_q15
    ("sp-f32-rad", 4, 24, 20, 14, 14, 3, 1, 1, 16, "rademacher", "f32", 16384),
    ("sp-f32-gauss", 3, 40, 64, 12, 10, 3, 1, 1, 20, "gaussian", "f32", 8192),
    ("sp-f16-rad-ws", 9, 64, 64, 14, 14, 3, 1, 1, 64, "rademacher", "f16", 12000),
    ("sp-bf16-gauss-s2", 8, 32, 48, 15, 15, 3, 2, 1, 32, "gaussian", "bf16", 20000),
    ("sp-f32-empty-rows", 2, 32, 16, 10, 10, 3, 1, 1, 4, "rademacher", "f32", 6000),   # some rows of Z are all zero
]


@pytest.mark.parametrize("e", SPARSE, ids=[e[0] for e in SPARSE])
@pytest.mark.parametrize("given_z", [False, True], ids=["seedZ", "givenZ"])
def test_block_sparse_probes(e, given_z):
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype, keep = e
    say("block-sparse probes %s, Z %s" % (name, "given" if given_z else "from the seed"))
    Ho, Wo = xo.out_extent(H, k, stride, pad), xo.out_extent(W, k, stride, pad)
    X = synth.draw((B, C_in, H, W), 51, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, Ho, Wo), 52, "normal", 1e-2, dtype)
    Z = xo.probe_matrix(OPROBE[probe], 53, C_in, r, keep)
    assert 0 < np.count_nonzero(Z) < Z.size
    d = xb.make_desc(B, C_in, C_out, H, W, k, stride, pad, r, dtype, probe, 53, keep_q15=keep)
    # the device generator drops the same entries
    Zg = torch.empty((C_in, r), dtype=torch.float32, device=DEV)
    xb.xconv_probe_matrix_dev(d, Zg)
    torch.cuda.synchronize()
    assert np.array_equal(Zg.cpu().numpy() == 0, Z == 0)
    assert np.max(np.abs(Zg.cpu().numpy() - Z)) <= 2.4e-7 * np.max(np.abs(Z))
    Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    Zd = torch.from_numpy(Z).to(DEV) if given_z else None
    if given_z:
        d.probe = xb.XCONV_USER_Z
    Xt = xb.alloc_xt(d, DEV)
    xb.xconv_probe_fwd(d, Xd, Xt, Zd, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))
    unp = torch.empty((B, r, H, W), dtype=torch.float32, device=DEV)
    xb.xconv_xt_unpack(d, Xt, unp)
    dW = torch.full((C_out, C_in, k, k), float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_estimate(d, dYd, Xt, Zd, dW, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
    torch.cuda.synchronize()

    class C:
        pass
    C.dtype = dtype
    Xt_o = xo.probe_fwd(X, Z, ODT[dtype])
    check_probe_output(C, unp.cpu().numpy(), Xt_o, z_exact=(probe == "rademacher"))
    want = xo.dw_from_xt(dY, Xt_o, Z, k, k, (stride, stride), (pad, pad), nnz_norm=True)
    got = dW.cpu().numpy().astype(np.float64)
    assert rel_max(got, want) <= GRAD_TOL[dtype]
    empty = np.count_nonzero(Z, axis=1) == 0
    assert np.all(got[:, empty] == 0.0)
    if name == "sp-f32-empty-rows":
        assert empty.any()


# Channels-last X and dY (layout NHWC): the probe reads X directly (fast path when C_in is a
# multiple of the 16-byte vector, any-shape kernel otherwise, tiles with a ragged tail of
# pixels), dY is brought into plane form first, the exact path takes X as it is when C_in is a
# multiple of 16 and pads the channels otherwise.  Same oracle, fed the NCHW arrays.
NHWC_EDGE = [
    ("nhwc-f32-c16", 3, 16, 24, 13, 11, 3, 1, 1, 8, "rademacher", "f32"),
    ("nhwc-f32-c40-gauss", 5, 40, 64, 10, 12, 3, 1, 1, 20, "gaussian", "f32"),
    ("nhwc-f32-c6-generic", 2, 6, 10, 9, 9, 3, 1, 1, 4, "rademacher", "f32"),
    ("nhwc-f32-s2", 4, 32, 32, 17, 16, 3, 2, 1, 16, "gaussian", "f32"),
    ("nhwc-bf16-c64-r64", 9, 64, 64, 14, 14, 3, 1, 1, 64, "rademacher", "bf16"),
    ("nhwc-f16-c72-r32", 8, 72, 96, 12, 12, 3, 1, 1, 32, "rademacher", "f16"),
    ("nhwc-f16-gauss-r24", 6, 48, 32, 11, 10, 3, 1, 1, 24, "gaussian", "f16"),
    ("nhwc-bf16-c12-generic", 3, 12, 16, 8, 8, 3, 1, 1, 8, "rademacher", "bf16"),
    ("nhwc-f16-k5-s2", 8, 32, 64, 15, 15, 5, 2, 2, 32, "rademacher", "f16"),
    ("nhwc-f16-1x1", 8, 32, 48, 9, 9, 1, 1, 0, 16, "rademacher", "f16"),
    ("nhwc-batch-65541-f16", 65541, 8, 8, 4, 4, 3, 1, 1, 4, "rademacher", "f16"),   # more images than one grid extent holds
    ("nhwc-batch-65541-f32-c6", 65541, 8, 6, 4, 4, 3, 1, 1, 4, "rademacher", "f32"),
]


@pytest.mark.parametrize("e", NHWC_EDGE, ids=[e[0] for e in NHWC_EDGE])
def test_channels_last_inputs(e):
    run_edge(e, nhwc=True)


def run_edge(e, nhwc=False):
    name, B, C_in, C_out, H, W, k, stride, pad, r, probe, dtype = e
    kH, kW = (k, k) if isinstance(k, int) else k
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    say("edge %s" % name)
    Ho, Wo = xo.out_extent(H, kH, sh, ph), xo.out_extent(W, kW, sw, pw)
    X = synth.draw((B, C_in, H, W), 11, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, Ho, Wo), 12, "normal", 1e-2, dtype)
    Z = xo.probe_matrix(OPROBE[probe], 13, C_in, r)
    d = xb.make_desc(B, C_in, C_out, H, W, (kH, kW), (sh, sw), (ph, pw), r, dtype, probe, 13,
                     layout=xb.XCONV_NHWC if nhwc else xb.XCONV_NCHW)
    if nhwc:
        Xd = xb.to_device(np.ascontiguousarray(X.transpose(0, 2, 3, 1)), dtype, DEV)
        dYd = xb.to_device(np.ascontiguousarray(dY.transpose(0, 2, 3, 1)), dtype, DEV)
    else:
        Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    Zd = torch.from_numpy(Z).to(DEV)
    Xt = xb.alloc_xt(d, DEV)
    Xt.fill_(0x7f)
    xb.xconv_probe_fwd(d, Xd, Xt, Zd, None)
    Xt2 = xb.alloc_xt(d, DEV)
    Xt2.fill_(0x7f)
    xb.xconv_probe_fwd(d, Xd, Xt2, Zd, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))   # Z packed into scratch first
    assert torch.equal(Xt, Xt2)
    unp = torch.empty((B, r, H, W), dtype=torch.float32, device=DEV)
    xb.xconv_xt_unpack(d, Xt, unp)
    dW = torch.full((C_out, C_in, kH, kW), float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_estimate(d, dYd, Xt, Zd, dW, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
    dWx = torch.full((C_out, C_in, kH, kW), float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_exact(d, dYd, Xd, dWx, xb.alloc_ws(d, xb.XCONV_OP_EXACT, DEV))
    torch.cuda.synchronize()

    class C:  # minimal stand-in for check_probe_output
        pass
    C.dtype = dtype
    Xt_o = xo.probe_fwd(X, Z, ODT[dtype])
    check_probe_output(C, unp.cpu().numpy(), Xt_o, z_exact=(probe == "rademacher"))
    want = xo.dw_from_xt(dY, Xt_o, Z, kH, kW, (sh, sw), (ph, pw))
    assert rel_max(dW.cpu().numpy().astype(np.float64), want) <= GRAD_TOL[dtype]
    want_x = xo.dw_exact(dY, X, kH, kW, (sh, sw), (ph, pw))
    assert rel_max(dWx.cpu().numpy().astype(np.float64), want_x) <= GRAD_TOL[dtype]


def test_full_rank_hadamard_probe_gives_exact_gradient_on_gpu():
    # r = C_in and Z Z^T = r I: the estimate equals the exact gradient
    say("hadamard invariant")
    B, C, H, W = 4, 16, 12, 12
    Hm = np.array([[1.0]])
    while Hm.shape[0] < C:
        Hm = np.block([[Hm, Hm], [Hm, -Hm]])
    Z = Hm.astype(np.float32)
    X = synth.draw((B, C, H, W), 21, "normal", 1.0, "f32")
    dY = synth.draw((B, 24, H, W), 22, "normal", 1.0, "f32")
    d = xb.make_desc(B, C, 24, H, W, 3, 1, 1, C, "f32", "user", 0)
    Xd, dYd, Zd = xb.to_device(X, "f32", DEV), xb.to_device(dY, "f32", DEV), torch.from_numpy(Z).to(DEV)
    Xt = xb.alloc_xt(d, DEV)
    xb.xconv_probe_fwd(d, Xd, Xt, Zd, None)
    dW = torch.empty((24, C, 3, 3), dtype=torch.float32, device=DEV)
    xb.xconv_dw_estimate(d, dYd, Xt, Zd, dW, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
    torch.cuda.synchronize()
    exact = xo.dw_exact(dY, X, 3, 3, (1, 1), (1, 1))
    assert rel_max(dW.cpu().numpy().astype(np.float64), exact) <= 1e-5


def test_generic_kernel_repeats_its_result_300_times():
    # A layer of the generic correlation kernel (fp32, 1x1 kernel, two 16-row tiles per wave, odd output width) whose
    # result used to differ about once in a hundred launches: a register copy had been scheduled in front of the wait
    # for the LDS read that fills it.  300 launches, every result equal to the first bit for bit, the first checked
    # against the oracle.
    say("generic kernel, 300 launches")
    B, C_in, C_out, H, W, r = 12, 64, 64, 9, 36, 32
    X = synth.draw((B, C_in, H, W), 6041, "relu_normal", 1.0, "f32")
    dY = synth.draw((B, C_out, 11, 19), 7041, "normal", 1e-2, "f32")
    d = xb.make_desc(B, C_in, C_out, H, W, (1, 1), (1, 2), (1, 1), r, "f32", "rademacher", 8041)
    assert xb.xconv_plan_info(d, xb.XCONV_OP_EXACT)["ws"] == 0
    Xd, dYd = xb.to_device(X, "f32", DEV), xb.to_device(dY, "f32", DEV)
    ws = xb.alloc_ws(d, xb.XCONV_OP_EXACT, DEV)
    first = None
    for it in range(300):
        dW = torch.full((C_out, C_in, 1, 1), float("nan"), dtype=torch.float32, device=DEV)
        xb.xconv_dw_exact(d, dYd, Xd, dW, ws)
        if first is None:
            first = dW
        else:
            assert torch.equal(dW, first), it
    want = xo.dw_exact(dY, X, 1, 1, (1, 2), (1, 1))
    assert rel_max(first.cpu().numpy().astype(np.float64), want) <= 1e-4


def test_estimate_is_deterministic_and_overwrites():
    say("determinism")
    cfg = SMALL[1]
    X, dY = synth.make_layer(cfg)
    Z = xo.probe_matrix(OPROBE[cfg.probe], cfg.seeds[2], cfg.C_in, cfg.r)
    d, Xt, _ = run_probe(cfg, X, Z)
    a = run_estimate(cfg, d, dY, Xt, Z)
    b = run_estimate(cfg, d, dY, Xt, Z)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------------------
# the five layers at full size, in the launch configuration the bench times
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_full_size_complete(name):
    # Every entry of the stored probe output and of the estimate against the oracle, Z drawn from the seed on both
    # sides, in the launch configuration the bench times (the oracle needs about half a minute for the largest layer).
    full_parity(synth.CONFIGS[name], seed_path=True, check_exact=(name in ("C1", "C2")))


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_full_size_exact_rows(name):
    # Exact gradient at full size: whole rows dW[m, :, :, :] for one output channel out of every 16, so that every
    # (output-channel tile x input-channel block x kernel offset) of the running plan is compared, a sixteenth of all
    # entries.  The estimate must also equal those oracle rows mixed by Z Z^T / r (holds at any size).
    cfg = synth.CONFIGS[name]
    say("%s full size, exact gradient, one output channel in 16" % name)
    X, dY = synth.make_layer(cfg)
    Z = xo.probe_matrix(OPROBE[cfg.probe], cfg.seeds[2], cfg.C_in, cfg.r)
    st, pd = (cfg.stride, cfg.stride), (cfg.pad, cfg.pad)
    d = xb.desc_from_config(cfg)
    got_x = run_exact(cfg, d, dY, X)
    assert np.all(np.isfinite(got_x))
    rng = np.random.default_rng(5)
    rows = np.array([16 * t + int(rng.integers(0, 16)) for t in range(cfg.C_out // 16)])
    rows[0], rows[-1] = 0, cfg.C_out - 1
    idx = np.array([(m, n, ky, kx) for m in rows for n in range(cfg.C_in) for ky in range(cfg.k) for kx in range(cfg.k)], dtype=np.int32)
    say("%s oracle rows (%d entries)" % (name, len(idx)))
    wx = xo.dw_exact_at(dY, X, idx, cfg.k, cfg.k, st, pd).reshape(len(rows), cfg.C_in, cfg.k, cfg.k)
    gx = got_x[rows]
    scale = np.max(np.abs(wx))
    assert np.max(np.abs(got_x)) <= 1.5 * scale          # no stray large entry in the rows that are not compared
    assert np.max(np.abs(gx - wx)) <= GRAD_TOL[cfg.dtype] * scale, (np.max(np.abs(gx - wx)), scale)
    _, Xt, _ = run_probe(cfg, X, None, seed_path=True)
    got = run_estimate(cfg, d, dY, Xt, None)
    G = Z.astype(np.float64) @ Z.astype(np.float64).T / cfg.r
    mixed = np.einsum("nq,mqyx->mnyx", G, wx)
    assert np.max(np.abs(got[rows] - mixed)) <= 2 * GRAD_TOL[cfg.dtype] * np.max(np.abs(mixed))


def test_byte_offsets_beyond_4_gib():
    # X, dY and the stored probe output of 4.8 GB each (fp16): 144 copies of a batch of 16 images.  The small batch
    # is checked against the oracle (probe output in full, sampled gradient entries); on the large one every copy's
    # stored probe output must equal the small batch's bit for bit, and both gradients are 144 times the small
    # batch's (same products, a longer fp32 sum).
    B0, rep, C, H, r, dtype = 16, 144, 64, 128, 64, "f16"
    say("4.8 GB tensors: %d copies of %d images, C=%d, %dx%d, r=%d" % (rep, B0, C, H, H, r))
    X = synth.draw((B0, C, H, H), 21, "relu_normal", 1.0, dtype)
    dY = synth.draw((B0, C, H, H), 22, "normal", 1e-2, dtype)
    Z = xo.probe_matrix(OPROBE["rademacher"], 23, C, r)

    def run(B, Xd, dYd):
        d = xb.make_desc(B, C, C, H, H, 3, 1, 1, r, dtype, "rademacher", 23)
        Xt = xb.alloc_xt(d, DEV)
        xb.xconv_probe_fwd(d, Xd, Xt, None, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))
        unp = torch.empty((B, r, H, H), dtype=torch.float32, device=DEV)
        xb.xconv_xt_unpack(d, Xt, unp)
        dW = torch.full((C, C, 3, 3), float("nan"), dtype=torch.float32, device=DEV)
        xb.xconv_dw_estimate(d, dYd, Xt, None, dW, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
        dWx = torch.full((C, C, 3, 3), float("nan"), dtype=torch.float32, device=DEV)
        xb.xconv_dw_exact(d, dYd, Xd, dWx, xb.alloc_ws(d, xb.XCONV_OP_EXACT, DEV))
        torch.cuda.synchronize()
        return unp, dW.cpu().numpy().astype(np.float64), dWx.cpu().numpy().astype(np.float64)

    X0, dY0 = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    unp0, dW0, dWx0 = run(B0, X0, dY0)
    Xt_o = xo.probe_fwd(X, Z, ODT[dtype])

    class Storage:  # minimal stand-in for check_probe_output
        pass
    Storage.dtype = dtype
    check_probe_output(Storage, unp0.cpu().numpy(), Xt_o, z_exact=True)
    rng = np.random.default_rng(6)
    idx = np.stack([rng.integers(0, C, 24), rng.integers(0, C, 24), rng.integers(0, 3, 24), rng.integers(0, 3, 24)], axis=1).astype(np.int32)
    want = xo.dw_from_xt_at(dY, Xt_o, Z, idx, 3, 3, (1, 1), (1, 1))
    g = np.array([dW0[tuple(i)] for i in idx])
    assert np.max(np.abs(g - want)) <= GRAD_TOL[dtype] * np.max(np.abs(want))
    wx = xo.dw_exact_at(dY, X, idx, 3, 3, (1, 1), (1, 1))
    gx = np.array([dWx0[tuple(i)] for i in idx])
    assert np.max(np.abs(gx - wx)) <= GRAD_TOL[dtype] * np.max(np.abs(wx))

    say("4.8 GB tensors: the large batch")
    Xb, dYb = X0.repeat(rep, 1, 1, 1), dY0.repeat(rep, 1, 1, 1)
    assert Xb.numel() * Xb.element_size() > 2 ** 32
    unp, dW, dWx = run(B0 * rep, Xb, dYb)
    assert bool((unp.view(rep, B0, r, H, H) == unp0.unsqueeze(0)).all())
    del unp
    assert rel_max(dW, rep * dW0) <= 1e-3 and rel_max(dWx, rep * dWx0) <= 1e-3


# ---------------------------------------------------------------------------
# seeded random shapes: every kernel choice the plans can make (generic, 16-bit and fp32
# producer/consumer kernels, strips, partial image groups, offset groups, both layouts, sparse
# probes) against the oracle
# ---------------------------------------------------------------------------
def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        dtype = ["f32", "bf16", "f16"][rng.integers(3)]
        k = [1, 2, 3, 3, 3, 5][rng.integers(6)]
        kH, kW = (k, k) if rng.random() < 0.8 else (k, [1, 3][rng.integers(2)])
        sh = [1, 1, 2, 3][rng.integers(4)]
        sw = sh if rng.random() < 0.8 else [1, 2][rng.integers(2)]
        ph, pw = int(rng.integers(0, kH // 2 + 2)), int(rng.integers(0, kW // 2 + 2))
        H, W = int(rng.integers(kH + 1, 30)), int(rng.integers(kW + 1, 44))
        if rng.random() < 0.5:
            W = (W + 3) // 4 * 4
        if (H + 2 * ph - kH) // sh + 1 < 1 or (W + 2 * pw - kW) // sw + 1 < 1:
            continue
        B = int(rng.integers(1, 20))
        C_in = int([4, 8, 16, 24, 32, 40, 64, 72][rng.integers(8)])
        C_out = int([8, 16, 24, 32, 48, 64, 96, 136][rng.integers(8)])
        r = int([1, 4, 8, 16, 20, 32, 64][rng.integers(7)])
        probe = ["rademacher", "gaussian"][rng.integers(2)]
        nhwc = bool(rng.random() < 0.3)
        keep = int([0, 0, 0, 12000, 24000][rng.integers(5)])
        if B * C_out * H * W * C_in > 6e7:      # keep the oracle quick
            continue
        out.append((len(out), B, C_in, C_out, H, W, (kH, kW), (sh, sw), (ph, pw), r, probe, dtype, nhwc, keep))
    return out


RANDOM_CASES = _random_cases(48, 20240607)


@pytest.mark.parametrize("case", RANDOM_CASES, ids=["rnd%02d-%s" % (c[0], c[11]) for c in RANDOM_CASES])
def test_random_shapes(case):
    idx, B, C_in, C_out, H, W, (kH, kW), (sh, sw), (ph, pw), r, probe, dtype, nhwc, keep = case
    say("random case %d: B%d C%d->%d %dx%d k%dx%d s%d,%d p%d,%d r%d %s %s %s keep=%d" % (
        idx, B, C_in, C_out, H, W, kH, kW, sh, sw, ph, pw, r, probe, dtype, "NHWC" if nhwc else "NCHW", keep))
    Ho, Wo = xo.out_extent(H, kH, sh, ph), xo.out_extent(W, kW, sw, pw)
    X = synth.draw((B, C_in, H, W), 6000 + idx, "relu_normal", 1.0, dtype)
    dY = synth.draw((B, C_out, Ho, Wo), 7000 + idx, "normal", 1e-2, dtype)
    Z = xo.probe_matrix(OPROBE[probe], 8000 + idx, C_in, r, keep)
    d = xb.make_desc(B, C_in, C_out, H, W, (kH, kW), (sh, sw), (ph, pw), r, dtype, probe, 8000 + idx,
                     layout=xb.XCONV_NHWC if nhwc else xb.XCONV_NCHW, keep_q15=keep)
    if nhwc:
        Xd = xb.to_device(np.ascontiguousarray(X.transpose(0, 2, 3, 1)), dtype, DEV)
        dYd = xb.to_device(np.ascontiguousarray(dY.transpose(0, 2, 3, 1)), dtype, DEV)
    else:
        Xd, dYd = xb.to_device(X, dtype, DEV), xb.to_device(dY, dtype, DEV)
    # Z from the seed on the device: Rademacher is bit-identical to the oracle's, Gaussian to an ulp
    Xt = xb.alloc_xt(d, DEV)
    xb.xconv_probe_fwd(d, Xd, Xt, None, xb.alloc_ws(d, xb.XCONV_OP_PROBE, DEV))
    dW = torch.full((C_out, C_in, kH, kW), float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_estimate(d, dYd, Xt, None, dW, xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, DEV))
    dWx = torch.full((C_out, C_in, kH, kW), float("nan"), dtype=torch.float32, device=DEV)
    xb.xconv_dw_exact(d, dYd, Xd, dWx, xb.alloc_ws(d, xb.XCONV_OP_EXACT, DEV))
    torch.cuda.synchronize()
    Xt_o = xo.probe_fwd(X, Z, ODT[dtype])
    want = xo.dw_from_xt(dY, Xt_o, Z, kH, kW, (sh, sw), (ph, pw), nnz_norm=keep != 0)
    got = dW.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    scale = max(np.max(np.abs(want)), 1e-30)
    assert np.max(np.abs(got - want)) / scale <= GRAD_TOL[dtype], xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)
    want_x = xo.dw_exact(dY, X, kH, kW, (sh, sw), (ph, pw))
    assert rel_max(dWx.cpu().numpy().astype(np.float64), want_x) <= GRAD_TOL[dtype], xb.xconv_plan_info(d, xb.XCONV_OP_EXACT)
