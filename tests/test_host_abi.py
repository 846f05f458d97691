"""Host-side checks of the C-ABI library: it loads, exports every entry point
the header declares, validates descriptors and reports sizes without touching
a GPU, and its host probe generator agrees with the oracle's.  CPU only."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import xconv_oracle as xo
from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "xconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(xconv(?:3d)?_[a-z0-9_]+)\s*\(", text))
    assert {"xconv_probe_fwd", "xconv_dw_estimate", "xconv_dw_exact", "xconv3d_probe_fwd", "xconv3d_dw_estimate"} <= names
    L = xb.lib()
    for n in sorted(names):
        assert hasattr(L, n), n


def test_desc_struct_layout_matches_header():
    assert ctypes.sizeof(xb.xconv_desc) == 16 * 4 + 8
    assert xb.xconv_desc.seed.offset == 64


def _good():
    return xb.make_desc(4, 16, 16, 32, 32, 3, 1, 1, 8, "f32", "rademacher", 3001)


def test_check_desc_statuses():
    assert xb.xconv_check_desc(_good()) == xb.XCONV_OK
    assert xb.lib().xconv_check_desc(None) == xb.XCONV_EINVAL
    for field, val in (("B", 0), ("C_in", -1), ("C_out", 0), ("H", 0), ("W", 0), ("kH", 0), ("kW", 0),
                       ("stride_h", 0), ("stride_w", 0), ("pad_h", -1), ("pad_w", -1), ("r", 0),
                       ("dtype", 3), ("dtype", -1), ("layout", 2), ("probe", 3), ("keep_q15", -1), ("keep_q15", 32768)):
        d = _good()
        setattr(d, field, val)
        assert xb.xconv_check_desc(d) == xb.XCONV_EINVAL, field
    d = _good()
    d.kH = d.kW = 40            # kernel larger than the padded image: empty output
    assert xb.xconv_check_desc(d) == xb.XCONV_EINVAL
    d = _good()
    d.layout = xb.XCONV_NHWC
    assert xb.xconv_check_desc(d) == xb.XCONV_OK
    for field, val in (("r", 1025), ("C_in", 70000), ("C_out", 70000)):
        d = _good()
        setattr(d, field, val)
        assert xb.xconv_check_desc(d) == xb.XCONV_EUNSUPPORTED, field
    d = xb.make_desc(1, 1, 1, 64, 64, 8, 1, 0, 1)     # 64 kernel offsets
    assert xb.xconv_check_desc(d) == xb.XCONV_EUNSUPPORTED
    assert "unsupported" in xb.xconv_status_string(xb.XCONV_EUNSUPPORTED)
    assert xb.xconv_status_string(0) == "ok"


def test_sizes():
    d = _good()
    assert xb.xconv_xt_bytes(d) == 4 * 32 * 32 * 16 * 4          # r = 8 is stored padded to 16 columns
    d16 = xb.make_desc(256, 256, 256, 28, 28, 3, 1, 1, 64, "f16")
    assert xb.xconv_xt_bytes(d16) == 256 * 28 * 28 * 64 * 2
    assert xb.xconv_workspace_bytes(d, xb.XCONV_OP_PROBE) >= 16 * 8 * 4
    west = xb.xconv_workspace_bytes(d, xb.XCONV_OP_ESTIMATE)
    wex = xb.xconv_workspace_bytes(d, xb.XCONV_OP_EXACT)
    assert west > 16 * 8 * 4 and wex > 4 * 32 * 32 * 16 * 4
    bad = _good()
    bad.r = 0
    assert xb.xconv_xt_bytes(bad) == 0 and xb.xconv_workspace_bytes(bad, 1) == 0
    assert xb.xconv_workspace_bytes(d, 7) == 0
    # every benchmark layer gets a plan and a modest scratch size
    for cfg in synth.CONFIGS.values():
        dd = xb.desc_from_config(cfg)
        assert xb.xconv_check_desc(dd) == xb.XCONV_OK
        w = xb.xconv_workspace_bytes(dd, xb.XCONV_OP_ESTIMATE)
        assert 0 < w < 256 * 2 ** 20, (cfg.name, w)
        assert xb.xconv_workspace_bytes(dd, xb.XCONV_OP_EXACT) > 0


@pytest.mark.parametrize("probe,code", [("rademacher", xo.RADEMACHER), ("gaussian", xo.GAUSSIAN)])
def test_host_probe_matrix_matches_oracle_generator(probe, code):
    for seed, C_in, r in ((3001, 16, 8), (3005, 256, 64), (2 ** 63 + 5, 7, 3)):
        d = xb.make_desc(1, C_in, 1, 8, 8, 3, 1, 1, r, "f32", probe, seed)
        Z = xb.xconv_probe_matrix(d)
        Zo = xo.probe_matrix(code, seed, C_in, r)
        if probe == "rademacher":
            assert np.array_equal(Z, Zo)
        else:
            # same stream words, same double-precision Box-Muller: at most an ulp apart
            assert np.max(np.abs(Z - Zo)) <= 2.4e-7 * np.max(np.abs(Zo))
            assert np.mean(Z == Zo) > 0.99
    # block-sparse probes: the same entries dropped as in the oracle's matrix
    for keep in (1, 8192, 16384, 32767):
        d = xb.make_desc(1, 48, 1, 8, 8, 3, 1, 1, 40, "f32", probe, 4242, keep_q15=keep)
        Z = xb.xconv_probe_matrix(d)
        Zo = xo.probe_matrix(code, 4242, 48, 40, keep)
        assert np.array_equal(Z == 0, Zo == 0)
        assert np.max(np.abs(Z - Zo)) <= 2.4e-7 * max(np.max(np.abs(Zo)), 1e-30)
    d = xb.make_desc(1, 4, 1, 8, 8, 3, 1, 1, 2, "f32", "user", 1)
    with pytest.raises(xb.XConvError) as e:
        xb.xconv_probe_matrix(d)
    assert e.value.status == xb.XCONV_EINVAL


def test_entry_points_reject_bad_arguments_before_any_launch():
    L = xb.lib()
    d = _good()
    p = ctypes.byref(d)
    one = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    assert L.xconv_probe_fwd(p, None, one, one, None, 0, None) == xb.XCONV_EINVAL
    assert L.xconv_probe_fwd(p, one, None, one, None, 0, None) == xb.XCONV_EINVAL
    assert L.xconv_probe_fwd(p, one, ctypes.c_void_p(4100), one, None, 0, None) == xb.XCONV_EINVAL   # Xt misaligned
    assert L.xconv_probe_fwd(p, one, one, None, None, 0, None) == xb.XCONV_EINVAL                    # no Z, no scratch
    assert L.xconv_probe_fwd(p, one, one, None, one, 16, None) == xb.XCONV_EWORKSPACE
    assert L.xconv_dw_estimate(p, None, one, one, one, one, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_dw_estimate(p, one, one, one, None, one, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_dw_estimate(p, one, one, one, one, None, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_dw_estimate(p, one, one, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    assert L.xconv_dw_exact(p, one, None, one, one, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_dw_exact(p, one, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    assert L.xconv_xt_unpack(p, None, one, None) == xb.XCONV_EINVAL
    du = _good()
    du.probe = xb.XCONV_USER_Z
    assert L.xconv_dw_estimate(ctypes.byref(du), one, one, None, one, one, 1 << 30, None) == xb.XCONV_EINVAL
    # a channels-last dY is always copied into plane form: its workspace is larger by that copy
    dn = _good()
    dn.layout = xb.XCONV_NHWC
    for op in (xb.XCONV_OP_ESTIMATE, xb.XCONV_OP_EXACT):
        assert xb.xconv_workspace_bytes(dn, op) > xb.xconv_workspace_bytes(_good(), op)


def test_volumetric_descriptor_and_sizes():
    assert ctypes.sizeof(xb.xconv3d_desc) == ctypes.sizeof(xb.xconv_desc) + 16
    good = lambda: xb.make_desc3d(2, 16, 32, 8, 12, 12, 3, 1, 1, r=8, dtype="bf16")
    v = good()
    assert xb.xconv3d_check_desc(v) == xb.XCONV_OK
    assert xb.lib().xconv3d_check_desc(None) == xb.XCONV_EINVAL
    for field, val in (("D", 0), ("kD", 0), ("pad_d", -1), ("stride_d", 0)):
        v = good()
        setattr(v, field, val)
        assert xb.xconv3d_check_desc(v) == xb.XCONV_EINVAL, field
    v = good()
    v.l.r = 0                                            # the in-plane part is validated as a 2-D layer
    assert xb.xconv3d_check_desc(v) == xb.XCONV_EINVAL
    for field, val in (("pad_d", 0), ("pad_d", 2), ("kD", 2)):                # D' = D - 2, D + 2, D + 1
        v = good()
        setattr(v, field, val)
        assert xb.xconv3d_check_desc(v) == xb.XCONV_OK, field
    for field, val in (("pad_d", 3), ("kD", 9)):                              # pad_d <= kD - 1, kD <= 7
        v = good()
        setattr(v, field, val)
        assert xb.xconv3d_check_desc(v) == xb.XCONV_EUNSUPPORTED, field
    v = good()
    v.D, v.pad_d = 2, 0                                   # kernel deeper than the volume: empty output
    assert xb.xconv3d_check_desc(v) == xb.XCONV_EINVAL
    v = good()
    v.l.layout = xb.XCONV_NHWC                             # channels-last volumes
    assert xb.xconv3d_check_desc(v) == xb.XCONV_OK
    v.l.B = 8000                                          # more depth slots than one grid extent: the copies go in pieces
    assert xb.xconv3d_check_desc(v) == xb.XCONV_OK and xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_ESTIMATE) > 0
    v = xb.make_desc3d(1, 4, 4, 6, 8, 8, (1, 3, 3), 1, (0, 1, 1), r=4)        # a stack of independent 2-D layers
    assert xb.xconv3d_check_desc(v) == xb.XCONV_OK
    assert xb.xconv3d_xt_bytes(v) == 6 * 8 * 8 * 16 * 4
    v = good()
    # per image one zero slot and 8 slices, two more zero slices for the deepest offset behind the run
    assert xb.xconv3d_xt_bytes(v) == (2 * 9 + 2) * 12 * 12 * 16 * 2
    v.pad_d = 0
    assert xb.xconv3d_xt_bytes(v) == (2 * 8 + 2) * 12 * 12 * 16 * 2
    v = good()
    v.stride_d = 2                                        # two runs (even and odd slots) of 2 * 5 + 1 slices
    assert xb.xconv3d_check_desc(v) == xb.XCONV_OK
    assert xb.xconv3d_xt_bytes(v) == 2 * (2 * 5 + 1) * 12 * 12 * 16 * 2
    v = good()
    assert xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_PROBE) >= 16 * 8 * 4
    west = xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_ESTIMATE)
    assert west > 2 * 9 * 32 * 12 * 12 * 2               # holds the slice-major copy of dY
    assert xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_EXACT) > (2 * 9 + 2) * 12 * 12 * 16 * 2     # channels-last X slices
    assert xb.xconv3d_workspace_bytes(v, 7) == 0
    L = xb.lib()
    p = ctypes.byref(v)
    one = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    assert L.xconv3d_probe_fwd(p, None, one, one, None, 0, None) == xb.XCONV_EINVAL
    assert L.xconv3d_probe_fwd(p, one, one, None, one, 16, None) == xb.XCONV_EWORKSPACE
    assert L.xconv3d_dw_estimate(p, one, one, one, one, None, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv3d_dw_estimate(p, one, one, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    assert L.xconv3d_dw_exact(p, one, None, one, one, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv3d_dw_exact(p, one, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    assert L.xconv3d_xt_unpack(p, None, one, None) == xb.XCONV_EINVAL


def test_pixel_probe_sizes_and_argument_checks():
    d = _good()                                            # B=4, C_in=16, 32x32, r=8, fp32
    assert xb.xconv_pixel_xbar_bytes(d) == 4 * 8 * 4
    wf = xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_PROBE)
    wb = xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_ESTIMATE)
    assert wf > 8 * 16 * 32 * 32 * 4 and wb > 16 * 16 * 32 * 32 * 4       # the probing vectors are redrawn in scratch
    assert xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_EXACT) == 0
    sparse = _good()
    sparse.keep_q15 = 100
    assert xb.xconv_pixel_xbar_bytes(sparse) == 4 * 8 * 4
    cl = _good()
    cl.layout = xb.XCONV_NHWC                               # channels-last: same state, the backward pass also repacks L
    assert xb.xconv_pixel_xbar_bytes(cl) == 4 * 8 * 4 and xb.xconv_pixel_workspace_bytes(cl, xb.XCONV_OP_PROBE) == wf
    assert xb.xconv_pixel_workspace_bytes(cl, xb.XCONV_OP_ESTIMATE) > wb
    for field, val in (("probe", xb.XCONV_USER_Z),):
        bad = _good()
        setattr(bad, field, val)
        assert xb.xconv_pixel_xbar_bytes(bad) == 0 and xb.xconv_pixel_workspace_bytes(bad, 0) == 0
        assert xb.lib().xconv_pixel_probe_fwd(ctypes.byref(bad), ctypes.c_void_p(4096), ctypes.c_void_p(4096),
                                               ctypes.c_void_p(4096), 1 << 30, None) == xb.XCONV_EUNSUPPORTED
    L = xb.lib()
    p = ctypes.byref(d)
    one = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    assert L.xconv_pixel_probe_fwd(p, None, one, one, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_pixel_probe_fwd(p, one, one, None, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_pixel_probe_fwd(p, ctypes.c_void_p(4100), one, one, 1 << 30, None) == xb.XCONV_EINVAL    # X misaligned
    assert L.xconv_pixel_probe_fwd(p, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    assert L.xconv_pixel_dw_estimate(p, one, None, one, one, 1 << 30, None) == xb.XCONV_EINVAL
    assert L.xconv_pixel_dw_estimate(p, one, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    bad = _good()
    bad.r = 0
    assert L.xconv_pixel_dw_estimate(ctypes.byref(bad), one, one, one, one, 1 << 30, None) == xb.XCONV_EINVAL


def test_independent_probing_sizes_and_limits():
    d = _good()                                            # B=4, C_in=16, 32x32, r=8, fp32
    assert xb.xconv_pixel_indep_xbar_bytes(d) == 4 * 16 * 8 * 4            # [B, C_in, r] floats
    wf = xb.xconv_pixel_indep_workspace_bytes(d, xb.XCONV_OP_PROBE)
    wb = xb.xconv_pixel_indep_workspace_bytes(d, xb.XCONV_OP_ESTIMATE)
    assert wf > 0 and wb > 0
    L = xb.lib()
    one = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    assert L.xconv_pixel_indep_probe_fwd(ctypes.byref(d), one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    assert L.xconv_pixel_indep_probe_fwd(ctypes.byref(d), None, one, one, 1 << 40, None) == xb.XCONV_EINVAL
    assert L.xconv_pixel_indep_dw_estimate(ctypes.byref(d), one, one, one, one, 64, None) == xb.XCONV_EWORKSPACE
    wide = _good()
    wide.r = 1024 // wide.C_in + 1                          # more than 1024 vectors in all: several passes over channel groups
    assert xb.xconv_pixel_indep_xbar_bytes(wide) == 4 * 16 * wide.r * 4 and xb.xconv_pixel_indep_workspace_bytes(wide, xb.XCONV_OP_ESTIMATE) > 0
    huge = _good()
    huge.C_in, huge.r = 4096, 32                            # C_in * r beyond 65536
    sparse = _good()
    sparse.keep_q15 = 16384                                 # block-sparse vectors belong to the multi-channel mode
    for bad in (huge, sparse):
        assert xb.xconv_pixel_indep_xbar_bytes(bad) == 0 and xb.xconv_pixel_indep_workspace_bytes(bad, xb.XCONV_OP_ESTIMATE) == 0
        assert L.xconv_pixel_indep_probe_fwd(ctypes.byref(bad), one, one, one, 1 << 40, None) == xb.XCONV_EUNSUPPORTED
        assert L.xconv_pixel_indep_dw_estimate(ctypes.byref(bad), one, one, one, one, 1 << 40, None) == xb.XCONV_EUNSUPPORTED
    edge = _good()
    edge.r = 1024 // edge.C_in
    assert xb.xconv_pixel_indep_xbar_bytes(edge) == 4 * 1024 * 4


def test_pixel_probe_state_reproduces_the_paper_memory_ratio():
    # Sec. 4.1 worked example: a 32x32 image with 16 input channels, r = 2^gamma probing vectors: the stored state of the
    # probe over pixels and channels is N*C_in/r = 2^(14-gamma) times smaller than the activation (same element size)
    path = os.path.join(ROOT, "tests", "golden", "paper_memory_ratio.txt")
    rows = [tuple(int(t) for t in line.split()) for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) == 8
    for gamma, ratio in rows:
        d = xb.make_desc(4, 16, 8, 32, 32, 3, 1, 1, 2 ** gamma, "f32")
        act = d.B * d.C_in * d.H * d.W * 4
        assert act // xb.xconv_pixel_xbar_bytes(d) == ratio
        # the channel probe keeps H*W values per probing vector instead: C_in / r (r is stored padded to 16 columns)
        assert act * 16 // xb.xconv_xt_bytes(d) == 16 * 16 // max(2 ** gamma, 16)


def test_synthetic_inputs_are_storage_representable_and_seeded():
    cfg = synth.small_variant(synth.CONFIGS["C3"], B=2, H=12, W=12, C_in=8, C_out=8)
    X, dY = synth.make_layer(cfg)
    X2, dY2 = synth.make_layer(cfg)
    assert np.array_equal(X, X2) and np.array_equal(dY, dY2)
    assert np.array_equal(synth.round_to_storage(X, "bf16"), X)
    assert X.min() == 0.0 and 0.3 < np.mean(X == 0.0) < 0.7           # post-ReLU: about half zeros
    assert abs(dY.std() - 0.1) < 0.02
    assert dY.shape == (2, 8, 6, 6)
    bits = synth.storage_bits(X, "bf16")
    assert bits.dtype == np.uint16
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), X)
    h = synth.draw((64,), 5, "normal", 1.0, "f16")
    assert np.array_equal(h.astype(np.float16).astype(np.float32), h)


def test_launch_plans_stay_within_the_device_limits_on_random_layers():
    # host plans only: every supported layer gets a plan whose LDS, split count and tile sizes are consistent
    rng = np.random.default_rng(77)
    seen = set()
    for _ in range(400):
        dtype = ["f32", "bf16", "f16"][rng.integers(3)]
        k = int(rng.integers(1, 6))
        s = int(rng.integers(1, 4))
        p = int(rng.integers(0, k + 1))
        H, W = int(rng.integers(k, 80)), int(rng.integers(k, 80))
        d = xb.make_desc(int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 300)), H, W, k, s, p,
                         int(rng.integers(1, 130)), dtype)
        if xb.xconv_check_desc(d) != xb.XCONV_OK:
            continue
        for op in (xb.XCONV_OP_ESTIMATE, xb.XCONV_OP_EXACT):
            ws = xb.xconv_workspace_bytes(d, op)
            assert ws > 0, (op, [getattr(d, f[0]) for f in d._fields_])
            plan = xb.xconv_plan_info(d, op)
            seen.add(plan["ws"])
            assert 1 <= plan["S"] <= plan["NS"]
            assert 0 < plan["lds_bytes"] <= 160 * 1024
            assert plan["WM"] * plan["WJ"] * plan["WK"] == 4
            assert plan["CS"] % 16 == 0 and plan["CS"] >= (d.r if op == xb.XCONV_OP_ESTIMATE else d.C_in)
            assert plan["NTM"] * plan["M_WG"] >= d.C_out and plan["NTJ"] * plan["J_WG"] == plan["CS"]
            assert ws < 2 ** 34
    assert seen == {0, 1, 2, 3}       # all four correlation kernels get layers


def test_plan_overrides_are_part_of_the_plan_cache_key(monkeypatch):
    # A plan made under one setting of an XCONV_* override is never handed out under another: the fp32
    # producer/consumer plan of one layer, asked for with one and then with two workgroups per compute unit (the
    # second request would hit the cached first plan if the key were the shape alone), and back again.
    d = xb.make_desc(8, 64, 64, 256, 256, 3, 1, 1, 16, "f32", "gaussian", 13)   # (many steps per split: both counts fill the units)
    monkeypatch.setenv("XCONV_WS32_OCC", "1")
    one = xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)
    monkeypatch.setenv("XCONV_WS32_OCC", "2")
    two = xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)
    monkeypatch.setenv("XCONV_WS32_OCC", "1")
    again = xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE)
    assert one["ws"] == 2 and two["ws"] == 2
    assert again == one
    assert 2 * two["lds_bytes"] <= 160 * 1024          # two workgroups share a compute unit's LDS
    assert two != one and two["S"] > one["S"]          # and the K-split counts both of them
    # the same for a split-count override of the 16-bit kernel
    h = xb.make_desc(9, 64, 64, 14, 14, 3, 1, 1, 64, "f16", "rademacher", 13)
    base = xb.xconv_plan_info(h, xb.XCONV_OP_ESTIMATE)
    monkeypatch.setenv("XCONV_ROW_SPLITS", "3")
    monkeypatch.setenv("XCONV_WS_SPLITS", "3")
    forced = xb.xconv_plan_info(h, xb.XCONV_OP_ESTIMATE)
    monkeypatch.delenv("XCONV_ROW_SPLITS")
    monkeypatch.delenv("XCONV_WS_SPLITS")
    assert forced["S"] == 3 and base["S"] != 3
    assert xb.xconv_plan_info(h, xb.XCONV_OP_ESTIMATE) == base


def test_static_scratch_entry_point_checks_before_it_touches_a_device():
    # xconv_dw_estimate_static: descriptor and size checks come first and need no GPU
    L = xb.lib()
    assert xb.xconv_static_scratch_bytes() == 40 * 1024 * 1024
    d = _good()
    d.r = 0
    assert L.xconv_dw_estimate_static(ctypes.byref(d), 16, 16, None, 16, None) == xb.XCONV_EINVAL
    big = xb.make_desc(64, 256, 512, 28, 28, 3, 1, 1, 256, "f16", "rademacher", 1)
    assert xb.xconv_workspace_bytes(big, xb.XCONV_OP_ESTIMATE) > xb.xconv_static_scratch_bytes()
    assert L.xconv_dw_estimate_static(ctypes.byref(big), 16, 16, None, 16, None) == xb.XCONV_EWORKSPACE


def test_sign_relu_sizes_and_argument_checks():
    assert [xb.xconv_relu_mask_bytes(n) for n in (0, 1, 64, 65, 1 << 20)] == [0, 8, 8, 16, 1 << 17]
    L = xb.lib()
    one = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    assert L.xconv_relu_fwd(0, None, None, None, 0, None) == xb.XCONV_OK            # nothing to do
    assert L.xconv_relu_fwd(3, one, one, one, 8, None) == xb.XCONV_EINVAL           # dtype
    assert L.xconv_relu_fwd(0, one, one, one, -1, None) == xb.XCONV_EINVAL
    assert L.xconv_relu_fwd(0, None, one, one, 8, None) == xb.XCONV_EINVAL
    assert L.xconv_relu_fwd(0, ctypes.c_void_p(4100), one, one, 8, None) == xb.XCONV_EINVAL   # X misaligned
    assert L.xconv_relu_fwd(0, one, one, ctypes.c_void_p(4100), 8, None) == xb.XCONV_EINVAL   # mask misaligned
    assert L.xconv_relu_bwd(1, one, None, one, 8, None) == xb.XCONV_EINVAL
    assert L.xconv_relu_bwd(2, one, one, one, (1 << 40) + 1, None) == xb.XCONV_EUNSUPPORTED


def test_matrix_rate_diagnostic_checks_its_arguments():
    L = xb.lib()
    one = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    big = xb.XCONV_DIAG_OUT_BYTES
    assert L.xconv_diag_mfma_rate(3, 10, one, big, None, None) == xb.XCONV_EINVAL          # dtype
    assert L.xconv_diag_mfma_rate(0, 0, one, big, None, None) == xb.XCONV_EINVAL           # iters
    assert L.xconv_diag_mfma_rate(0, (1 << 24) + 1, one, big, None, None) == xb.XCONV_EINVAL
    assert L.xconv_diag_mfma_rate(2, 10, None, big, None, None) == xb.XCONV_EINVAL
    assert L.xconv_diag_mfma_rate(2, 10, ctypes.c_void_p(4098), big, None, None) == xb.XCONV_EINVAL
    assert L.xconv_diag_mfma_rate(2, 10, one, big - 1, None, None) == xb.XCONV_EWORKSPACE


def test_host_planning_is_thread_safe():
    # size and plan queries from several threads at once (an autograd backward thread beside the forward thread)
    # agree with the answers of one thread
    import threading
    rng = np.random.default_rng(99)
    descs = []
    while len(descs) < 64:
        k = int(rng.integers(1, 6))
        d = xb.make_desc(int(rng.integers(1, 64)), int(rng.integers(1, 200)), int(rng.integers(1, 200)), int(rng.integers(k, 60)),
                         int(rng.integers(k, 60)), k, int(rng.integers(1, 3)), int(rng.integers(0, k)), int(rng.integers(1, 100)),
                         ["f32", "bf16", "f16"][rng.integers(3)])
        if xb.xconv_check_desc(d) == xb.XCONV_OK:
            descs.append(d)

    def answers(order):
        out = {}
        for i in order:
            d = descs[i]
            out[i] = (xb.xconv_xt_bytes(d), xb.xconv_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), xb.xconv_workspace_bytes(d, xb.XCONV_OP_EXACT),
                      tuple(sorted(xb.xconv_plan_info(d, xb.XCONV_OP_ESTIMATE).items())), xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_ESTIMATE))
        return out

    results = [None] * 8

    def work(t):
        results[t] = answers(np.random.default_rng(t).permutation(len(descs)))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(8)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    want = answers(range(len(descs)))
    assert all(r == want for r in results)

