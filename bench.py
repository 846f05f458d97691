#!/usr/bin/env python3
"""Benchmark of the XConv weight-gradient hot path on one MI355X.

A step is one pass of the whole path over one synthetic layer: xconv_probe_fwd
(Z regenerated from the step's seed, Xt written) followed by xconv_dw_estimate
(Z regenerated again, correlation, reduction + Z/r expansion), i.e. Algorithm 1
forward step 2-3 and backward steps 1-4.  Inputs are resident in HBM before the
timed region; several buffer sets are rotated so that the working set does not
sit in the 256 MB Infinity Cache.

Prints one JSON line (see README/DESIGN for the fields).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0}

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE scaled by a copy kernel of known size; see
# profiles/).  bytes, or None where not measured yet.
MEASURED_TRAFFIC = {
    # (FETCH_SIZE * 2 + WRITE_SIZE) KiB per launch, profiles/xconv_kernels_<config>.txt
    ("C1", "corr_ws32_kernel"): 3.8e6, ("C1", "probe_kernel"): 0.7e6,
    ("C2", "corr_ws32_kernel"): 53.1e6, ("C2", "probe_kernel"): 42.1e6,
    ("C3", "corr_kernel"): 73.1e6, ("C3", "probe_kernel"): 64.5e6,
    ("C4", "corr_ws32_kernel"): 218.0e6, ("C4", "probe_kernel"): 168.0e6,
    ("C5", "corr_row_kernel"): 218.2e6, ("C5", "probe_kernel"): 129.5e6,
}


def elem_bytes(dtype):
    return 4 if dtype == "f32" else 2


def algorithmic(cfg):
    """Algorithmic bytes and flops per launch of each kernel of the path."""
    s = elem_bytes(cfg.dtype)
    P = cfg.B * cfg.Ho * cfg.Wo
    k2 = cfg.k * cfg.k
    probe_bytes = (cfg.C_in + cfg.r) * cfg.B * cfg.H * cfg.W * s
    probe_flops = 2.0 * cfg.B * cfg.H * cfg.W * cfg.C_in * cfg.r
    corr_bytes = P * cfg.C_out * s + cfg.B * cfg.H * cfg.W * cfg.r * s + cfg.C_out * cfg.r * k2 * 4
    corr_flops = 2.0 * P * cfg.C_out * cfg.r * k2
    exact_bytes = P * cfg.C_out * s + cfg.B * cfg.H * cfg.W * cfg.C_in * s + cfg.C_out * cfg.C_in * k2 * 4
    exact_flops = 2.0 * P * cfg.C_out * cfg.C_in * k2
    return dict(probe_bytes=probe_bytes, probe_flops=probe_flops, corr_bytes=corr_bytes, corr_flops=corr_flops,
                exact_bytes=exact_bytes, exact_flops=exact_flops,
                act_bytes_saved=(cfg.C_in - cfg.r) * cfg.B * cfg.H * cfg.W * s)


class Layer:
    """Device buffers of one layer, `nsets` rotating copies."""

    def __init__(self, cfg, nsets, dev, nhwc=False):
        import numpy as np
        import torch
        from paper_2106_06998_amd import binding as xb
        from paper_2106_06998_amd import synth
        self.cfg, self.xb = cfg, xb
        self.desc = xb.desc_from_config(cfg)
        X, dY = synth.make_layer(cfg)
        self.host = (X, dY)
        if nhwc:            # the same values handed over channels-last
            self.desc.layout = xb.XCONV_NHWC
            X = np.ascontiguousarray(X.transpose(0, 2, 3, 1))
            dY = np.ascontiguousarray(dY.transpose(0, 2, 3, 1))
        self.sets = []
        for i in range(nsets):
            Xd = xb.to_device(X, cfg.dtype, dev)
            dYd = xb.to_device(dY, cfg.dtype, dev)
            self.sets.append(dict(
                X=Xd, dY=dYd, Xt=xb.alloc_xt(self.desc, dev),
                dW=torch.empty((cfg.C_out, cfg.C_in, cfg.k, cfg.k), dtype=torch.float32, device=dev),
                ws=xb.alloc_ws(self.desc, xb.XCONV_OP_ESTIMATE, dev),
                wsx=None))
        self.dev = dev

    def step(self, i):
        s = self.sets[i % len(self.sets)]
        self.desc.seed = self.cfg.seeds[2] + i          # a fresh seed per iteration (Algorithm 1)
        self.xb.xconv_probe_fwd(self.desc, s["X"], s["Xt"], None, s["ws"])
        self.xb.xconv_dw_estimate(self.desc, s["dY"], s["Xt"], None, s["dW"], s["ws"])

    def exact(self, i):
        s = self.sets[i % len(self.sets)]
        if s["wsx"] is None:
            s["wsx"] = self.xb.alloc_ws(self.desc, self.xb.XCONV_OP_EXACT, self.dev)
        self.xb.xconv_dw_exact(self.desc, s["dY"], s["X"], s["dW"], s["wsx"])


def time_region(fn, steps, warmup):
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_times(xb, fn, steps, warmup):
    """Average duration of each kernel over `steps` timed steps, from HIP events
    the library records on its launch stream around every kernel."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    xb.xconv_prof_enable(True)
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    xb.xconv_prof_enable(False)
    acc = {}
    for kid, ms in xb.xconv_prof_collect():
        name = xb.xconv_prof_kernel_name(kid)
        a = acc.setdefault(name, [0.0, 0])
        a[0] += ms
        a[1] += 1
    return {k: v[0] / v[1] for k, v in acc.items()}, wall


def machine_rates(xb, dev):
    """What this machine delivers to plain reference kernels, next to the published peaks the fractions are stated against:
    a 256 MiB device copy (bytes read + written per second), and the library's matrix-instruction issue loop
    (xconv_diag_mfma_rate) for fp32 and fp16."""
    import torch
    src = torch.full((64 * 2 ** 20,), 1.0, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(3):
        dst.copy_(src)
    ev[0].record()
    for _ in range(10):
        dst.copy_(src)
    ev[1].record()
    torch.cuda.synchronize()
    copy_gbps = 10 * 2 * src.numel() * 4 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    del src, dst
    out = {"hbm_copy_gbps": copy_gbps, "hbm_copy": "256 MiB torch device copy, read + written bytes, 10 copies"}
    scratch = xb.alloc_bytes(xb.XCONV_DIAG_OUT_BYTES, dev)
    for dt, iters in (("f16", 4000), ("f32", 2000)):
        for _ in range(2):
            xb.xconv_diag_mfma_rate(dt, iters, scratch)
        torch.cuda.synchronize()
        xb.xconv_prof_enable(True)
        flops = 0.0
        for _ in range(5):
            flops = xb.xconv_diag_mfma_rate(dt, iters, scratch)
        torch.cuda.synchronize()
        xb.xconv_prof_enable(False)
        ms = [m for kid, m in xb.xconv_prof_collect() if xb.xconv_prof_kernel_name(kid) == "mfma_rate_kernel"]
        out["mfma_issue_tflops_" + dt] = flops / (sum(ms) / len(ms) * 1e-3) / 1e12
    out["mfma_issue"] = "xconv_diag_mfma_rate: 4 independent 32x32 accumulators per wave, 2 waves per SIMD, random operand bits"
    return out


def nsets_for(cfg):
    s = elem_bytes(cfg.dtype)
    per_set = (cfg.B * cfg.C_in * cfg.H * cfg.W + cfg.B * cfg.C_out * cfg.Ho * cfg.Wo + cfg.B * cfg.r * cfg.H * cfg.W) * s
    n = int(600e6 // per_set) + 1               # > 2x the 256 MB Infinity Cache in rotation
    return max(3, min(n, 16))


def measure_config(cfg, steps, warmup, dev, with_exact=False, nhwc=False):
    from paper_2106_06998_amd import binding as xb
    L = Layer(cfg, nsets_for(cfg), dev, nhwc)
    ms_step = time_region(L.step, steps, warmup)
    kt, wall_prof = kernel_times(xb, L.step, steps, warmup)
    alg = algorithmic(cfg)
    out = dict(name=cfg.name, dtype=cfg.dtype, ms_per_layer=ms_step, ms_per_layer_with_events=wall_prof,
               kernels_ms=kt, plan=xb.xconv_plan_info(L.desc, xb.XCONV_OP_ESTIMATE),
               act_bytes_saved=alg["act_bytes_saved"], buffer_sets=len(L.sets))
    tp = kt.get("probe_kernel", kt.get("probe_generic_kernel"))
    tc = kt.get("corr_kernel")
    if tp:
        out["probe"] = dict(ms=tp, gbps=alg["probe_bytes"] / tp / 1e6, gflops=alg["probe_flops"] / tp / 1e6,
                            hbm_frac=alg["probe_bytes"] / tp / 1e6 / PEAK_HBM_GBS)
    if tc:
        out["corr"] = dict(ms=tc, gbps=alg["corr_bytes"] / tc / 1e6, gflops=alg["corr_flops"] / tc / 1e6,
                           hbm_frac=alg["corr_bytes"] / tc / 1e6 / PEAK_HBM_GBS,
                           mfma_frac=alg["corr_flops"] / tc / 1e9 / PEAK_MFMA_TFLOPS[cfg.dtype])
    if with_exact:
        ms_x = time_region(L.exact, max(steps // 4, 5), max(warmup // 4, 2))
        out["exact_ms"] = ms_x
        out["exact_gflops"] = alg["exact_flops"] / ms_x / 1e6
        out["estimate_vs_exact_speedup"] = ms_x / ms_step
        # the rest of the layer on the library's own kernels (forward convolution, exact input gradient)
        if not nhwc:
            import torch
            td = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[cfg.dtype]
            Wd = (torch.randn(cfg.C_out, cfg.C_in, cfg.k, cfg.k, device=dev) / (cfg.C_in * cfg.k * cfg.k) ** 0.5).to(td)
            Yd = torch.empty((cfg.B, cfg.C_out, cfg.Ho, cfg.Wo), dtype=td, device=dev)
            dXd = torch.empty((cfg.B, cfg.C_in, cfg.H, cfg.W), dtype=td, device=dev)
            n_fast = max(steps // 10, 3)
            ms_f = time_region(lambda i: xb.xconv_conv_fwd(L.desc, L.sets[i % len(L.sets)]["X"], Wd, Yd), n_fast, 2)
            ms_b = time_region(lambda i: xb.xconv_dx_exact(L.desc, L.sets[i % len(L.sets)]["dY"], Wd, dXd), n_fast, 2)
            out["conv_fwd_ms"], out["dx_exact_ms"] = ms_f, ms_b
            out["conv_fwd_gflops"] = alg["exact_flops"] / ms_f / 1e6
            out["dx_exact_gflops"] = alg["exact_flops"] / ms_b / 1e6
        # the framework's own exact weight gradient on the same tensors (MIOpen through torch), for context only
        if not nhwc:
            try:
                import torch

                def lib_dw(i):
                    s = L.sets[i % len(L.sets)]
                    torch.nn.grad.conv2d_weight(s["X"], (cfg.C_out, cfg.C_in, cfg.k, cfg.k), s["dY"], stride=cfg.stride, padding=cfg.pad)

                out["torch_exact_dw_ms"] = time_region(lib_dw, max(steps // 4, 5), max(warmup // 4, 3))
            except Exception as e:      # a missing or failing library kernel must not break the benchmark line
                out["torch_exact_dw_ms"] = None
                out["torch_exact_dw_error"] = str(e)[:200]
    return out, L


def host_cpu():
    """(logical cores of the host, CPU model string), read at run time."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return os.cpu_count() or 0, model


def cpu_baseline(cfg, host, budget_s=15.0):
    """The CPU oracle, as it stands (plain C, one thread), on a bounded sample of the same layer: the
    first `Bs` images of the batch, `Bs` chosen from a one-image trial so that the sample takes about
    `budget_s` seconds (the oracle's work is linear in the batch), the time scaled to the whole batch."""
    from oracle import xconv_oracle as xo
    X, dY = host
    Z = xo.probe_matrix({"rademacher": xo.RADEMACHER, "gaussian": xo.GAUSSIAN}[cfg.probe], cfg.seeds[2], cfg.C_in, cfg.r)
    dt = {"f32": xo.F32, "bf16": xo.BF16, "f16": xo.F16}[cfg.dtype]
    st, pd = (cfg.stride, cfg.stride), (cfg.pad, cfg.pad)

    def run(nb):
        t0 = time.perf_counter()
        Xt = xo.probe_fwd(X[:nb], Z, dt)
        xo.dw_from_xt(dY[:nb], Xt, Z, cfg.k, cfg.k, st, pd)
        return time.perf_counter() - t0

    t1 = run(1)
    Bs = max(1, min(cfg.B, int(budget_s / max(t1, 1e-6))))
    t = run(Bs)
    ncores, model = host_cpu()
    return dict(value=t * cfg.B / Bs * 1e3, unit="ms/layer", cores=1, kind="oracle", host_cores=ncores, host_cpu=model,
                sample_seconds=t, sample_images=Bs,
                sample="images 0..%d of the %d of layer %s (probe_fwd + dw_from_xt), one repetition of %.1f s, plain C -O2, one "
                       "thread of the host's %d; value = that time scaled by %d/%d (the oracle's work is linear in the batch)" % (
                           Bs - 1, cfg.B, cfg.name, t, ncores, cfg.B, Bs))


# Volumetric layers (3x3x3 kernels on cubic patches, the regime of the paper's volumetric
# finetuning experiment); not part of the headline metric, measured with --volumetric.
VOLUMES = {
    "V1": dict(B=2, C_in=64, C_out=64, dims=(64, 64, 64), k=3, pad=1, r=16, dtype="f32", probe="gaussian", seeds=(1101, 2101, 3101)),
    "V2": dict(B=1, C_in=128, C_out=128, dims=(48, 48, 48), k=3, pad=1, r=32, dtype="f16", probe="rademacher", seeds=(1102, 2102, 3102)),
}


def measure_volume(name, steps, warmup, dev, with_cpu, with_exact=True):
    import torch
    from paper_2106_06998_amd import binding as xb
    from paper_2106_06998_amd import synth
    c = VOLUMES[name]
    B, C_in, C_out, (D, H, W), k, r, dtype = c["B"], c["C_in"], c["C_out"], c["dims"], c["k"], c["r"], c["dtype"]
    v = xb.make_desc3d(B, C_in, C_out, D, H, W, k, 1, c["pad"], r, dtype, c["probe"], c["seeds"][2])
    X, dY = synth.make_volume(B, C_in, C_out, (D, H, W), (D, H, W), c["seeds"], dtype)
    sets = []
    for _ in range(3):
        sets.append(dict(X=xb.to_device(X, dtype, dev), dY=xb.to_device(dY, dtype, dev),
                         Xt=xb.alloc_bytes(xb.xconv3d_xt_bytes(v), dev),
                         dW=torch.empty((C_out, C_in, k, k, k), dtype=torch.float32, device=dev),
                         ws=xb.alloc_bytes(xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_ESTIMATE), dev)))

    def step(i):
        s = sets[i % len(sets)]
        v.l.seed = c["seeds"][2] + i
        xb.xconv3d_probe_fwd(v, s["X"], s["Xt"], None, s["ws"])
        xb.xconv3d_dw_estimate(v, s["dY"], s["Xt"], None, s["dW"], s["ws"])

    ms_step = time_region(step, steps, warmup)
    kt, _ = kernel_times(xb, step, steps, warmup)
    ms_exact = None
    if with_exact:
        wsx = xb.alloc_bytes(xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_EXACT), dev)

        def exact(i):
            s = sets[i % len(sets)]
            xb.xconv3d_dw_exact(v, s["dY"], s["X"], s["dW"], wsx)

        ms_exact = time_region(exact, max(steps // 4, 5), max(warmup // 4, 2))
    es = elem_bytes(dtype)
    vox = B * D * H * W
    probe_bytes = (C_in + r) * vox * es
    corr_flops = 2.0 * vox * C_out * r * k * k          # one launch: the k*k in-plane offsets of one kernel-depth offset
    corr_bytes = vox * C_out * es + vox * r * es + C_out * r * k * k * 4
    tp, tc = kt.get("probe_kernel", kt.get("probe_generic_kernel")), kt["corr_kernel"]
    out = dict(name=name, dtype=dtype, ms_per_layer=ms_step, kernels_ms=kt,
               probe=dict(ms=tp, gbps=probe_bytes / tp / 1e6, hbm_frac=probe_bytes / tp / 1e6 / PEAK_HBM_GBS),
               corr=dict(ms=tc, launches_per_layer=k, gflops=corr_flops / tc / 1e6, gbps=corr_bytes / tc / 1e6,
                         mfma_frac=corr_flops / tc / 1e9 / PEAK_MFMA_TFLOPS[dtype]),
               act_bytes_saved=(C_in - r) * vox * es, exact_ms=ms_exact, estimate_vs_exact_speedup=(ms_exact / ms_step if ms_exact else None),
               workload="%s: B=%d C_in=%d C_out=%d D=H=W=%d k=%dx%dx%d pad=%d r=%d %s probes, %s storage, NCDHW" % (
                   name, B, C_in, C_out, D, k, k, k, c["pad"], r, c["probe"], dtype))
    if with_cpu:
        # the oracle on the whole layer, once
        from oracle import xconv_oracle as xo
        Xs, dYs = X, dY
        Z = xo.probe_matrix({"rademacher": xo.RADEMACHER, "gaussian": xo.GAUSSIAN}[c["probe"]], c["seeds"][2], C_in, r)
        t0 = time.perf_counter()
        Xt = xo.probe_fwd3d(Xs, Z, {"f32": xo.F32, "bf16": xo.BF16, "f16": xo.F16}[dtype])
        xo.dw_from_xt3d(dYs, Xt, Z, (k, k, k), (1, 1, 1), (c["pad"],) * 3)
        t = time.perf_counter() - t0
        out["cpu_baseline"] = dict(value=t * 1e3, unit="ms/layer", cores=1, kind="oracle",
                                   sample="full %s layer (probe_fwd3d + dw_from_xt3d), 1 repetition, plain C -O2, one thread" % name)
    return out, corr_flops, corr_bytes

def measure_pixel(cfg, steps, warmup, dev, with_cpu, indep=False):
    """The estimator with probing vectors over pixels and channels on a benchmark layer: forward and
    backward timed separately (they run in different passes of training), kernels by HIP events.
    indep: independent probing (xconv_pixel_indep_*), r vectors per input channel."""
    import torch
    from paper_2106_06998_amd import binding as xb
    from paper_2106_06998_amd import synth
    d = xb.desc_from_config(cfg)
    X, dY = synth.make_layer(cfg)
    ws_bytes = xb.xconv_pixel_indep_workspace_bytes if indep else xb.xconv_pixel_workspace_bytes
    probe_fwd = xb.xconv_pixel_indep_probe_fwd if indep else xb.xconv_pixel_probe_fwd
    dw_estimate = xb.xconv_pixel_indep_dw_estimate if indep else xb.xconv_pixel_dw_estimate
    nvec = cfg.C_in * cfg.r if indep else cfg.r            # stored values per image
    if ws_bytes(d, xb.XCONV_OP_ESTIMATE) == 0:
        raise SystemExit("bench.py: %s with r=%d is outside what this mode supports (independent probing: C_in*r <= 65536)" % (cfg.name, cfg.r))
    sets = []
    for _ in range(3):
        sets.append(dict(X=xb.to_device(X, cfg.dtype, dev), dY=xb.to_device(dY, cfg.dtype, dev),
                         xbar=torch.empty((cfg.B, nvec), dtype=torch.float32, device=dev),
                         dW=torch.empty((cfg.C_out, cfg.C_in, cfg.k, cfg.k), dtype=torch.float32, device=dev),
                         wsf=xb.alloc_bytes(ws_bytes(d, xb.XCONV_OP_PROBE), dev),
                         wsb=xb.alloc_bytes(ws_bytes(d, xb.XCONV_OP_ESTIMATE), dev)))

    def fwd(i):
        s = sets[i % len(sets)]
        d.seed = cfg.seeds[2] + i
        probe_fwd(d, s["X"], s["xbar"], s["wsf"])

    def bwd(i):
        s = sets[i % len(sets)]
        d.seed = cfg.seeds[2] + i
        dw_estimate(d, s["dY"], s["xbar"], s["dW"], s["wsb"])

    def both(i):
        fwd(i)
        bwd(i)

    ms_step = time_region(both, steps, warmup)
    kf, ms_f = kernel_times(xb, fwd, steps, warmup)
    kb, ms_b = kernel_times(xb, bwd, steps, warmup)
    es = elem_bytes(cfg.dtype)
    K = cfg.C_in * cfg.H * cfg.W
    fwd_bytes = cfg.B * K * es + cfg.B * nvec * 4
    bwd_flops = 2.0 * cfg.r * cfg.Ho * cfg.Wo * cfg.C_out * cfg.C_in * cfg.k * cfg.k
    out = dict(name=cfg.name, dtype=cfg.dtype, ms_per_layer=ms_step, fwd_ms_with_events=ms_f, bwd_ms_with_events=ms_b,
               fwd_kernels_ms=kf, bwd_kernels_ms=kb,
               fwd=dict(gbps=fwd_bytes / (sum(kf.values())) / 1e6),
               bwd=dict(shifted_product_gflops=bwd_flops / kb["corr_kernel"] / 1e6,
                        mfma_frac=bwd_flops / kb["corr_kernel"] / 1e9 / PEAK_MFMA_TFLOPS[cfg.dtype]),
               stored_bytes=cfg.B * nvec * 4, act_bytes=cfg.B * K * es,
               workload="%s: B=%d C_in=%d C_out=%d H=W=%d k=%d stride=%d pad=%d r=%d %s probes over %s, %s storage" % (
                   cfg.name, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.probe,
                   "the pixels of every input channel on its own (independent probing)" if indep else "pixels and channels", cfg.dtype))
    if with_cpu and indep:
        from oracle import xconv_oracle as xo
        dt = {"f32": xo.F32, "bf16": xo.BF16, "f16": xo.F16}[cfg.dtype]
        t0 = time.perf_counter()
        Z = xo.pixel_probe_matrix({"rademacher": xo.RADEMACHER, "gaussian": xo.GAUSSIAN}[cfg.probe], cfg.seeds[2], cfg.C_in, cfg.H,
                                  cfg.W, cfg.r)
        xbar = xo.pixel_indep_probe_fwd(X, Z)
        xo.pixel_indep_dw_estimate(dY, xbar, Z, cfg.C_in, cfg.H, cfg.W, cfg.k, cfg.k, (cfg.stride, cfg.stride), (cfg.pad, cfg.pad))
        t = time.perf_counter() - t0
        out["cpu_baseline"] = dict(value=t * 1e3, unit="ms/layer", cores=1, kind="oracle",
                                   sample="full %s layer (pixel_probe_matrix + pixel_indep_probe_fwd + pixel_indep_dw_estimate), "
                                          "1 repetition, plain C -O2, one thread" % cfg.name)
    elif with_cpu:
        from oracle import xconv_oracle as xo
        dt = {"f32": xo.F32, "bf16": xo.BF16, "f16": xo.F16}[cfg.dtype]
        t0 = time.perf_counter()
        Z = xo.pixel_probe_matrix({"rademacher": xo.RADEMACHER, "gaussian": xo.GAUSSIAN}[cfg.probe], cfg.seeds[2], cfg.C_in, cfg.H,
                                  cfg.W, cfg.r)
        xbar = xo.pixel_probe_fwd(X, Z)
        xo.pixel_dw_estimate(dY, xbar, Z, cfg.C_in, cfg.H, cfg.W, cfg.k, cfg.k, (cfg.stride, cfg.stride), (cfg.pad, cfg.pad))
        t = time.perf_counter() - t0
        out["cpu_baseline"] = dict(value=t * 1e3, unit="ms/layer", cores=1, kind="oracle",
                                   sample="full %s layer (pixel_probe_matrix + pixel_probe_fwd + pixel_dw_estimate), 1 repetition, "
                                          "plain C -O2, one thread" % cfg.name)
    return out, bwd_flops

def measure_network(steps, warmup, dev, layers=12, B=128, C=64, HW=32, r=16, dtype="f32", probe="gaussian"):
    """Forward + backward of a stack of 3x3 convolutions and ReLUs (the geometry of layer C2), with torch's layers
    and with the layers swapped by convert_net: time per step, peak memory above the resident tensors, and the bytes
    autograd keeps for the backward pass."""
    import torch
    from paper_2106_06998_amd.layer import convert_net

    def build():
        torch.manual_seed(11)
        mods = []
        for _ in range(layers):
            mods += [torch.nn.Conv2d(C, C, 3, padding=1), torch.nn.ReLU()]
        return torch.nn.Sequential(*mods).to(dev).to(td)

    td = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    x = torch.randn(B, C, HW, HW, device=dev).relu_().to(td)
    out = {}
    # "channel", "multi": everything on the library's kernels (engine="library": forward convolution, input gradient, probe,
    # estimate); "*_framework_conv": the forward convolution and the input gradient on torch's operators instead
    for name, kw in (("torch", None), ("channel", dict(r=r, mode="channel", relu=True, probe=probe)),
                     ("multi", dict(r=r, mode="multi", relu=True, probe=probe)),
                     ("channel_framework_conv", dict(r=r, mode="channel", relu=True, probe=probe, engine="framework")),
                     ("multi_framework_conv", dict(r=r, mode="multi", relu=True, probe=probe, engine="framework"))):
        net = build()
        if kw:
            net, n = convert_net(net, **kw)
            assert n == layers

        def step():
            net.zero_grad(set_to_none=True)
            net(x).float().mean().backward()

        seen, params = {}, {p.data_ptr() for p in net.parameters()}

        def pack(t):
            if t.data_ptr() not in params:
                seen[t.data_ptr()] = t.numel() * t.element_size()
            return t

        with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
            y = net(x)
        y.float().mean().backward()
        del y
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        base = torch.cuda.memory_allocated()
        torch.cuda.reset_peak_memory_stats()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        out[name] = dict(ms_per_step=ms, peak_bytes_above_resident=torch.cuda.max_memory_allocated() - base,
                         saved_bytes=sum(seen.values()))
        del net
    out["workload"] = "%d x [Conv2d(%d, %d, 3, padding=1) + ReLU], B=%d, %dx%d, %s, r=%d %s probes" % (layers, C, C, B, HW, HW, dtype, r, probe)
    return out


def measure_accuracy(cfg, dev, rs=(4, 8, 16, 32, 64), seeds=8):
    """Relative error ||dW_est - dW_exact|| / ||dW_exact|| of one draw (root mean square over `seeds` draws) against
    the number of probing vectors, for the three probing modes on one layer (the paper's gradient-error-against-r
    experiment on synthetic tensors); the exact gradient is xconv_dw_exact."""
    import dataclasses
    import torch
    from paper_2106_06998_amd import binding as xb
    from paper_2106_06998_amd import synth
    X, dY = synth.make_layer(cfg)
    Xd, dYd = xb.to_device(X, cfg.dtype, dev), xb.to_device(dY, cfg.dtype, dev)
    dW = torch.empty((cfg.C_out, cfg.C_in, cfg.k, cfg.k), dtype=torch.float32, device=dev)
    d0 = xb.desc_from_config(cfg)
    ex = torch.empty_like(dW)
    xb.xconv_dw_exact(d0, dYd, Xd, ex, xb.alloc_ws(d0, xb.XCONV_OP_EXACT, dev))
    ex = ex.double()
    out = {"r": list(rs), "channel": [], "multi": [], "independent": [], "state_bytes": {"channel": [], "multi": [], "independent": []}}
    for r in rs:
        d = xb.desc_from_config(dataclasses.replace(cfg, r=r))
        for mode in ("channel", "multi", "independent"):
            if mode == "channel":
                state = xb.alloc_xt(d, dev)
                wsp, wse = xb.alloc_ws(d, xb.XCONV_OP_PROBE, dev), xb.alloc_ws(d, xb.XCONV_OP_ESTIMATE, dev)
                nbytes = cfg.B * r * cfg.H * cfg.W * elem_bytes(cfg.dtype)
            else:
                ind = mode == "independent"
                nbytes = (xb.xconv_pixel_indep_xbar_bytes if ind else xb.xconv_pixel_xbar_bytes)(d)
                wsb = xb.xconv_pixel_indep_workspace_bytes if ind else xb.xconv_pixel_workspace_bytes
                state = torch.empty(max(nbytes // 4, 1), dtype=torch.float32, device=dev)
                wsp, wse = xb.alloc_bytes(wsb(d, xb.XCONV_OP_PROBE), dev), xb.alloc_bytes(wsb(d, xb.XCONV_OP_ESTIMATE), dev)
            if nbytes == 0:
                out[mode].append(None)
                out["state_bytes"][mode].append(None)
                continue
            acc = 0.0
            for s in range(seeds):
                d.seed = 910000 + 97 * r + s
                if mode == "channel":
                    xb.xconv_probe_fwd(d, Xd, state, None, wsp)
                    xb.xconv_dw_estimate(d, dYd, state, None, dW, wse)
                elif mode == "multi":
                    xb.xconv_pixel_probe_fwd(d, Xd, state, wsp)
                    xb.xconv_pixel_dw_estimate(d, dYd, state, dW, wse)
                else:
                    xb.xconv_pixel_indep_probe_fwd(d, Xd, state, wsp)
                    xb.xconv_pixel_indep_dw_estimate(d, dYd, state, dW, wse)
                acc += float(((dW.double() - ex).norm() / ex.norm()) ** 2)
            out[mode].append((acc / seeds) ** 0.5)
            out["state_bytes"][mode].append(nbytes)
    out["act_bytes"] = cfg.B * cfg.C_in * cfg.H * cfg.W * elem_bytes(cfg.dtype)
    return out


def workload_string(cfg, nhwc):
    return "%s: B=%d C_in=%d C_out=%d H=W=%d k=%d stride=%d pad=%d r=%d %s probes, %s storage, %s" % (
        cfg.name, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.probe, cfg.dtype,
        "NHWC" if nhwc else "NCHW")


CORR_KERNEL_NAMES = {0: "corr_kernel", 1: "corr_ws_kernel", 2: "corr_ws32_kernel", 3: "corr_row_kernel"}


def roofline_of(cfg, res):
    """Roofline object of the correlation launch (the dominant kernel of every layer): the matrix-core peak
    of the storage type, or HBM when the layer's algorithmic bytes take longer at 8 TB/s than its flops at
    that peak.  `achieved` = algorithmic flops (bytes) of the one launch / its event-timed duration."""
    alg = algorithmic(cfg)
    c = res["corr"]
    kname = CORR_KERNEL_NAMES[res["plan"].get("ws", 0)]
    mfma_bound = (alg["corr_flops"] / (PEAK_MFMA_TFLOPS[cfg.dtype] * 1e12)) >= (alg["corr_bytes"] / (PEAK_HBM_GBS * 1e9))
    if mfma_bound:
        ach = c["gflops"] / 1e3
        roof = dict(bound="mfma", achieved=ach, peak=PEAK_MFMA_TFLOPS[cfg.dtype], unit="TFLOP/s", frac=ach / PEAK_MFMA_TFLOPS[cfg.dtype])
    else:
        roof = dict(bound="hbm", achieved=c["gbps"], peak=PEAK_HBM_GBS, unit="GB/s", frac=c["gbps"] / PEAK_HBM_GBS)
    roof.update(kernel=kname, kernel_ms=c["ms"], traffic=MEASURED_TRAFFIC.get((cfg.name, kname)),
                mfma_frac=c["mfma_frac"], hbm_frac=c["hbm_frac"])
    return roof


def probe_roofline_of(cfg, res):
    p = res["probe"]
    return dict(bound="hbm", achieved=p["gbps"], peak=PEAK_HBM_GBS, unit="GB/s", frac=p["hbm_frac"], kernel="probe_kernel",
                kernel_ms=p["ms"], traffic=MEASURED_TRAFFIC.get((cfg.name, "probe_kernel")))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C5",
                    help="layer the headline value is quoted on (default: C5, the largest layer, the one the roofline bars are stated on)")
    ap.add_argument("--headline-only", action="store_true", help="do not measure the other four benchmark layers (field per_config)")
    ap.add_argument("--nhwc", action="store_true", help="hand X and dY over channels-last (layout XCONV_NHWC) instead of NCHW")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-exact", action="store_true", help="skip timing xconv_dw_exact (for clean per-kernel profiles)")
    ap.add_argument("--volumetric", action="store_true",
                    help="measure the volumetric (3-D convolution) layers V1 and V2 instead of the headline layer")
    ap.add_argument("--pixel-probe", action="store_true",
                    help="measure the estimator with probing vectors over pixels and channels (xconv_pixel_*) on --config instead")
    ap.add_argument("--independent", action="store_true",
                    help="with --pixel-probe: independent probing (xconv_pixel_indep_*), r probing vectors per input channel")
    ap.add_argument("--r", type=int, default=0, help="with --pixel-probe: number of probing vectors instead of the layer's own")
    ap.add_argument("--accuracy", action="store_true",
                    help="error of the dW estimate against the number of probing vectors for the three probing modes on --config")
    ap.add_argument("--network", action="store_true",
                    help="forward + backward of a stack of convolutions and ReLUs, torch's layers against XConv2d + SignReLU")
    ap.add_argument("--net-probe", default="gaussian", choices=["gaussian", "rademacher"], help="with --network: probe distribution")
    ap.add_argument("--net-dtype", default="f32", choices=["f32", "bf16", "f16"], help="with --network: storage type of the stack")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of 256 MiB ten times (reference reading for the FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU part in this build (got --gpus %d)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2106_06998_amd import binding as xb
    from paper_2106_06998_amd import synth
    xb.lib()                                     # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = "cuda:0"
    if args.copy_calibration:
        src = torch.full((64 * 2 ** 20,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        flush = torch.empty((128 * 2 ** 20,), dtype=torch.float32, device=dev)
        for _ in range(10):
            flush.fill_(0.0)          # push src/dst out of the Infinity Cache between copies
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4, "copies": 10}))
        return 0
    if args.volumetric:
        res, flops, nbytes = measure_volume("V1", args.steps, args.warmup, dev, not args.no_cpu, not args.no_exact)
        ach = res["corr"]["gflops"] / 1e3
        line = {
            "metric": "ms/layer for the XConv dW estimate of a 3-D layer (xconv3d_probe_fwd + xconv3d_dw_estimate), 1 GPU",
            "value": res["ms_per_layer"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": res["ms_per_layer"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": res["dtype"], "data": "synthetic", "config": {"workload": res["workload"]},
            "roofline": dict(bound="mfma", achieved=ach, peak=PEAK_MFMA_TFLOPS[res["dtype"]], unit="TFLOP/s",
                             frac=ach / PEAK_MFMA_TFLOPS[res["dtype"]], kernel="corr_ws32_kernel", kernel_ms=res["corr"]["ms"],
                             traffic=None),
            "detail": res,
        }
        if "cpu_baseline" in res:
            line["cpu_baseline"] = res.pop("cpu_baseline")
        torch.cuda.empty_cache()
        r2, _, _ = measure_volume("V2", max(args.steps // 2, 10), max(args.warmup // 2, 3), dev, False, not args.no_exact)
        line["per_config"] = [r2]
        print(json.dumps(line))
        return 0
    if args.accuracy:
        cfg = synth.CONFIGS[args.config]
        res = measure_accuracy(cfg, dev)
        i16 = res["r"].index(16)
        line = {
            "metric": "relative error of one draw of the dW estimate at r=16 (channel probes), 1 GPU", "value": res["channel"][i16],
            "unit": "relative L2 error", "n_gpus": 1, "steps": 8, "warmup": 0, "ms_per_step": None, "higher_is_better": False,
            "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": "%s: B=%d C_in=%d C_out=%d H=W=%d k=%d stride=%d pad=%d, %s probes, %s storage, r swept" % (
                cfg.name, cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.k, cfg.stride, cfg.pad, cfg.probe, cfg.dtype)},
            "detail": res,
        }
        print(json.dumps(line))
        return 0
    if args.network:
        res = measure_network(min(args.steps, 30), min(args.warmup, 5), dev, dtype=args.net_dtype, probe=args.net_probe)
        line = {
            "metric": "ms/step (forward + backward) of a convolution + ReLU stack with XConv2d (channel probes) and SignReLU, 1 GPU",
            "value": res["channel"]["ms_per_step"], "unit": "ms", "n_gpus": 1, "steps": min(args.steps, 30), "warmup": min(args.warmup, 5),
            "ms_per_step": res["channel"]["ms_per_step"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": args.net_dtype, "data": "synthetic", "config": {"workload": res.pop("workload")}, "detail": res,
        }
        print(json.dumps(line))
        return 0
    if args.pixel_probe:
        cfg = synth.CONFIGS[args.config]
        if args.r > 0:
            import dataclasses
            cfg = dataclasses.replace(cfg, r=args.r)
        res, flops = measure_pixel(cfg, args.steps, args.warmup, dev, not args.no_cpu, indep=args.independent)
        tc = res["bwd_kernels_ms"]["corr_kernel"]
        ach = flops / tc / 1e9
        line = {
            "metric": ("ms/layer for the XConv dW estimate with independent probing (xconv_pixel_indep_probe_fwd + "
                       "xconv_pixel_indep_dw_estimate), 1 GPU") if args.independent else
                      "ms/layer for the XConv dW estimate with probes over pixels and channels (xconv_pixel_probe_fwd + xconv_pixel_dw_estimate), 1 GPU",
            "value": res["ms_per_layer"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": res["ms_per_layer"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": cfg.dtype, "data": "synthetic", "config": {"workload": res["workload"]},
            "roofline": dict(bound="mfma", achieved=ach, peak=PEAK_MFMA_TFLOPS[cfg.dtype], unit="TFLOP/s",
                             frac=ach / PEAK_MFMA_TFLOPS[cfg.dtype], kernel="shifted product (correlation kernel of the backward pass)",
                             kernel_ms=tc, traffic=None),
            "detail": res,
        }
        if "cpu_baseline" in res:
            line["cpu_baseline"] = res.pop("cpu_baseline")
        print(json.dumps(line))
        return 0
    cfg = synth.CONFIGS[args.config]
    res, L = measure_config(cfg, args.steps, args.warmup, dev, with_exact=not args.no_exact, nhwc=args.nhwc)
    alg = algorithmic(cfg)
    line = {
        "metric": "ms/layer for the XConv dW estimate (xconv_probe_fwd + xconv_dw_estimate), 1 GPU",
        "value": res["ms_per_layer"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_layer"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload_string(cfg, args.nhwc)},
        "gbps": (alg["probe_bytes"] + alg["corr_bytes"]) / res["ms_per_layer"] / 1e6,
        "gflops": (alg["probe_flops"] + alg["corr_flops"]) / res["ms_per_layer"] / 1e6,
        "roofline": roofline_of(cfg, res),
        "probe_roofline": probe_roofline_of(cfg, res),
        "detail": res,
    }
    # the same fractions against what plain reference kernels reach on this machine (context: the headline fractions above are
    # against the published peaks)
    mr = machine_rates(xb, dev)
    line["machine"] = mr

    def against_measured(rf, pf, dtype):
        ref = mr["hbm_copy_gbps"] if rf["bound"] == "hbm" else mr["mfma_issue_tflops_" + ("f32" if dtype == "f32" else "f16")]
        rf["frac_of_measured"] = rf["achieved"] / ref
        pf["frac_of_measured"] = pf["achieved"] / mr["hbm_copy_gbps"]

    against_measured(line["roofline"], line["probe_roofline"], cfg.dtype)
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(cfg, L.host)
    del L
    if not args.headline_only:
        per = []
        for name, c in synth.CONFIGS.items():
            if name == cfg.name:
                continue
            torch.cuda.empty_cache()
            r, Lc = measure_config(c, max(args.steps // 2, 10), max(args.warmup // 2, 3), dev, with_exact=False)
            del Lc
            r["workload"] = workload_string(c, False)
            r["roofline"] = roofline_of(c, r)
            r["probe_roofline"] = probe_roofline_of(c, r)
            against_measured(r["roofline"], r["probe_roofline"], c.dtype)
            per.append(r)
        line["per_config"] = per
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
