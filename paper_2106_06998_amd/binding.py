"""Thin ctypes binding of libxconv (include/xconv.h): argument marshalling only.

Every function has the name and the argument order of its C entry point.
Device buffers are torch tensors on a ROCm device (or raw integer addresses);
the stream defaults to torch's current stream.  Nothing here computes: all
arithmetic runs in the HIP kernels of the library.  If the library has not been
built the first call raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("XCONV_LIB", os.path.join(_HERE, "libxconv.so"))   # override: A/B runs of two builds

XCONV_OK, XCONV_EINVAL, XCONV_EUNSUPPORTED, XCONV_EWORKSPACE, XCONV_EHIP = range(5)
XCONV_F32, XCONV_BF16, XCONV_F16 = 0, 1, 2
XCONV_NCHW, XCONV_NHWC = 0, 1
XCONV_RADEMACHER, XCONV_GAUSSIAN, XCONV_USER_Z = 0, 1, 2
XCONV_OP_PROBE, XCONV_OP_ESTIMATE, XCONV_OP_EXACT = 0, 1, 2

DTYPES = {"f32": XCONV_F32, "bf16": XCONV_BF16, "f16": XCONV_F16}
PROBES = {"rademacher": XCONV_RADEMACHER, "gaussian": XCONV_GAUSSIAN, "user": XCONV_USER_Z}


class xconv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "C_in", "C_out", "H", "W", "kH", "kW", "stride_h", "stride_w", "pad_h", "pad_w",
                 "r", "dtype", "layout", "probe", "keep_q15")] + [("seed", ctypes.c_uint64)]


class xconv3d_desc(ctypes.Structure):
    _fields_ = [("l", xconv_desc), ("D", ctypes.c_int32), ("kD", ctypes.c_int32), ("stride_d", ctypes.c_int32),
                ("pad_d", ctypes.c_int32)]


class XConvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, xconv_status_string(status), status))


_lib = None


def lib():
    """Load libxconv.so; fails loudly when the HIP extension is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libxconv.so is not built (%s). Run `python -m paper_2106_06998_amd.build` "
                "or __graft_entry__.build(); there is no fallback path." % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(xconv_desc)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.xconv_check_desc.restype = i32
        L.xconv_check_desc.argtypes = [P]
        L.xconv_xt_bytes.restype = sz
        L.xconv_xt_bytes.argtypes = [P]
        L.xconv_workspace_bytes.restype = sz
        L.xconv_workspace_bytes.argtypes = [P, i32]
        L.xconv_probe_matrix.restype = i32
        L.xconv_probe_matrix.argtypes = [P, vp]
        L.xconv_probe_matrix_dev.restype = i32
        L.xconv_probe_matrix_dev.argtypes = [P, vp, vp]
        L.xconv_probe_fwd.restype = i32
        L.xconv_probe_fwd.argtypes = [P, vp, vp, vp, vp, sz, vp]
        L.xconv_dw_estimate.restype = i32
        L.xconv_dw_estimate.argtypes = [P, vp, vp, vp, vp, vp, sz, vp]
        L.xconv_dw_exact.restype = i32
        L.xconv_dw_exact.argtypes = [P, vp, vp, vp, vp, sz, vp]
        L.xconv_conv_fwd.restype = i32
        L.xconv_conv_fwd.argtypes = [P, vp, vp, vp, vp]
        L.xconv_dx_exact.restype = i32
        L.xconv_dx_exact.argtypes = [P, vp, vp, vp, vp]
        L.xconv_dw_estimate_static.restype = i32
        L.xconv_dw_estimate_static.argtypes = [P, vp, vp, vp, vp, vp]
        L.xconv_static_scratch_bytes.restype = sz
        L.xconv_static_scratch_bytes.argtypes = []
        L.xconv_plan_info.restype = i32
        L.xconv_plan_info.argtypes = [P, i32, vp]
        L.xconv_xt_unpack.restype = i32
        L.xconv_xt_unpack.argtypes = [P, vp, vp, vp]
        P3 = ctypes.POINTER(xconv3d_desc)
        L.xconv3d_check_desc.restype = i32
        L.xconv3d_check_desc.argtypes = [P3]
        L.xconv3d_xt_bytes.restype = sz
        L.xconv3d_xt_bytes.argtypes = [P3]
        L.xconv3d_workspace_bytes.restype = sz
        L.xconv3d_workspace_bytes.argtypes = [P3, i32]
        L.xconv3d_probe_fwd.restype = i32
        L.xconv3d_probe_fwd.argtypes = [P3, vp, vp, vp, vp, sz, vp]
        L.xconv3d_dw_estimate.restype = i32
        L.xconv3d_dw_estimate.argtypes = [P3, vp, vp, vp, vp, vp, sz, vp]
        L.xconv3d_dw_exact.restype = i32
        L.xconv3d_dw_exact.argtypes = [P3, vp, vp, vp, vp, sz, vp]
        L.xconv3d_xt_unpack.restype = i32
        L.xconv3d_xt_unpack.argtypes = [P3, vp, vp, vp]
        L.xconv_pixel_xbar_bytes.restype = sz
        L.xconv_pixel_xbar_bytes.argtypes = [P]
        L.xconv_pixel_workspace_bytes.restype = sz
        L.xconv_pixel_workspace_bytes.argtypes = [P, i32]
        L.xconv_pixel_probe_fwd.restype = i32
        L.xconv_pixel_probe_fwd.argtypes = [P, vp, vp, vp, sz, vp]
        L.xconv_pixel_dw_estimate.restype = i32
        L.xconv_pixel_dw_estimate.argtypes = [P, vp, vp, vp, vp, sz, vp]
        L.xconv_relu_mask_bytes.restype = sz
        L.xconv_relu_mask_bytes.argtypes = [ctypes.c_longlong]
        L.xconv_relu_fwd.restype = i32
        L.xconv_relu_fwd.argtypes = [i32, vp, vp, vp, ctypes.c_longlong, vp]
        L.xconv_relu_bwd.restype = i32
        L.xconv_relu_bwd.argtypes = [i32, vp, vp, vp, ctypes.c_longlong, vp]
        L.xconv_pixel_indep_xbar_bytes.restype = sz
        L.xconv_pixel_indep_xbar_bytes.argtypes = [P]
        L.xconv_pixel_indep_workspace_bytes.restype = sz
        L.xconv_pixel_indep_workspace_bytes.argtypes = [P, i32]
        L.xconv_pixel_indep_probe_fwd.restype = i32
        L.xconv_pixel_indep_probe_fwd.argtypes = [P, vp, vp, vp, sz, vp]
        L.xconv_pixel_indep_dw_estimate.restype = i32
        L.xconv_pixel_indep_dw_estimate.argtypes = [P, vp, vp, vp, vp, sz, vp]
        L.xconv_diag_mfma_rate.restype = i32
        L.xconv_diag_mfma_rate.argtypes = [i32, i32, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
        L.xconv_prof_enable.restype = None
        L.xconv_prof_enable.argtypes = [i32]
        L.xconv_prof_collect.restype = i32
        L.xconv_prof_collect.argtypes = [vp, vp, i32]
        L.xconv_prof_kernel_name.restype = ctypes.c_char_p
        L.xconv_prof_kernel_name.argtypes = [i32]
        L.xconv_status_string.restype = ctypes.c_char_p
        L.xconv_status_string.argtypes = [i32]
        _lib = L
    return _lib


def make_desc(B, C_in, C_out, H, W, k, stride=1, pad=0, r=1, dtype="f32", probe="rademacher", seed=0, layout=XCONV_NCHW,
              keep_q15=0):
    kH, kW = (k, k) if isinstance(k, int) else k
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return xconv_desc(B, C_in, C_out, H, W, kH, kW, sh, sw, ph, pw, r,
                      DTYPES[dtype] if isinstance(dtype, str) else dtype, layout,
                      PROBES[probe] if isinstance(probe, str) else probe, keep_q15, seed)


def desc_from_config(cfg, seed=None):
    """xconv_desc of a synth.LayerConfig (Z seed = cfg.seeds[2] unless given)."""
    return make_desc(cfg.B, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.k, cfg.stride, cfg.pad, cfg.r, cfg.dtype, cfg.probe,
                     cfg.seeds[2] if seed is None else seed)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _check(status, where):
    if status != XCONV_OK:
        raise XConvError(status, where)


def xconv_status_string(status):
    return lib().xconv_status_string(int(status)).decode()


def xconv_check_desc(desc):
    return int(lib().xconv_check_desc(ctypes.byref(desc)))


def xconv_xt_bytes(desc):
    return int(lib().xconv_xt_bytes(ctypes.byref(desc)))


def xconv_workspace_bytes(desc, op):
    return int(lib().xconv_workspace_bytes(ctypes.byref(desc), int(op)))


def xconv_probe_matrix(desc):
    Z = np.empty((desc.C_in, desc.r), dtype=np.float32)
    _check(lib().xconv_probe_matrix(ctypes.byref(desc), ctypes.c_void_p(Z.ctypes.data)), "xconv_probe_matrix")
    return Z


def xconv_probe_matrix_dev(desc, Z_dev, stream=None):
    _check(lib().xconv_probe_matrix_dev(ctypes.byref(desc), _ptr(Z_dev), _stream(stream)), "xconv_probe_matrix_dev")


def xconv_probe_fwd(desc, X_dev, Xt_dev, Z_dev=None, ws_dev=None, stream=None):
    _check(lib().xconv_probe_fwd(ctypes.byref(desc), _ptr(X_dev), _ptr(Xt_dev), _ptr(Z_dev), _ptr(ws_dev),
                                 _nbytes(ws_dev), _stream(stream)), "xconv_probe_fwd")


def xconv_dw_estimate(desc, dY_dev, Xt_dev, Z_dev, dW_dev, ws_dev, stream=None):
    _check(lib().xconv_dw_estimate(ctypes.byref(desc), _ptr(dY_dev), _ptr(Xt_dev), _ptr(Z_dev), _ptr(dW_dev),
                                   _ptr(ws_dev), _nbytes(ws_dev), _stream(stream)), "xconv_dw_estimate")


def xconv_conv_fwd(desc, X_dev, W_dev, Y_dev, stream=None):
    _check(lib().xconv_conv_fwd(ctypes.byref(desc), _ptr(X_dev), _ptr(W_dev), _ptr(Y_dev), _stream(stream)), "xconv_conv_fwd")


def xconv_dx_exact(desc, dY_dev, W_dev, dX_dev, stream=None):
    _check(lib().xconv_dx_exact(ctypes.byref(desc), _ptr(dY_dev), _ptr(W_dev), _ptr(dX_dev), _stream(stream)), "xconv_dx_exact")


def xconv_dw_estimate_static(desc, dY_dev, Xt_dev, Z_dev, dW_dev, stream=None):
    _check(lib().xconv_dw_estimate_static(ctypes.byref(desc), _ptr(dY_dev), _ptr(Xt_dev), _ptr(Z_dev), _ptr(dW_dev),
                                          _stream(stream)), "xconv_dw_estimate_static")


def xconv_static_scratch_bytes():
    return int(lib().xconv_static_scratch_bytes())


def xconv_dw_exact(desc, dY_dev, X_dev, dW_dev, ws_dev, stream=None):
    _check(lib().xconv_dw_exact(ctypes.byref(desc), _ptr(dY_dev), _ptr(X_dev), _ptr(dW_dev), _ptr(ws_dev),
                                _nbytes(ws_dev), _stream(stream)), "xconv_dw_exact")


PLAN_FIELDS = ("S", "NS", "RB", "CW", "WM", "WJ", "WK", "M_WG", "J_WG", "lds_bytes", "NTM", "NTJ", "NOG", "CS", "NCHR", "ws")


def xconv_plan_info(desc, op):
    out = (ctypes.c_int32 * 16)()
    _check(lib().xconv_plan_info(ctypes.byref(desc), int(op), ctypes.cast(out, ctypes.c_void_p)), "xconv_plan_info")
    return dict(zip(PLAN_FIELDS, [int(v) for v in out]))


def xconv_xt_unpack(desc, Xt_dev, out_dev, stream=None):
    _check(lib().xconv_xt_unpack(ctypes.byref(desc), _ptr(Xt_dev), _ptr(out_dev), _stream(stream)), "xconv_xt_unpack")


# ---- volumetric layers ---------------------------------------------------------
def make_desc3d(B, C_in, C_out, D, H, W, k, stride=1, pad=0, r=1, dtype="f32", probe="rademacher", seed=0, keep_q15=0,
                layout=XCONV_NCHW):
    """k, stride and pad are (depth, height, width) triples or one int for all three; layout XCONV_NHWC means
    channels-last volumes [B, D, H, W, C]."""
    kD, kH, kW = (k, k, k) if isinstance(k, int) else k
    sd, sh, sw = (stride, stride, stride) if isinstance(stride, int) else stride
    pd, ph, pw = (pad, pad, pad) if isinstance(pad, int) else pad
    return xconv3d_desc(make_desc(B, C_in, C_out, H, W, (kH, kW), (sh, sw), (ph, pw), r, dtype, probe, seed, layout, keep_q15),
                        D, kD, sd, pd)


def xconv3d_check_desc(desc):
    return int(lib().xconv3d_check_desc(ctypes.byref(desc)))


def xconv3d_xt_bytes(desc):
    return int(lib().xconv3d_xt_bytes(ctypes.byref(desc)))


def xconv3d_workspace_bytes(desc, op):
    return int(lib().xconv3d_workspace_bytes(ctypes.byref(desc), int(op)))


def xconv3d_probe_fwd(desc, X_dev, Xt_dev, Z_dev=None, ws_dev=None, stream=None):
    _check(lib().xconv3d_probe_fwd(ctypes.byref(desc), _ptr(X_dev), _ptr(Xt_dev), _ptr(Z_dev), _ptr(ws_dev),
                                   _nbytes(ws_dev), _stream(stream)), "xconv3d_probe_fwd")


def xconv3d_dw_estimate(desc, dY_dev, Xt_dev, Z_dev, dW_dev, ws_dev, stream=None):
    _check(lib().xconv3d_dw_estimate(ctypes.byref(desc), _ptr(dY_dev), _ptr(Xt_dev), _ptr(Z_dev), _ptr(dW_dev),
                                     _ptr(ws_dev), _nbytes(ws_dev), _stream(stream)), "xconv3d_dw_estimate")


def xconv3d_dw_exact(desc, dY_dev, X_dev, dW_dev, ws_dev, stream=None):
    _check(lib().xconv3d_dw_exact(ctypes.byref(desc), _ptr(dY_dev), _ptr(X_dev), _ptr(dW_dev), _ptr(ws_dev),
                                  _nbytes(ws_dev), _stream(stream)), "xconv3d_dw_exact")


def xconv3d_xt_unpack(desc, Xt_dev, out_dev, stream=None):
    _check(lib().xconv3d_xt_unpack(ctypes.byref(desc), _ptr(Xt_dev), _ptr(out_dev), _stream(stream)), "xconv3d_xt_unpack")


# ---- probing vectors over pixels and channels ---------------------------------------
def xconv_pixel_xbar_bytes(desc):
    return int(lib().xconv_pixel_xbar_bytes(ctypes.byref(desc)))


def xconv_pixel_workspace_bytes(desc, op):
    return int(lib().xconv_pixel_workspace_bytes(ctypes.byref(desc), int(op)))


def xconv_pixel_probe_fwd(desc, X_dev, Xbar_dev, ws_dev, stream=None):
    _check(lib().xconv_pixel_probe_fwd(ctypes.byref(desc), _ptr(X_dev), _ptr(Xbar_dev), _ptr(ws_dev), _nbytes(ws_dev),
                                       _stream(stream)), "xconv_pixel_probe_fwd")


def xconv_pixel_dw_estimate(desc, dY_dev, Xbar_dev, dW_dev, ws_dev, stream=None):
    _check(lib().xconv_pixel_dw_estimate(ctypes.byref(desc), _ptr(dY_dev), _ptr(Xbar_dev), _ptr(dW_dev), _ptr(ws_dev),
                                         _nbytes(ws_dev), _stream(stream)), "xconv_pixel_dw_estimate")


XCONV_DIAG_OUT_BYTES = 8192


def xconv_diag_mfma_rate(dtype, iters, out_dev, stream=None):
    """Enqueues the matrix-instruction issue loop; returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(lib().xconv_diag_mfma_rate(int(DTYPES[dtype]) if isinstance(dtype, str) else int(dtype), int(iters), _ptr(out_dev),
                                      _nbytes(out_dev), ctypes.byref(flops), _stream(stream)), "xconv_diag_mfma_rate")
    return flops.value


def xconv_prof_enable(on):
    lib().xconv_prof_enable(1 if on else 0)


def xconv_prof_collect(max_records=65536):
    ids = (ctypes.c_int32 * max_records)()
    ms = (ctypes.c_float * max_records)()
    n = lib().xconv_prof_collect(ctypes.cast(ids, ctypes.c_void_p), ctypes.cast(ms, ctypes.c_void_p), max_records)
    return [(int(ids[i]), float(ms[i])) for i in range(n)]


def xconv_prof_kernel_name(kernel_id):
    return lib().xconv_prof_kernel_name(int(kernel_id)).decode()


# ---- device-memory plumbing (torch is used for allocation only) --------------
def alloc_bytes(nbytes, device="cuda:0"):
    import torch
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def alloc_xt(desc, device="cuda:0"):
    return alloc_bytes(xconv_xt_bytes(desc), device)


def alloc_ws(desc, op, device="cuda:0"):
    return alloc_bytes(xconv_workspace_bytes(desc, op), device)


def to_device(values_f32, dtype, device="cuda:0"):
    """Upload storage-representable float32 values as a tensor of the storage dtype."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(values_f32, dtype=np.float32))
    td = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    return t.to(td).to(device)


# ---- independent probing: every input channel with probing vectors of its own --------
def xconv_pixel_indep_xbar_bytes(desc):
    return int(lib().xconv_pixel_indep_xbar_bytes(ctypes.byref(desc)))


def xconv_pixel_indep_workspace_bytes(desc, op):
    return int(lib().xconv_pixel_indep_workspace_bytes(ctypes.byref(desc), int(op)))


def xconv_pixel_indep_probe_fwd(desc, X_dev, Xbar_dev, ws_dev, stream=None):
    _check(lib().xconv_pixel_indep_probe_fwd(ctypes.byref(desc), _ptr(X_dev), _ptr(Xbar_dev), _ptr(ws_dev), _nbytes(ws_dev),
                                             _stream(stream)), "xconv_pixel_indep_probe_fwd")


def xconv_pixel_indep_dw_estimate(desc, dY_dev, Xbar_dev, dW_dev, ws_dev, stream=None):
    _check(lib().xconv_pixel_indep_dw_estimate(ctypes.byref(desc), _ptr(dY_dev), _ptr(Xbar_dev), _ptr(dW_dev), _ptr(ws_dev),
                                               _nbytes(ws_dev), _stream(stream)), "xconv_pixel_indep_dw_estimate")


# ---- ReLU that keeps one sign bit per element -----------------------------------------
def xconv_relu_mask_bytes(n):
    return int(lib().xconv_relu_mask_bytes(int(n)))


def xconv_relu_fwd(dtype, X_dev, Y_dev, mask_dev, n, stream=None):
    _check(lib().xconv_relu_fwd(DTYPES[dtype] if isinstance(dtype, str) else dtype, _ptr(X_dev), _ptr(Y_dev), _ptr(mask_dev), int(n),
                                _stream(stream)), "xconv_relu_fwd")


def xconv_relu_bwd(dtype, dY_dev, mask_dev, dX_dev, n, stream=None):
    _check(lib().xconv_relu_bwd(DTYPES[dtype] if isinstance(dtype, str) else dtype, _ptr(dY_dev), _ptr(mask_dev), _ptr(dX_dev), int(n),
                                _stream(stream)), "xconv_relu_bwd")

