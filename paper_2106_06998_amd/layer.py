"""Drop-in convolution layer around the weight-gradient estimator (the usage the paper's code
example shows: a layer with a probing size next to the usual arguments, and a helper that swaps the
convolutions of an existing network).

What the layer changes is what is kept between the forward and the backward pass (Algorithm 1):
instead of the input X it stores the probe output, r/C_in of X for probes over the channels
(mode "channel"), B*r numbers for probes over pixels and channels (mode "multi", Eq. (6)), B*C_in*r
for independent probing (mode "independent"); the weight gradient then comes from the matching
estimate entry point of the library.  For 2-D layers the forward convolution and the input gradient
are exact and run on the library's own kernels as well (xconv_conv_fwd, xconv_dx_exact;
engine="library", the default), or on the framework's operators (engine="framework"); the bias is
added, and its gradient summed, by the framework.  Volumetric layers use the framework's forward
convolution and input gradient.

Z is drawn from a seed that changes with every forward call (Algorithm 1: seed and probing matrix
are redrawn for each layer and iteration); nothing but the seed is kept of it.
"""
import itertools

import torch
import torch.nn.functional as F

from . import binding as xb

MODES = ("channel", "multi", "independent")
_DTYPE = {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}
_calls = itertools.count(1)


def _pair(v):
    return (v, v) if isinstance(v, int) else tuple(v)


def _aligned(t):
    """The library takes 16-byte aligned tensors; a view into the middle of a storage may not be."""
    return t if t.data_ptr() % 16 == 0 else t.clone(memory_format=torch.preserve_format)


def _layout_of(x):
    """(layout code, tensor whose memory is in that layout)."""
    if x.is_contiguous():
        return xb.XCONV_NCHW, _aligned(x)
    if x.is_contiguous(memory_format=torch.channels_last):
        return xb.XCONV_NHWC, _aligned(x)
    return xb.XCONV_NCHW, x.contiguous()


def _as_layout(t, layout):
    if layout == xb.XCONV_NHWC:
        return _aligned(t.contiguous(memory_format=torch.channels_last))
    return _aligned(t.contiguous())


def _library_conv_ok(x, weight):
    return x.is_cuda and x.dtype in _DTYPE and weight.dtype == x.dtype and weight.device == x.device


def _empty_like_layout(shape, dtype, device, layout):
    return torch.empty(shape, dtype=dtype, device=device,
                       memory_format=torch.channels_last if layout == xb.XCONV_NHWC else torch.contiguous_format)


class _XConvFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, stride, padding, r, probe, mode, seed, engine):
        ctx.own = engine == "library" and _library_conv_ok(x, weight)
        if ctx.own:
            # forward convolution on the library's kernel (Alg. 1 forward step 1)
            lay, xs0 = _layout_of(x.detach())
            B, C_in, H, W = x.shape
            d0 = xb.make_desc(B, C_in, weight.shape[0], H, W, tuple(weight.shape[2:]), stride, padding, 1, _DTYPE[x.dtype],
                              "rademacher", 0, lay)
            Ho = (H + 2 * padding[0] - weight.shape[2]) // stride[0] + 1
            Wo = (W + 2 * padding[1] - weight.shape[3]) // stride[1] + 1
            y = _empty_like_layout((B, weight.shape[0], Ho, Wo), x.dtype, x.device, lay)
            with torch.cuda.device(x.device):
                xb.xconv_conv_fwd(d0, xs0, weight.detach().contiguous(), y)
            if bias is not None:
                y += bias.detach().view(1, -1, 1, 1)
        else:
            y = F.conv2d(x, weight, bias, stride, padding)
        ctx.has_state = False
        ctx.stride, ctx.padding, ctx.x_shape = stride, padding, x.shape
        ctx.has_bias = bias is not None
        if not weight.requires_grad:
            ctx.save_for_backward(weight)
            return y
        if not x.is_cuda:
            raise RuntimeError("XConv2d: the estimator runs on the GPU only (input on %s)" % x.device)
        if x.dtype not in _DTYPE:
            raise RuntimeError("XConv2d: storage type %s is not supported (float32, bfloat16, float16)" % x.dtype)
        layout, xs = _layout_of(x.detach())
        B, C_in, H, W = x.shape
        d = xb.make_desc(B, C_in, weight.shape[0], H, W, tuple(weight.shape[2:]), stride, padding, r, _DTYPE[x.dtype], probe,
                         seed, layout)
        dev = x.device
        with torch.cuda.device(dev):
            if mode == "channel":
                if xb.xconv_xt_bytes(d) == 0 or xb.xconv_workspace_bytes(d, xb.XCONV_OP_ESTIMATE) == 0:
                    raise RuntimeError("XConv2d: layer not supported by the library (%s, r=%d)" % (tuple(x.shape), r))
                state = xb.alloc_bytes(xb.xconv_xt_bytes(d), dev)
                xb.xconv_probe_fwd(d, xs, state, None, xb.alloc_bytes(xb.xconv_workspace_bytes(d, xb.XCONV_OP_PROBE), dev))
            else:
                indep = mode == "independent"
                nbytes = (xb.xconv_pixel_indep_xbar_bytes if indep else xb.xconv_pixel_xbar_bytes)(d)
                wbytes = (xb.xconv_pixel_indep_workspace_bytes if indep else xb.xconv_pixel_workspace_bytes)(d, xb.XCONV_OP_PROBE)
                if nbytes == 0 or wbytes == 0:
                    raise RuntimeError("XConv2d: layer not supported in mode %r (%s, r=%d)" % (mode, tuple(x.shape), r))
                state = torch.empty(nbytes // 4, dtype=torch.float32, device=dev)
                (xb.xconv_pixel_indep_probe_fwd if indep else xb.xconv_pixel_probe_fwd)(d, xs, state, xb.alloc_bytes(wbytes, dev))
        ctx.save_for_backward(weight, state)
        ctx.has_state, ctx.desc, ctx.mode, ctx.layout, ctx.x_dtype = True, d, mode, layout, x.dtype
        return y

    @staticmethod
    def backward(ctx, dy):
        saved = ctx.saved_tensors
        weight = saved[0]
        dx = dw = db = None
        if ctx.needs_input_grad[0]:
            if ctx.own and dy.dtype == weight.dtype:
                # exact input gradient on the library's kernel (Sec. 2: backpropagation through the layer stays exact)
                lay, dys0 = _layout_of(dy.detach())
                B, C_in, H, W = ctx.x_shape
                d0 = xb.make_desc(B, C_in, weight.shape[0], H, W, tuple(weight.shape[2:]), ctx.stride, ctx.padding, 1,
                                  _DTYPE[dy.dtype], "rademacher", 0, lay)
                dx = _empty_like_layout(tuple(ctx.x_shape), dy.dtype, dy.device, lay)
                with torch.cuda.device(dy.device):
                    xb.xconv_dx_exact(d0, dys0, weight.detach().contiguous(), dx)
            else:
                dx = torch.nn.grad.conv2d_input(ctx.x_shape, weight, dy, stride=ctx.stride, padding=ctx.padding)
        if ctx.has_state and ctx.needs_input_grad[1]:
            state, d, dev = saved[1], ctx.desc, dy.device
            dys = _as_layout(dy.to(ctx.x_dtype), ctx.layout)
            dw32 = torch.empty(weight.shape, dtype=torch.float32, device=dev)
            with torch.cuda.device(dev):
                if ctx.mode == "channel":
                    ws = xb.alloc_bytes(xb.xconv_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), dev)
                    xb.xconv_dw_estimate(d, dys, state, None, dw32, ws)
                elif ctx.mode == "multi":
                    ws = xb.alloc_bytes(xb.xconv_pixel_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), dev)
                    xb.xconv_pixel_dw_estimate(d, dys, state, dw32, ws)
                else:
                    ws = xb.alloc_bytes(xb.xconv_pixel_indep_workspace_bytes(d, xb.XCONV_OP_ESTIMATE), dev)
                    xb.xconv_pixel_indep_dw_estimate(d, dys, state, dw32, ws)
            dw = dw32.to(weight.dtype)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            db = dy.sum(dim=(0, 2, 3))
        return dx, dw, db, None, None, None, None, None, None, None


class XConv2d(torch.nn.Conv2d):
    """torch.nn.Conv2d whose weight gradient is the estimate from `r` probing vectors.

    r: number of probing vectors (the paper's probing size); probe: "rademacher" or "gaussian";
    mode: "channel" (probes over the input channels, state r/C_in of X), "multi" (probes over pixels
    and channels, Eq. (6), state B*r numbers) or "independent" (every input channel on its own).
    Supported: dilation 1, groups 1, zero padding given as numbers.  In eval mode, or when the
    weight needs no gradient, it is a plain convolution.  `last_seed` is the seed of the latest
    training forward call.  engine: "library" runs the forward convolution and the exact input
    gradient on this library's kernels too, "framework" on torch's operators.
    """

    def __init__(self, in_channels, out_channels, kernel_size, r=16, stride=1, padding=0, bias=True, probe="rademacher",
                 mode="channel", base_seed=0, engine="library", **kw):
        super().__init__(in_channels, out_channels, kernel_size, stride=stride, padding=padding, bias=bias, **kw)
        if _pair(self.dilation) != (1, 1) or self.groups != 1 or self.padding_mode != "zeros" or isinstance(self.padding, str):
            raise ValueError("XConv2d: dilation 1, groups 1 and numeric zero padding only")
        if mode not in MODES:
            raise ValueError("XConv2d: mode must be one of %s" % (MODES,))
        if probe not in ("rademacher", "gaussian"):
            raise ValueError("XConv2d: probe must be 'rademacher' or 'gaussian'")
        if engine not in ("library", "framework"):
            raise ValueError("XConv2d: engine must be 'library' or 'framework'")
        self.r, self.probe, self.mode, self.base_seed, self.last_seed = int(r), probe, mode, int(base_seed), None
        self.engine = engine

    def forward(self, x):
        if not (self.training and torch.is_grad_enabled() and self.weight.requires_grad):
            return super().forward(x)
        self.last_seed = (self.base_seed * 0x9E3779B1 + next(_calls)) & 0x7FFFFFFFFFFFFFFF
        return _XConvFunction.apply(x, self.weight, self.bias, _pair(self.stride), _pair(self.padding), self.r, self.probe,
                                    self.mode, self.last_seed, self.engine)

    def extra_repr(self):
        return super().extra_repr() + ", r=%d, probe=%s, mode=%s" % (self.r, self.probe, self.mode)


class _SignReLUFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x):
        if not x.is_cuda:
            raise RuntimeError("SignReLU: runs on the GPU only (input on %s)" % x.device)
        if x.dtype not in _DTYPE:
            raise RuntimeError("SignReLU: storage type %s is not supported (float32, bfloat16, float16)" % x.dtype)
        # values in memory order: the mask is per element, whatever the layout
        xs = x.detach()
        if not (xs.is_contiguous() or xs.is_contiguous(memory_format=torch.channels_last)
                or (xs.dim() == 5 and xs.is_contiguous(memory_format=torch.channels_last_3d))):
            xs = xs.contiguous()
        xs = _aligned(xs)
        y = torch.empty_like(xs)          # same strides as xs
        n = xs.numel()
        mask = torch.empty(max(xb.xconv_relu_mask_bytes(n) // 8, 1), dtype=torch.int64, device=x.device)
        with torch.cuda.device(x.device):
            xb.xconv_relu_fwd(_DTYPE[x.dtype], xs, y, mask, n)
        ctx.save_for_backward(mask)
        ctx.meta = (tuple(y.shape), tuple(y.stride()), y.dtype)     # not y itself: nothing but the mask is kept
        return y

    @staticmethod
    def backward(ctx, dy):
        (mask,) = ctx.saved_tensors
        shape, strides, dtype = ctx.meta
        # the gradient in the memory order of the output
        g = torch.empty_strided(shape, strides, dtype=dtype, device=dy.device)
        g.copy_(dy)
        with torch.cuda.device(g.device):
            xb.xconv_relu_bwd(_DTYPE[g.dtype], g, mask, g, g.numel())
        return g


class SignReLU(torch.nn.Module):
    """ReLU that keeps one bit per element for its backward pass instead of its output (which the
    next convolution no longer stores once it is an XConv layer)."""

    def forward(self, x):
        if not (torch.is_grad_enabled() and x.requires_grad):
            return F.relu(x)
        return _SignReLUFunction.apply(x)


def _triple(v):
    return (v, v, v) if isinstance(v, int) else tuple(v)


class _XConv3dFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, stride, padding, r, probe, seed):
        y = F.conv3d(x, weight, bias, stride, padding)
        ctx.has_state = False
        ctx.stride, ctx.padding, ctx.x_shape = stride, padding, x.shape
        ctx.has_bias = bias is not None
        if not weight.requires_grad:
            ctx.save_for_backward(weight)
            return y
        if not x.is_cuda:
            raise RuntimeError("XConv3d: the estimator runs on the GPU only (input on %s)" % x.device)
        if x.dtype not in _DTYPE:
            raise RuntimeError("XConv3d: storage type %s is not supported (float32, bfloat16, float16)" % x.dtype)
        xs, layout = x.detach(), xb.XCONV_NCHW
        if not xs.is_contiguous():
            if xs.is_contiguous(memory_format=torch.channels_last_3d):
                layout = xb.XCONV_NHWC
            else:
                xs = xs.contiguous()
        xs = _aligned(xs)
        B, C_in, D, H, W = x.shape
        v = xb.make_desc3d(B, C_in, weight.shape[0], D, H, W, tuple(weight.shape[2:]), stride, padding, r, _DTYPE[x.dtype], probe,
                           seed, 0, layout)
        dev = x.device
        if xb.xconv3d_xt_bytes(v) == 0 or xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_ESTIMATE) == 0:
            raise RuntimeError("XConv3d: layer not supported by the library (%s, kernel %s, padding %s, r=%d)" % (
                tuple(x.shape), tuple(weight.shape[2:]), padding, r))
        with torch.cuda.device(dev):
            state = xb.alloc_bytes(xb.xconv3d_xt_bytes(v), dev)
            xb.xconv3d_probe_fwd(v, xs, state, None, xb.alloc_bytes(xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_PROBE), dev))
        ctx.save_for_backward(weight, state)
        ctx.has_state, ctx.desc, ctx.layout, ctx.x_dtype = True, v, layout, x.dtype
        return y

    @staticmethod
    def backward(ctx, dy):
        saved = ctx.saved_tensors
        weight = saved[0]
        dx = dw = db = None
        if ctx.needs_input_grad[0]:
            dx = torch.nn.grad.conv3d_input(ctx.x_shape, weight, dy, stride=ctx.stride, padding=ctx.padding)
        if ctx.has_state and ctx.needs_input_grad[1]:
            state, v, dev = saved[1], ctx.desc, dy.device
            dys = dy.to(ctx.x_dtype)
            dys = _aligned(dys.contiguous(memory_format=torch.channels_last_3d) if ctx.layout == xb.XCONV_NHWC else dys.contiguous())
            dw32 = torch.empty(weight.shape, dtype=torch.float32, device=dev)
            with torch.cuda.device(dev):
                xb.xconv3d_dw_estimate(v, dys, state, None, dw32, xb.alloc_bytes(xb.xconv3d_workspace_bytes(v, xb.XCONV_OP_ESTIMATE), dev))
            dw = dw32.to(weight.dtype)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            db = dy.sum(dim=(0, 2, 3, 4))
        return dx, dw, db, None, None, None, None, None


class XConv3d(torch.nn.Conv3d):
    """torch.nn.Conv3d whose weight gradient is the estimate from `r` probing vectors over the input
    channels (the stored state is r/C_in of X).  Supported: dilation 1, groups 1, numeric zero padding,
    kernel depth up to 7 and depth padding below the kernel depth; NCDHW or channels-last volumes."""

    def __init__(self, in_channels, out_channels, kernel_size, r=16, stride=1, padding=0, bias=True, probe="rademacher",
                 base_seed=0, **kw):
        super().__init__(in_channels, out_channels, kernel_size, stride=stride, padding=padding, bias=bias, **kw)
        if _triple(self.dilation) != (1, 1, 1) or self.groups != 1 or self.padding_mode != "zeros" or isinstance(self.padding, str):
            raise ValueError("XConv3d: dilation 1, groups 1 and numeric zero padding only")
        if probe not in ("rademacher", "gaussian"):
            raise ValueError("XConv3d: probe must be 'rademacher' or 'gaussian'")
        self.r, self.probe, self.base_seed, self.last_seed = int(r), probe, int(base_seed), None

    def forward(self, x):
        if not (self.training and torch.is_grad_enabled() and self.weight.requires_grad):
            return super().forward(x)
        self.last_seed = (self.base_seed * 0x9E3779B1 + next(_calls)) & 0x7FFFFFFFFFFFFFFF
        return _XConv3dFunction.apply(x, self.weight, self.bias, _triple(self.stride), _triple(self.padding), self.r, self.probe,
                                      self.last_seed)

    def extra_repr(self):
        return super().extra_repr() + ", r=%d, probe=%s" % (self.r, self.probe)


def convert_net(model, r=16, probe="rademacher", mode="channel", min_in_channels=None, relu=False, engine="library"):
    """Replaces, in place, every torch.nn.Conv2d (and, in mode "channel", torch.nn.Conv3d) of `model` that the layer supports (dilation 1,
    groups 1, zero padding, and at least `min_in_channels` input channels; default: more than r in
    mode "channel", where fewer channels than probing vectors save nothing) by an XConv2d that
    shares its parameters.  relu=True also replaces every torch.nn.ReLU by a SignReLU, which keeps one bit per
    element instead of its output.  Returns the model and the number of convolutions replaced."""
    if min_in_channels is None:
        min_in_channels = r + 1 if mode == "channel" else 1
    n = 0
    for parent in list(model.modules()):
        for name, child in list(parent.named_children()):
            if relu and type(child) is torch.nn.ReLU:
                setattr(parent, name, SignReLU())
                continue
            if type(child) is torch.nn.Conv3d and mode == "channel":
                kD, pd = child.kernel_size[0], child.padding[0] if not isinstance(child.padding, str) else -1
                if (_triple(child.dilation) != (1, 1, 1) or child.groups != 1 or child.padding_mode != "zeros" or pd < 0 or pd > kD - 1
                        or kD > 7 or child.in_channels < min_in_channels):
                    continue
                new = XConv3d(child.in_channels, child.out_channels, child.kernel_size, r=r, stride=child.stride,
                              padding=child.padding, bias=child.bias is not None, probe=probe, base_seed=n + 1,
                              device=child.weight.device, dtype=child.weight.dtype)
                new.weight, new.bias = child.weight, child.bias
                new.train(child.training)
                setattr(parent, name, new)
                n += 1
                continue
            if type(child) is not torch.nn.Conv2d:
                continue
            if (_pair(child.dilation) != (1, 1) or child.groups != 1 or child.padding_mode != "zeros" or isinstance(child.padding, str)
                    or child.in_channels < min_in_channels):
                continue
            new = XConv2d(child.in_channels, child.out_channels, child.kernel_size, r=r, stride=child.stride, padding=child.padding,
                          bias=child.bias is not None, probe=probe, mode=mode, base_seed=n + 1, engine=engine,
                          device=child.weight.device, dtype=child.weight.dtype)
            new.weight, new.bias = child.weight, child.bias
            new.train(child.training)
            setattr(parent, name, new)
            n += 1
    return model, n
