"""The library enqueues on the stream it is given and allocates nothing, so a layer runs the same on
a side stream and inside a captured HIP graph: both against the eager result on the default stream,
which the parity tests check against the oracle (results are deterministic, hence bit-equal)."""
import numpy as np
import pytest
import torch

from paper_2106_06998_amd import binding as xb
from paper_2106_06998_amd import synth
from test_gpu_parity import DEV, say

pytestmark = pytest.mark.gpu

LAYERS = [
    ("f32", 6, 32, 48, 17, 15, 3, 1, 1, 16, "gaussian"),       # fp32 producer/consumer kernel
    ("f16", 9, 64, 64, 14, 14, 3, 1, 1, 64, "rademacher"),     # 16-bit producer/consumer kernel
    ("bf16", 3, 20, 18, 7, 9, 3, 2, 1, 20, "rademacher"),      # generic kernels, repacked dY
]


class Layer:
    def __init__(self, e):
        dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = e
        self.e = e
        self.d = xb.make_desc(B, C_in, C_out, H, W, k, st, pad, r, dtype, probe, 99)
        Ho, Wo = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
        self.X = xb.to_device(synth.draw((B, C_in, H, W), 31, "relu_normal", 1.0, dtype), dtype, DEV)
        self.dY = xb.to_device(synth.draw((B, C_out, Ho, Wo), 32, "normal", 1e-2, dtype), dtype, DEV)
        self.Xt = xb.alloc_xt(self.d, DEV)
        self.dW = torch.empty((C_out, C_in, k, k), dtype=torch.float32, device=DEV)
        self.wsp = xb.alloc_ws(self.d, xb.XCONV_OP_PROBE, DEV)
        self.wse = xb.alloc_ws(self.d, xb.XCONV_OP_ESTIMATE, DEV)

    def step(self, stream=None):
        xb.xconv_probe_fwd(self.d, self.X, self.Xt, None, self.wsp, stream)
        xb.xconv_dw_estimate(self.d, self.dY, self.Xt, None, self.dW, self.wse, stream)

    def refill(self, salt):
        dtype, B, C_in, C_out, H, W, k, st, pad, r, probe = self.e
        self.X.copy_(xb.to_device(synth.draw(tuple(self.X.shape), 41 + salt, "relu_normal", 1.0, dtype), dtype, DEV))
        self.dY.copy_(xb.to_device(synth.draw(tuple(self.dY.shape), 51 + salt, "normal", 1e-2, dtype), dtype, DEV))


@pytest.mark.parametrize("e", LAYERS, ids=[e[0] for e in LAYERS])
def test_side_stream_gives_the_default_stream_result(e):
    say("side stream %s" % (e,))
    L = Layer(e)
    L.step()
    torch.cuda.synchronize()
    want = L.dW.clone()
    L.dW.fill_(float("nan"))
    L.Xt.fill_(0x7f)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    L.step(side)                        # explicit stream argument, not the current stream
    side.synchronize()
    assert torch.equal(L.dW, want)
    L.dW.fill_(float("nan"))
    torch.cuda.synchronize()
    with torch.cuda.stream(side):       # the binding's default: torch's current stream
        L.step()
    side.synchronize()
    assert torch.equal(L.dW, want)


@pytest.mark.parametrize("e", LAYERS, ids=[e[0] for e in LAYERS])
def test_captured_graph_replays_give_the_eager_result(e):
    say("graph capture %s" % (e,))
    L = Layer(e)
    L.step()                            # eager once: kernel attributes are set outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.step()
    for salt in range(3):               # new inputs in the same buffers, eager work and synchronisation between replays
        L.refill(salt)
        L.step()
        torch.cuda.synchronize()
        want = L.dW.clone()
        L.dW.fill_(float("nan"))
        L.Xt.fill_(0x7f)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(L.dW, want), salt
        assert bool(torch.isfinite(L.dW).all())


def test_two_layers_on_two_streams_at_once():
    # the library keeps no state between calls: layers with buffers of their own, enqueued alternately on two
    # streams, give what each gives alone
    say("two streams at once")
    a, b = Layer(LAYERS[0]), Layer(LAYERS[1])
    a.step()
    b.step()
    torch.cuda.synchronize()
    want_a, want_b = a.dW.clone(), b.dW.clone()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(4):
        a.dW.fill_(float("nan"))
        b.dW.fill_(float("nan"))
        torch.cuda.synchronize()
        xb.xconv_probe_fwd(a.d, a.X, a.Xt, None, a.wsp, sa)
        xb.xconv_probe_fwd(b.d, b.X, b.Xt, None, b.wsp, sb)
        xb.xconv_dw_estimate(a.d, a.dY, a.Xt, None, a.dW, a.wse, sa)
        xb.xconv_dw_estimate(b.d, b.dY, b.Xt, None, b.dW, b.wse, sb)
        sa.synchronize()
        sb.synchronize()
        assert torch.equal(a.dW, want_a) and torch.equal(b.dW, want_b), rep

