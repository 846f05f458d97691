"""MI355X-native XConv weight-gradient path (channel-probe variant).

The compute lives in a C-ABI shared library built from csrc/ (hand-written HIP
for gfx950); `binding` is the thin ctypes front end with the same entry-point
names.  Importing the package does not load the library; the first call does,
and it raises if the library has not been built.  `layer` holds a drop-in
torch.nn.Conv2d replacement (XConv2d, convert_net) built on those entry points.
"""
__all__ = ["binding", "synth", "layer"]
