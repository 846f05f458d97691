"""Seeded synthetic layer inputs shared by the tests, the bench and the oracle
checks.  This module holds none of the method's arithmetic: it only draws X and
dY with the shapes and value distributions of the benchmark layers and rounds
them to the storage type, so that the CPU oracle and the GPU library can be fed
byte-identical inputs.

The five layers stand in for the workloads the paper measures on (small-image
CNN layers, ResNet/SqueezeNet-style layers, high-resolution U-Net layers and the
half-precision finetuning regime, Sec. 5 and the appendix benchmark grid); the
datasets themselves are not used.
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    B: int
    C_in: int
    C_out: int
    H: int
    W: int
    k: int
    stride: int
    pad: int
    r: int
    probe: str          # "rademacher" | "gaussian"
    dtype: str          # "f32" | "bf16" | "f16"  (storage of X, dY and the stored probe output)
    x_dist: str         # "normal" | "relu_normal"
    dy_var: float       # variance of dY
    seeds: tuple = field(default=(0, 0, 0))   # (X, dY, Z)

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.k) // self.stride + 1


CONFIGS = {
    "C1": LayerConfig("C1", 4, 16, 16, 32, 32, 3, 1, 1, 8, "rademacher", "f32", "normal", 1.0, (1001, 2001, 3001)),
    "C2": LayerConfig("C2", 128, 64, 64, 32, 32, 3, 1, 1, 16, "gaussian", "f32", "relu_normal", 1e-2, (1002, 2002, 3002)),
    "C3": LayerConfig("C3", 64, 128, 256, 56, 56, 3, 2, 1, 32, "rademacher", "bf16", "relu_normal", 1e-2, (1003, 2003, 3003)),
    "C4": LayerConfig("C4", 8, 64, 64, 256, 256, 3, 1, 1, 16, "gaussian", "f32", "relu_normal", 1e-3, (1004, 2004, 3004)),
    "C5": LayerConfig("C5", 256, 256, 256, 28, 28, 3, 1, 1, 64, "rademacher", "f16", "relu_normal", 1e-2, (1005, 2005, 3005)),
}


def round_to_storage(a, dtype):
    """Round a float32 array to the storage type (ties to even) and return it
    as float32 holding exactly representable values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = a.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(a.shape)
    raise ValueError(dtype)


def storage_bits(a, dtype):
    """Bit pattern of already-rounded float32 values in the storage type
    (float32 array for f32, uint16 array for the 16-bit types)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "f16":
        return a.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return (a.view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def draw(shape, seed, dist, var=1.0, dtype="f32"):
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if dist == "relu_normal":
        np.maximum(a, 0.0, out=a)
    elif dist != "normal":
        raise ValueError(dist)
    if var != 1.0:
        a *= np.float32(np.sqrt(var))
    return round_to_storage(a, dtype)


def make_layer(cfg: LayerConfig):
    """Return (X, dY) as float32 arrays of storage-representable values."""
    X = draw((cfg.B, cfg.C_in, cfg.H, cfg.W), cfg.seeds[0], cfg.x_dist, 1.0, cfg.dtype)
    dY = draw((cfg.B, cfg.C_out, cfg.Ho, cfg.Wo), cfg.seeds[1], "normal", cfg.dy_var, cfg.dtype)
    return X, dY


def small_variant(cfg: LayerConfig, B=None, H=None, W=None, C_in=None, C_out=None, r=None, name=None):
    """A reduced copy of a config (same structure, smaller extents) for
    element-by-element parity runs that the oracle finishes in seconds."""
    d = dict(cfg.__dict__)
    for key, val in (("B", B), ("H", H), ("W", W), ("C_in", C_in), ("C_out", C_out), ("r", r)):
        if val is not None:
            d[key] = val
    d["name"] = name or (cfg.name + "-small")
    return LayerConfig(**d)


def make_volume(B, C_in, C_out, dims, out_dims, seeds, dtype="f32", dy_var=1e-2):
    """(X [B,C_in,D,H,W], dY [B,C_out,D',H',W']) of a volumetric layer: post-activation inputs and
    small residuals like the 2-D layers, standing in for the CT patches of the paper's volumetric
    finetuning experiment."""
    X = draw((B, C_in) + tuple(dims), seeds[0], "relu_normal", 1.0, dtype)
    dY = draw((B, C_out) + tuple(out_dims), seeds[1], "normal", dy_var, dtype)
    return X, dY
