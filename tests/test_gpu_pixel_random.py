"""Seeded random shapes through the estimators with probing vectors over pixels (xconv_pixel_* and
xconv_pixel_indep_*), both layouts, against the CPU oracle to the tolerances of the written-out
cases: odd planes (the forward product's fallback), ragged vector and channel groups, strides,
paddings, block-sparse vectors."""
import numpy as np
import pytest

from test_gpu_pixel_indep import run_indep
from test_gpu_pixel_probe import run_pixel

pytestmark = pytest.mark.gpu


def random_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        dtype = ["f32", "bf16", "f16"][rng.integers(3)]
        k = int([1, 2, 3, 3, 5][rng.integers(5)])
        st = int([1, 1, 2, 3][rng.integers(4)])
        pad = int(rng.integers(0, k // 2 + 2))
        H, W = int(rng.integers(k, 20)), int(rng.integers(k, 20))
        if rng.random() < 0.4:
            W = (W + 3) // 4 * 4
        if (H + 2 * pad - k) // st + 1 < 1 or (W + 2 * pad - k) // st + 1 < 1:
            continue
        B = int(rng.integers(1, 40))
        C_in, C_out = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        r = int([1, 2, 3, 4, 8, 16, 20, 33, 64][rng.integers(9)])
        probe = ["rademacher", "gaussian"][rng.integers(2)]
        indep = bool(rng.random() < 0.5)
        nhwc = bool(rng.random() < 0.35)
        keep = 0 if indep else int([0, 0, 12000, 24000][rng.integers(4)])
        if B * C_out * H * W * C_in * r > 4e7:        # keep the oracle quick
            continue
        out.append((len(out), indep, nhwc, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe, keep))
    return out


CASES = random_cases(40, 20240911)


@pytest.mark.parametrize("c", CASES, ids=["rnd%02d-%s-%s%s" % (c[0], "indep" if c[1] else "multi", c[3], "-cl" if c[2] else "") for c in CASES])
def test_random_pixel_probe_shapes(c):
    i, indep, nhwc, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe, keep = c
    name = "random-%02d" % i
    if indep:
        run_indep((name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe), nhwc=nhwc)
    else:
        e = (name, dtype, B, C_in, C_out, H, W, k, st, pad, r, probe) + ((keep,) if keep else ())
        run_pixel(e, nhwc=nhwc)
