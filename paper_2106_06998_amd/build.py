"""Build libxconv.so (hand-written HIP for gfx950) in-tree with hipcc.

python -m paper_2106_06998_amd.build        # compile every source, link
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libxconv.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["xconv_api.hip", "probe_kernels.hip", "corr_kernels.hip", "corr_ws_kernels.hip", "corr_row_kernels.hip", "corr_ws32_kernels.hip", "pixel_kernels.hip", "relu_kernels.hip", "conv_kernels.hip", "diag_kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# XCONV_SANITIZE_HOST=1: a second library whose host code (descriptor checks, plans, size arithmetic) is built under
# AddressSanitizer and UndefinedBehaviorSanitizer; the device code is the same.  tests/run_host_sanitizers.py uses it.
SANITIZE_HOST = os.environ.get("XCONV_SANITIZE_HOST", "0") == "1"
if SANITIZE_HOST:
    LIB = os.path.join(HERE, "libxconv_san.so")
    OBJDIR = os.path.join(HERE, "_build_san")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed fp32 vector ops are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(src):
    obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
    cmd = [HIPCC] + FLAGS + (SAN_FLAGS if SANITIZE_HOST else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    if out.strip():
        print(out)
    return obj


def build(verbose=True):
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if SANITIZE_HOST:
        cmd += ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
