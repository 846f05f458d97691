"""Compile the CPU oracle (plain C, gcc -O2) into oracle/libxconv_oracle.so.

Test infrastructure only: building the checker is not using it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "xconv_oracle.c")
# XCONV_ORACLE_SANITIZE=1: a second build under AddressSanitizer and UndefinedBehaviorSanitizer (the process that
# loads it has to preload the sanitizer runtime; tests/run_host_sanitizers.py does)
SANITIZE = os.environ.get("XCONV_ORACLE_SANITIZE", "0") == "1"
LIB = os.path.join(HERE, "libxconv_oracle_san.so" if SANITIZE else "libxconv_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if SANITIZE else ["-O2"]
    cmd = ["gcc"] + opt + ["-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-ffp-contract=off", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
