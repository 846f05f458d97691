"""Run the CPU-only tests of the oracle and of the library's host code under AddressSanitizer and
UndefinedBehaviorSanitizer.

    python tests/run_host_sanitizers.py

Builds oracle/libxconv_oracle_san.so (gcc) and paper_2106_06998_amd/libxconv_san.so (hipcc, host code only
instrumented), then runs the oracle pins and the host ABI tests in a child process that preloads the sanitizer
runtimes.  No GPU is touched: those tests make no compute calls.  Leak checking is off (the interpreter itself
never frees everything).  Not collected by pytest; exits with the child's status."""
import os
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def runtime(compiler, name):
    return subprocess.run([compiler, "-print-file-name=" + name], stdout=subprocess.PIPE, text=True, check=True).stdout.strip()


def main():
    env = dict(os.environ, XCONV_ORACLE_SANITIZE="1", XCONV_SANITIZE_HOST="1")
    subprocess.run([sys.executable, "-m", "oracle.build"], cwd=ROOT, env=env, check=True)
    subprocess.run([sys.executable, "-m", "paper_2106_06998_amd.build"], cwd=ROOT, env=env, check=True)
    # one AddressSanitizer runtime per process: the library's host code is built by clang, the oracle by gcc; gcc's
    # runtime is preloaded and serves both (the interface the instrumented code calls is the same)
    pre = [runtime("gcc", "libasan.so"), runtime("gcc", "libubsan.so")]
    env.update(LD_PRELOAD=":".join(pre), ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               XCONV_LIB=os.path.join(ROOT, "paper_2106_06998_amd", "libxconv_san.so"))
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "tests/test_oracle_pins.py", "tests/test_host_abi.py"]
    rc = subprocess.run(cmd, cwd=ROOT, env=env).returncode
    if "--keep" not in sys.argv:   # the instrumented builds are only for this run
        for p in ("oracle/libxconv_oracle_san.so", "paper_2106_06998_amd/libxconv_san.so"):
            if os.path.exists(os.path.join(ROOT, p)):
                os.remove(os.path.join(ROOT, p))
        shutil.rmtree(os.path.join(ROOT, "paper_2106_06998_amd", "_build_san"), ignore_errors=True)
    return rc


if __name__ == "__main__":
    sys.exit(main())
