"""The correlation kernels issue their LDS fragment reads and staged global loads as opaque instructions and wait for
them by hand.  The compiler does not know that such a register is not valid until its wait: any register copy it places
between the request and the wait reads stale data (seen once: a copy "a = a_next" behind the wait was emitted in
front of it, and one accumulator tile of a workgroup came out wrong about once in a hundred launches).  This test
compiles the hand-scheduled sources to assembly and checks that no v_mov reads a register that a hand-issued ds_read
or buffer_load has written before the hand-placed s_waitcnt that covers it.  Host only (hipcc cross-compiles)."""
import os
import re
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2106_06998_amd", "csrc")
SOURCES = ["corr_kernels.hip", "corr_ws_kernels.hip", "corr_ws32_kernels.hip", "corr_row_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _regs(reg):
    if reg.startswith("v["):
        a, b = map(int, reg[2:-1].split(":"))
        return ["v%d" % k for k in range(a, b + 1)]
    return [reg]


def early_copies(text):
    """(function, line number, instruction) of every suspicious copy in one assembly file."""
    found = []
    for f in re.split(r"\n(?=_ZN2xc[^\n]*:\s*;\s*@)", text)[1:]:
        name = f.split(":", 1)[0]
        pend = {"lgkmcnt": {}, "vmcnt": {}}
        inasm = False
        for i, line in enumerate(f.split("\n")):
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                inasm = True
                continue
            if t.startswith(";;#ASMEND"):
                inasm = False
                continue
            m = re.match(r"ds_read_b(?:32|64|128) (v\[?\d+(?::\d+)?\]?)", t)
            if inasm and m:
                for r in _regs(m.group(1)):
                    pend["lgkmcnt"][r] = i
                continue
            m = re.match(r"buffer_load_dword(?:x\d)? (v\[?\d+(?::\d+)?\]?)", t)
            if inasm and m:
                for r in _regs(m.group(1)):
                    pend["vmcnt"][r] = i
                continue
            if "s_waitcnt" in t:
                # requests return in order: all but the n youngest are done
                for key, p in pend.items():
                    m = re.search(key + r"\((\d+)\)", t)
                    if m:
                        order = sorted(set(p.values()))
                        done = set(order[:max(0, len(order) - int(m.group(1)))])
                        for r, v in list(p.items()):
                            if v in done:
                                del p[r]
                continue
            m = re.match(r"v_mov_b32(?:_e32)? (v\d+), (v\d+)", t)
            if m and (m.group(2) in pend["lgkmcnt"] or m.group(2) in pend["vmcnt"]):
                found.append((name, i, t))
            m = re.match(r"v_\w+ (v\d+),", t)
            if m and not inasm:      # overwritten by ordinary code: no longer a pending request's register
                pend["lgkmcnt"].pop(m.group(1), None)
                pend["vmcnt"].pop(m.group(1), None)
    return found


def test_the_scan_flags_a_copy_in_front_of_its_wait():
    bad = """
_ZN2xc4demoEv:                          ; @_ZN2xc4demoEv
	;;#ASMSTART
	ds_read_b32 v138, v63
	;;#ASMEND
	v_mov_b32_e32 v27, v138
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
"""
    good = bad.replace("\tv_mov_b32_e32 v27, v138\n", "").replace("\t;;#ASMEND\n\n", "\t;;#ASMEND\n") + "\tv_mov_b32_e32 v27, v138\n"
    assert len(early_copies(bad)) == 1
    assert early_copies(good) == []


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_no_fragment_register_is_copied_before_its_wait():
    tmp = tempfile.mkdtemp(prefix="xconv_isa_")
    try:
        def compile_one(src):
            out = os.path.join(tmp, src.replace(".hip", ".s"))
            cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                   "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", out]
            p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            assert p.returncode == 0, p.stdout[-2000:]
            return src, open(out).read()

        with ThreadPoolExecutor(max_workers=4) as ex:
            texts = list(ex.map(compile_one, SOURCES))
        for src, text in texts:
            assert "v_mfma" in text, src
            assert early_copies(text) == [], src
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
