"""Host-only check of the decode kernel's generated code: the page ring lives on loads in flight, and the kernel
issues and awaits them from inline assembly.  A wait on vector memory that the compiler inserts by itself drains
the ring (it waits for every page in flight), so outside the kernel's prologue and its two answered arrival
counters there must be none, in any instantiation; and the wave-uniform reads of lengths and page ids must go
through the scalar path (a vector load in the loop is how such a wait gets there)."""
import os
import re
import subprocess

import pytest

from paper_2604_23838_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def decode_kernels(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "jd_fused_mfma.s"
    flags = [f for f in B.FLAGS if f != "-fPIC"]
    cmd = [B._hipcc(), *flags, "-I", os.path.join(ROOT, "include"), "--cuda-device-only", "-S",
           os.path.join(B.CSRC, "jd_fused_mfma.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    kernels, name, body = {}, None, []
    for line in open(out):
        m = re.match(r"^(_ZN\S*decode_fused_kernel\S*):", line)
        if m:
            name, body = m.group(1), []
        elif line.startswith(".Lfunc_end") and name:
            kernels[name] = body
            name = None
        elif name:
            body.append(line)
    assert len(kernels) == 5, list(kernels)
    return kernels


def compiler_lines(body):
    inside = False
    for line in body:
        if "#ASMSTART" in line:
            inside = True
        elif "#ASMEND" in line:
            inside = False
        elif not inside:
            yield line


def test_no_compiler_inserted_wait_drains_the_page_ring(decode_kernels):
    for name, body in decode_kernels.items():
        waits = [l for l in compiler_lines(body) if "s_waitcnt" in l and "vmcnt" in l]
        # three in the prologue (the scan of the lengths, before any page is requested) and one behind each of the
        # two arrival counters whose answer is awaited (after the last page)
        assert len(waits) <= 5, (name, len(waits))


def test_uniform_reads_take_the_scalar_path(decode_kernels):
    for name, body in decode_kernels.items():
        vector = [l for l in compiler_lines(body) if re.search(r"\b(global|buffer|flat)_load_dword\b", l)]
        # the prologue's per-thread reads of the lengths and of the header
        assert len(vector) <= 3, (name, len(vector))
        assert any("s_load_dword" in l for l in compiler_lines(body)), name
