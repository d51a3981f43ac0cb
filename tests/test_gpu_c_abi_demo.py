"""GPU: the plain-C demo program (examples/c_abi_demo.c, built by build()) runs against
libspt.so with nothing but the HIP runtime and prints the results it checked itself."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_runs_against_the_c_abi():
    exe = os.path.join(ROOT, "examples", "c_abi_demo")
    srcs = [os.path.join(ROOT, "include", "spt.h"), os.path.join(ROOT, "examples", "c_abi_demo.c")]
    stale = os.path.exists(exe) and any(os.path.getmtime(f) > os.path.getmtime(exe) for f in srcs)
    if not os.path.exists(exe) or stale:              # normally built by __graft_entry__.build()
        from paper_1804_10112_amd import build as spt_build
        spt_build.build_example()
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr + out.stdout
    assert "y = 7 13 0 69" in out.stdout and out.stdout.strip().endswith("ok")
