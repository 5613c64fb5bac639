"""The C ABI without Python in between: tests/c_abi_demo.cpp, built by build.build_demo() against include/sqa.h and
libsqa.so, runs Algorithm 1 end to end with memory from the HIP runtime and checks itself."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "paper_2404_04793_amd", "_build", "c_abi_demo")


@pytest.mark.gpu
def test_c_abi_demo_runs_the_whole_path():
    if not os.path.exists(EXE):
        pytest.skip("not built: python -m paper_2404_04793_amd.build --demo (__graft_entry__.build() does it)")
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert r.stdout.strip().endswith("c_abi_demo ok"), r.stdout[-2000:]
