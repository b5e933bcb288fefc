"""The C ABI used from a plain C++ host program (no Python, no torch in that process):
tests/native/abi_direct.cpp, built by __graft_entry__.build(), links libqadagrad.so and the CPU
checker and compares them bit for bit; this test runs it and reads its result."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "native", "abi_direct")


def test_c_program_matches_checker():
    if not os.path.exists(EXE):
        pytest.skip("tests/native/abi_direct not built: run __graft_entry__.build()")
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.pathsep.join(
        [os.path.join(ROOT, "paper_2208_05631_amd"), os.path.join(ROOT, "oracle"),
         env.get("LD_LIBRARY_PATH", "")])
    r = subprocess.run([EXE], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    out = r.stdout
    assert sum(line.startswith("step ") and "identical" in line for line in out.splitlines()) == 4
    assert "qa_aggregate_unpack: identical" in out
    assert "qa_quantize_pack_static: identical" in out
    assert "steps with one scale for Q(SynQ): identical" in out
    assert "qa_local_grad: within 1e-6" in out
