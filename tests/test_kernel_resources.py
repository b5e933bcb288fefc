"""Compile-time guard for the kernels whose speed hinges on occupancy: the step kernel is tuned
for four waves per SIMD (at most 128 vector registers) and must not spill; one more register
block costs a wave per SIMD and about 6 % of the step time on an MI355X.  hipcc cross-compiles
for gfx950 without a GPU, so this runs with the CPU tests."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2208_05631_amd", "csrc")


def resource_usage(source):
    import __graft_entry__ as entry
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as tmp:
        cmd = ["hipcc", *flags, "--cuda-device-only", "-c", "-I" + os.path.join(ROOT, "include"),
               "-I" + CSRC, os.path.join(CSRC, source), "-o", os.path.join(tmp, "k.o"),
               "-Rpass-analysis=kernel-resource-usage"]
        err = subprocess.run(cmd, check=True, capture_output=True, text=True, cwd=tmp).stderr
    out = {}
    pat = (r"Function Name: (\S+).*?VGPRs: (\d+).*?ScratchSize \[bytes/lane\]: (\d+)"
           r".*?Occupancy \[waves/SIMD\]: (\d+).*?LDS Size \[bytes/block\]: (\d+)")
    for m in re.finditer(pat, err, re.S):
        out[m.group(1)] = dict(vgprs=int(m.group(2)), scratch=int(m.group(3)), waves=int(m.group(4)),
                               lds=int(m.group(5)))
    return out


@pytest.fixture(scope="module")
def step_kernels():
    return {k: v for k, v in resource_usage("qa_step.hip").items() if "step_lut_kernel" in k}


def test_no_step_kernel_variant_spills(step_kernels):
    assert len(step_kernels) >= 40                       # every template combination was seen
    spilling = {k: v for k, v in step_kernels.items() if v["scratch"] != 0}
    assert not spilling, spilling


def test_step_kernel_variants_keep_four_waves_per_simd(step_kernels):
    low = {k: v for k, v in step_kernels.items() if v["vgprs"] > 128 or v["waves"] < 4}
    assert not low, low
    # four work-groups per CU must also fit the 160 KiB of LDS
    assert all(v["lds"] <= 40 * 1024 for v in step_kernels.values())
