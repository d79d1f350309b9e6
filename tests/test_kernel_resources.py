"""CPU-only check of the compiled kernels' resource usage (hipcc cross-compiles gfx950 without a GPU).

The persistent kernels are sized from the occupancy the compiler's register count allows, and a kernel that spills to
scratch memory is refused by the launcher (its grid might not be resident all at once), which silently falls back to
the flat kernels: correct, but 10-20 % slower.  So a change that pushes one of them over its register budget must be seen here."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2110_01595_amd", "csrc")
PERSISTENT = ("encode_phase_kernel", "encode_tile_phase_kernel", "recombine_phase_kernel", "project_recombine_kernel", "majority_rows_kernel")


def resource_remarks(source):
    cmd = ["hipcc", "-c", "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, os.path.join(CSRC, source), "-o", os.devnull,
           "-Rpass-analysis=kernel-resource-usage"]
    text = subprocess.run(cmd, capture_output=True, text=True, check=True).stderr
    kernels = {}
    name = None
    for line in text.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            kernels[name] = {}
        for key in ("VGPRs", r"ScratchSize \[bytes/lane\]", r"Occupancy \[waves/SIMD\]"):
            m = re.search(r"\s%s: (\d+)" % key, line)
            if m and name:
                kernels[name][key.split(" ")[0]] = int(m.group(1))
    return kernels


@pytest.mark.parametrize("source", ["encode.hip", "decode.hip", "fused.hip", "majority.hip"])
def test_persistent_kernels_keep_eight_waves_per_simd_and_do_not_spill(source):
    kernels = resource_remarks(source)
    seen = 0
    for name, use in kernels.items():
        if any(p in name for p in PERSISTENT):
            seen += 1
            assert use["ScratchSize"] == 0, (name, use)
            assert use["Occupancy"] >= 8, (name, use)
    assert seen > 0, "no persistent kernel found in %s: the name list is stale" % source
