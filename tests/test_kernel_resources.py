"""Compile-time properties the launch configurations rely on (no GPU needed): the projection
kernels must not spill to scratch, and the shapes that are meant to run two workgroups per CU
must leave room for them (registers per wave, both register files counted)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_09244_amd", "csrc")


def _resource_usage(src):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-c",
           os.path.join(CSRC, src), "-o", os.devnull, "-Rpass-analysis=kernel-resource-usage"]
    out = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert out.returncode == 0, out.stderr[-2000:]
    kernels, cur = {}, None
    for line in out.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = kernels.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return kernels


def test_projection_kernels_fit_their_launch_shapes():
    k = _resource_usage("gemm.hip")
    gemm = {n: v for n, v in k.items() if "gemm_kernel" in n}
    assert len(gemm) == 28                                   # 7 tile shapes x 4 epilogues
    for name, v in gemm.items():
        assert v["ScratchSize"] == 0, (name, v)              # (a spill reload in the main loop
        four_wave_big = ("ILi256ELi256ELi64ELi2ELi2ELi2E" in name    # would also wait on the loads)
                         or "ILi288ELi192ELi64ELi2ELi2ELi2E" in name)
        assert v["Occupancy"] >= (1 if four_wave_big else 2), (name, v)
        if four_wave_big:                                    # accumulators in the second file
            assert v["AGPRs"] >= 240 and v["VGPRs"] <= 256, (name, v)
    # 128x128 on four waves with two stages is launched two workgroups per CU
    two_per_cu = [v for n, v in gemm.items() if "ILi128ELi128ELi64ELi2ELi2ELi2E" in n]
    assert len(two_per_cu) == 4
    for v in two_per_cu:
        assert v["VGPRs"] + v["AGPRs"] <= 256, v


def test_attention_kernel_keeps_two_workgroups_per_cu():
    k = _resource_usage("attention.hip")
    att = {n: v for n, v in k.items() if "attention_kernel" in n}
    assert att
    for name, v in att.items():
        assert v["ScratchSize"] == 0 and v["Occupancy"] >= 2, (name, v)
