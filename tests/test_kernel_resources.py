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


def _device_assembly(src, tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    out_s = os.path.join(str(tmp_path), src + ".s")
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S",
           "--cuda-device-only", os.path.join(CSRC, src), "-o", out_s]
    out = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert out.returncode == 0, out.stderr[-2000:]
    return open(out_s).read().split("\n")


def _waits_among_mfmas(lines, kernel_prefix):
    """Per kernel: the compiler's own `s_waitcnt vmcnt` (not those written in inline asm) that
    stand between the first and the last MFMA instruction."""
    starts = [i for i, l in enumerate(lines) if re.match(r"^%s.*:\s*(;.*)?$" % kernel_prefix, l)]
    found = {}
    for a, b in zip(starts, starts[1:] + [len(lines)]):
        seg = lines[a:b]
        end = next((i for i, l in enumerate(seg) if "s_endpgm" in l), len(seg))
        seg = seg[:end]
        mf = [i for i, l in enumerate(seg) if "v_mfma" in l]
        if not mf:
            continue
        in_asm, waits = False, []
        for i, l in enumerate(seg):
            if "ASMSTART" in l:
                in_asm = True
            elif "ASMEND" in l:
                in_asm = False
            elif not in_asm and "s_waitcnt" in l and "vmcnt" in l and mf[0] <= i <= mf[-1]:
                waits.append(l.strip())
        found[lines[a].rstrip(":")] = waits
    return found


def _waits_in_innermost_mfma_loops(lines, kernel_prefix):
    """Per kernel: the compiler's own vmcnt waits inside the innermost loops that hold MFMA
    instructions (label ... backward branch, no loop inside), wherever in the loop they stand."""
    starts = [i for i, l in enumerate(lines) if re.match(r"^%s.*:" % kernel_prefix, l)]
    found, n_loops = {}, 0
    for a0, b0 in zip(starts, starts[1:] + [len(lines)]):
        k = lines[a0:b0]
        k = k[:next((i for i, l in enumerate(k) if "s_endpgm" in l), len(k))]
        labels = {m.group(1): i for i, l in enumerate(k)
                  for m in [re.match(r"^(\.LBB\d+_\d+):", l)] if m}
        loops = []
        for i, l in enumerate(k):
            m = re.search(r"s_c?branch\w* (\.LBB\d+_\d+)", l)
            if m and m.group(1) in labels and labels[m.group(1)] < i:
                loops.append((labels[m.group(1)], i))
        for a, b in loops:
            if any(a2 >= a and b2 <= b and (a2, b2) != (a, b) for a2, b2 in loops):
                continue
            body = k[a:b]
            if sum("v_mfma" in x for x in body) < 8:
                continue
            n_loops += 1
            in_asm, waits = False, []
            for x in body:
                if "ASMSTART" in x:
                    in_asm = True
                elif "ASMEND" in x:
                    in_asm = False
                elif not in_asm and "s_waitcnt" in x and "vmcnt" in x:
                    waits.append(x.strip())
            if waits:
                found[lines[a0].split(":")[0]] = waits
    return found, n_loops


def test_no_compiler_vmcnt_wait_inside_the_projection_main_loops(tmp_path):
    """A wait at the head of the main loop (for loads or stores of a previous tile's epilogue
    that the compiler still counts) stands before the loop's first MFMA in program order, yet
    runs every iteration and waits for the direct loads just issued.  The kernel clears the
    compiler's count once per tile; no main loop of any configuration may hold such a wait."""
    found, n_loops = _waits_in_innermost_mfma_loops(_device_assembly("gemm.hip", tmp_path),
                                                    "_ZN4mvla11gemm_kernelI")
    assert n_loops == 28
    assert not found, found


@pytest.mark.parametrize("src,prefix,n_kernels", [("gemm.hip", "_ZN4mvla11gemm_kernelI", 28),
                                                  ("attention.hip", "_ZN4mvla16attention_kernelI", 2)])
def test_no_compiler_wait_catches_the_direct_loads(src, prefix, n_kernels, tmp_path):
    """The global->LDS loads are issued from inline asm and waited for explicitly.  A wait the
    compiler adds for one of ITS loads (a spill reload, an operand fetched before the loop) counts
    every outstanding load, so inside the MFMA loops it would also wait for the direct loads of
    the next tile: there must be none between the first and the last MFMA of a kernel."""
    found = _waits_among_mfmas(_device_assembly(src, tmp_path), prefix)
    assert len(found) == n_kernels, sorted(found)
    for name, waits in found.items():
        assert not waits, (name, waits)
