"""The generated code of the MFMA-tiled kernels' stage loops (CPU only: hipcc cross-compiles gfx950 to assembly).

The LDS-DMA loads of those loops are issued by asm statements that the compiler's wait-count bookkeeping does not
see.  A register the compiler reloads from scratch before such a loop and first uses inside it therefore gets an
`s_waitcnt vmcnt(n)` inside the loop with n counted from the compiler's own loads only, which in fact waits for the
DMA of the coming stages, in every stage.  The kernels are written so that this does not happen; this test keeps it
so: in the bf16 kernels every steady-state stage loop (a loop with one barrier and MFMAs) holds exactly one vmcnt
wait, the hand-placed vmcnt(4), and no scratch access."""
import os
import re
import shutil
import subprocess

import pytest

from paper_2505_19645_amd import build as hip_build

CSRC = os.path.join(os.path.dirname(os.path.abspath(hip_build.__file__)), "csrc")


def stage_loops(asm_lines):
    """(mfma count, [vmcnt arguments], scratch op count) of every loop with one barrier, MFMAs and DMA loads."""
    labels = {}
    for i, line in enumerate(asm_lines):
        m = re.match(r"^(\.LBB\d+_\d+):", line)
        if m:
            labels[m.group(1)] = i
    out = []
    for i, line in enumerate(asm_lines):
        m = re.search(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", line)
        if not m or m.group(1) not in labels or labels[m.group(1)] >= i:
            continue
        seg = asm_lines[labels[m.group(1)]:i]
        if sum("s_barrier" in x for x in seg) != 1:
            continue
        mfma = sum("v_mfma" in x for x in seg)
        if mfma == 0 or not any("global_load_lds" in x for x in seg):  # (a steady-state stage issues DMA loads)
            continue
        waits = [re.search(r"vmcnt\((\d+)\)", x).group(1) for x in seg if "vmcnt(" in x]
        out.append((mfma, waits, sum("scratch_" in x for x in seg)))
    return out


def test_no_compiler_placed_wait_in_the_bf16_stage_loops(tmp_path):
    hipcc = hip_build.HIPCC
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    asm = str(tmp_path / "expert_tiled.s")
    cmd = [hipcc] + hip_build.FLAGS + ["--cuda-device-only", "-S", os.path.join(CSRC, "expert_tiled.hip"), "-o", asm]
    b = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert b.returncode == 0, b.stderr[-4000:]
    lines = open(asm).read().split("\n")
    checked = 0
    for mode in (0, 1):  # gate/up, down; bf16 weights (E4M3 codes pass through registers: the compiler waits for them)
        name = f"_Z19expert_tiled_kernelILi{mode}ELb0EE"
        starts = [i for i, l in enumerate(lines) if re.match(name + r"\w*:", l)]
        assert len(starts) == 1, name
        end = next(i for i in range(starts[0], len(lines)) if "s_endpgm" in lines[i])
        loops = stage_loops(lines[starts[0]:end])
        # the whole-tile and the cut-schedule instance, each with 1..4 token tiles per wave
        assert sorted({m for m, _, _ in loops}) == [16, 32, 48, 64], loops
        for mfma, waits, scratch in loops:
            assert waits == ["4"] and scratch == 0, (name, mfma, waits, scratch)
            checked += 1
    assert checked >= 16
