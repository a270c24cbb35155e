"""Host-side check of the generated code (no GPU): the steady-state loops of the two MFMA-bound kernels that run one
wavefront per SIMD hold no register spills.

Both kernels sit at the edge of the register file, and a spill that lands inside the loop costs far more than its
instruction: a scratch load shares the vector-memory counter with the direct-to-LDS loads, so the loop's
`s_waitcnt vmcnt(0)` then waits for it too (a one-line change of a loop bound that moved one scratch load into the
256-column prefill kernel's loop made every launch 4-5 % slower, with every test green).  The check compiles the
source to assembly with the build's own flags and looks at the basic blocks that carry the loops' MFMAs.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2509_16495_amd import build as BLD

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc to compile to assembly")


def _blocks_of(source, kernel_substr, tmp_path):
    """Basic blocks of the kernel whose mangled name contains `kernel_substr`: [label, mfmas, spill ops, instructions]."""
    out = os.path.join(str(tmp_path), source + ".s")
    flags = [f for f in BLD.FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.check_call(["hipcc", *flags, "--cuda-device-only", "-S", os.path.join(BLD.CSRC, source), "-o", out],
                          cwd=BLD.CSRC, stderr=subprocess.DEVNULL)
    blocks, cur, inside = [], None, False
    for line in open(out):
        s = line.strip()
        m = re.match(r"^([A-Za-z_.$][\w.$]*):", line)
        if m and not m.group(1).startswith(".L"):      # a function label
            inside = kernel_substr in m.group(1)
            cur = None
            continue
        if not inside:
            continue
        if m:
            cur = [m.group(1), 0, 0, 0]
            blocks.append(cur)
        elif cur is not None and s and not s.startswith((";", ".")):
            cur[3] += 1
            cur[1] += "v_mfma" in s
            cur[2] += ("scratch_" in s) or ("v_readlane" in s) or ("v_writelane" in s)
    return blocks


def test_prefill64_steady_state_loop_has_no_spills(tmp_path):
    blocks = _blocks_of("prefill_mfma64.hip", "prefill64_kernel", tmp_path)
    heavy = [i for i, b in enumerate(blocks) if b[1] >= 24]      # bodies of an iteration: 32 MFMAs, a few of them in a block in front
    # the steady-state bodies (two of the attempt that follows no reference, two of those that follow the maximum) are the
    # short ones; the bodies next to a pass's ends carry wait states in front of every MFMA and are far longer
    steady = [i for i in heavy if blocks[i][3] < 300]
    assert len(steady) >= 4, [tuple(b) for b in blocks if b[1]]
    for i in steady:
        body = blocks[i]
        assert body[2] == 0, ("spill traffic in a steady-state body", tuple(body))
        front = blocks[i - 1]                                   # barrier, refill of the ring and the body's first MFMAs
        assert front[1] + body[1] == 32, (tuple(front), tuple(body))
        assert front[2] == 0, ("spill traffic in front of a steady-state body", tuple(front))


def test_proj_gemm_main_loop_has_no_spills(tmp_path):
    for kernel in ("proj_gemm_kernelILb0ELb0", "proj_gemm_kernelILb1ELb0"):   # bf16 and FP8, not split over k
        blocks = _blocks_of("proj_gemm.hip", kernel, tmp_path)
        loops = [b for b in blocks if b[1] >= 64]                # a stage pair of the main loop: 128 (bf16) or 64 (FP8) MFMAs
        assert loops, (kernel, [tuple(b) for b in blocks if b[1]])
        for b in loops:
            assert b[2] == 0, ("spill traffic in the main loop", kernel, tuple(b))
