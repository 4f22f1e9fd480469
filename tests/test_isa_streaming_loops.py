"""The weight-streaming loops of every kernel instance and of every out-of-line task body must hold no access to
scratch memory: a reload of a spilled register is a memory load that queues behind the whole ring of weight loads in
flight, and whether the compiler puts one there changes with unrelated edits (it cost the MoE instance 15 % of a step
before the staged path became a function of its own).  Checked on the ISA the build produces: no basic block contains
both a matrix instruction and a scratch access.  CPU only (hipcc cross-compiles)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_13327_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_no_scratch_access_inside_a_block_with_matrix_instructions(tmp_path):
    asm = tmp_path / "megakernel.s"
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unused-command-line-argument", os.path.join(CSRC, "megakernel.hip"), "-o", str(asm)],
                          stderr=subprocess.DEVNULL)
    funcs, name = {}, None
    for line in asm.read_text().split("\n"):
        m = re.match(r"^(_Z[A-Za-z0-9_]+):", line)
        if m:
            name = m.group(1)
            funcs[name] = [[]]
        elif name is not None:
            if re.match(r"^\.LBB[0-9_]+:", line):
                funcs[name].append([])
            funcs[name][-1].append(line)
    assert any("megakernel_static" in f for f in funcs) and any("gemm_tiles_chunked" in f for f in funcs)
    n_mfma_blocks, bad = 0, []
    for fn, blocks in funcs.items():
        for b in blocks:
            if any("v_mfma" in x for x in b):
                n_mfma_blocks += 1
                if any("scratch_" in x for x in b):
                    bad.append(fn)
    assert n_mfma_blocks > 100          # the check sees the streaming loops at all
    # Known and accepted: the 64-column, 4-tile chunked body reloads one 16-byte value in two blocks of its conditional
    # last revolutions (its ring is 4 loads deep there, not 16; the steady state is clean).
    known = [f for f in bad if "gemm_tiles_chunkedILi4ELi4E" in f]
    assert len(known) <= 2
    rest = sorted(set(bad) - set(known))
    assert not rest, f"scratch access next to matrix instructions in: {rest}"
