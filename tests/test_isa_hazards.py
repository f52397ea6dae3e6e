"""Host-side check of the generated gfx950 code around the GEMM's assembly blocks.

The grouped GEMM moves its operands with global_load_lds_dwordx4 written as inline assembly.  The
compiler pads its own instructions with the wait states the hardware requires but does not look
inside an assembly block, so the block is written not to need any from outside:
  * the copy takes its address from a vector register pair (saddr = off).  A scalar base would be
    a scalar register read as a memory address, which must not happen within five wait states of
    a vector instruction writing that register (how the compiler restores a spilled scalar);
  * M0 (the LDS destination) is written inside the block, one wait state in front of the copy.
This test compiles the kernel with the library's flags and checks the generated code for exactly
that shape, and that nothing else in the kernel reads or writes M0.
"""
import os
import re
import subprocess
import tempfile

from paper_2605_27081_amd import build as libbuild

SRC = os.path.join(libbuild.CSRC, "gemm_bf16.hip")


def _real_instruction(line: str) -> bool:
    t = line.strip()
    return bool(t) and not t.startswith(";") and not t.startswith(".") and not t.endswith(":")


def test_direct_to_lds_copies_need_no_outside_wait_states():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm.s")
        flags = [f for f in libbuild.FLAGS if f != "-fPIC"]
        r = subprocess.run([libbuild.HIPCC, *flags, "-S", "--cuda-device-only", SRC, "-o", out],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        lines = [l.strip() for l in open(out).read().split("\n") if _real_instruction(l)]
    copies = 0
    for i, line in enumerate(lines):
        if "m0" in re.split(r"[;]", line)[0] and not line.startswith("global_load_lds"):
            assert re.match(r"s_mov_b32 m0, s\d+$", line), f"unexpected use of M0: '{line}'"
            assert lines[i + 1] == "s_nop 0" and lines[i + 2].startswith("global_load_lds_dwordx4"), (
                f"'{line}' is not followed by a wait state and a copy: {lines[i + 1:i + 3]}")
        if not line.startswith("global_load_lds"):
            continue
        copies += 1
        assert re.match(r"global_load_lds_dwordx4 v\[\d+:\d+\], off$", line), (
            f"copy with a scalar base or an unexpected form: '{line}'")
        assert lines[i - 1] == "s_nop 0" and re.match(r"s_mov_b32 m0, s\d+$", lines[i - 2]), (
            f"copy not preceded by its own M0 write and wait state: {lines[i - 2:i + 1]}")
    assert copies >= 16, f"only {copies} direct-to-LDS copies found: has the kernel changed?"
