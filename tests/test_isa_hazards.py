"""Host-side check of the generated gfx950 code around the GEMM's assembly blocks.

The grouped GEMM moves its operands with global_load_lds_dwordx4 written as inline assembly, with the
base address in a scalar register pair.  A scalar register written by a vector instruction (the way
the compiler restores a spilled scalar: v_readlane) may not be used as a memory address within five
wait states, and the compiler pads its own memory instructions but does not look inside an assembly
block.  This test compiles the kernel with the library's flags and checks that no copy in the
generated code has its base written by a vector instruction within the seven instructions before it.
"""
import os
import re
import subprocess
import tempfile

from paper_2605_27081_amd import build as libbuild

SRC = os.path.join(libbuild.CSRC, "gemm_bf16.hip")
VALU_WRITES_SGPR = re.compile(r"(v_readlane_b32|v_readfirstlane_b32|v_cmp\w*_e64|v_mad_u64_u32|v_add_co\w*|v_sub_co\w*|v_subrev_co\w*|v_div_scale\w*)\s+s\[?(\d+)")


def _real_instruction(line: str) -> bool:
    t = line.strip()
    return bool(t) and not t.startswith(";") and not t.startswith(".") and not t.endswith(":")


def test_no_vector_written_scalar_base_in_front_of_a_copy():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm.s")
        flags = [f for f in libbuild.FLAGS if f != "-fPIC"]
        r = subprocess.run([libbuild.HIPCC, *flags, "-S", "--cuda-device-only", "-c", SRC, "-o", out],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        lines = open(out).read().split("\n")
    copies = 0
    for i, line in enumerate(lines):
        m = re.search(r"global_load_lds_dwordx4 v\d+, s\[(\d+):(\d+)\]", line)
        if not m:
            continue
        copies += 1
        lo, hi = int(m.group(1)), int(m.group(2))
        seen, j = 0, i - 1
        while j >= 0 and seen < 7:
            if _real_instruction(lines[j]):
                seen += 1
                w = VALU_WRITES_SGPR.match(lines[j].strip())
                assert not (w and lo <= int(w.group(2)) <= hi), (
                    f"line {i + 1}: {line.strip()} uses s[{lo}:{hi}], written {seen} instruction(s) earlier by "
                    f"'{lines[j].strip()}': pad copy16_to_lds with wait states")
            j -= 1
    assert copies >= 16, f"only {copies} direct-to-LDS copies found: has the kernel changed?"
