"""The 256-row prefill kernel keeps its output accumulators, Q fragments and matrix operands in
FIXED accumulation registers that only its inline assembly touches; the compiler is told of
them statement by statement (clobbers) but not that they stay live in between.  That is safe
exactly as long as the compiler puts nothing of its own into accumulation registers, which it
only does to spill: this test compiles the kernel and checks that it did not (no instruction on
an accumulation register outside an inline-assembly block, no scratch memory), and that the
generated register header is the one its generator writes."""
import os
import re
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_14201_amd", "csrc")


def test_register_header_is_what_its_generator_writes():
    out = subprocess.run([sys.executable, os.path.join(CSRC, "gen_wide_regs.py")], check=True,
                         capture_output=True, text=True).stdout
    with open(os.path.join(CSRC, "flashd_wide_regs.h")) as f:
        assert f.read() == out


@pytest.mark.timeout(300)
def test_compiler_keeps_out_of_the_accumulation_registers():
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "wide.s")
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature",
               "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", asm,
               os.path.join(CSRC, "flashd_wide.hip")]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(asm).read()
    kernels = re.findall(r"^(_ZN6flashd11wide_kernel\w+):", text, flags=re.M)
    assert len(kernels) == 2, kernels            # f16 and bf16
    in_asm, outside = False, []
    for line in text.splitlines():
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
        elif t.startswith(";;#ASMEND"):
            in_asm = False
        elif not in_asm and not t.startswith(";") and re.match(r"(v_accvgpr|scratch_)", t):
            outside.append(t)
    assert not outside, outside[:5]
    assert re.findall(r"; ScratchSize: (\d+)", text) == ["0", "0"]
    # room left in the ordinary registers, so that a small change does not start spilling
    assert all(int(n) <= 256 for n in re.findall(r"; NumVgprs: (\d+)", text))
