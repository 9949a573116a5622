"""The 64-row attention kernel as the compiler emits it (no GPU needed: hipcc cross-compiles).

The kernel writes its second product's matrix instructions as asm so that the accumulators live in accumulation
registers; the compiler then knows nothing of those instructions' latency.  The source waits the results out wherever
something else may read them (a rescale, the way out, a run-time branch behind which the compiler moves registers);
this test checks in the ISA that it did so everywhere, that nothing spills, and that the loop has the mix of LDS and
matrix instructions it was built for."""
import os
import re
import subprocess

import pytest

from isa_lint import parse, violations
from paper_2501_08071_amd import build as B

SRC = "attn_fwd_rows64_gfx950.hip"


@pytest.fixture(scope="module")
def isa(tmp_path_factory):
    if not os.path.exists(B.HIPCC):
        pytest.skip("no hipcc")
    out = str(tmp_path_factory.mktemp("isa") / "rows64.s")
    cmd = [B.HIPCC, *[f for f in B.FLAGS if f != "-fPIC"], *B.SOURCE_FLAGS[SRC], "--cuda-device-only", "-S", "-x", "hip",
           os.path.join(B.CSRC, SRC), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return open(out).read()


def test_accumulators_are_waited_out_before_anything_else_touches_them(isa):
    kernels = parse(isa, "attn_fwd_rows64_kernel")
    assert len(kernels) == 4                     # two element types, with and without the causal mask
    for name, (ins, labels) in kernels.items():
        asm_acc = [a for op, a in ins if op.startswith("v_mfma") and a.split(",")[0].strip().startswith("a[")]
        assert len(asm_acc) >= 100, name         # the second product does accumulate in accumulation registers
        bad = violations(ins, labels)
        assert not bad, (name, bad[:4])


def test_no_spills_and_the_operand_sharing_shows(isa):
    kernels = parse(isa, "attn_fwd_rows64_kernel")
    for name, (ins, _) in kernels.items():
        ops = [op for op, _ in ins]
        assert not any(op.startswith("scratch_") for op in ops), name       # nothing spills to memory
        # every K/V operand read feeds two matrix instructions: over the whole kernel text (the loop with 0.75 LDS reads
        # per matrix instruction, plus prologue, the single-sub-tile steps of the causal instances at 1.5, and the
        # way out) the ratio stays below 1.2; the 32-row kernel's loop has 1.5
        lds = sum(op.startswith("ds_read") for op in ops)
        mfma = sum(op.startswith("v_mfma") for op in ops)
        assert lds < 1.2 * mfma, (name, lds, mfma)
    for m in re.finditer(r"\.vgpr_spill_count:\s+(\d+)", isa):
        assert int(m.group(1)) == 0
