"""The 384 x 256 Gram kernel pins its accumulator tiles through inline-assembly MFMAs, which the compiler's hazard
handling cannot see: the loop is only correct while the compiler neither spills nor copies an accumulator inside it.
This test compiles the kernel the way the build does and checks exactly that in the generated ISA (CPU only)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _isa(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2603_28845_amd import build
    out = tmp_path / "gram.s"
    cmd = [hipcc, *build.HIPCC_FLAGS, *build.EXTRA_FLAGS.get("gram.hip", []), "-S", "--cuda-device-only",
           os.path.join(build.CSRC, "gram.hip"), "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text()


def test_wide_gram_loop_is_straight_line(tmp_path):
    text = _isa(tmp_path)
    found = 0
    for m in re.finditer(r"^(_ZN\S*gram_bf16_ring_kernelINS\d+_8RingWideELb[01]E\S*):[^\n]*\n(.*?)^\.Lfunc_end", text, re.S | re.M):
        body = m.group(2).split("\n")
        mf = [i for i, l in enumerate(body) if "v_mfma_f32_32x32x16_bf16" in l]
        assert len(mf) == 48, (m.group(1), len(mf))           # two half-iterations of 24 tiles, nowhere else
        loop = body[mf[0]:mf[-1] + 1]
        assert not any("scratch_" in l for l in loop), "an accumulator or operand is spilled inside the loop"
        assert not any("v_accvgpr" in l for l in loop), "an accumulator is copied between the register halves inside the loop"
        acc = set()
        for i in mf:                                          # 16 tiles in AGPRs, 8 in VGPRs, each its own registers
            acc.add(re.search(r"v_mfma_f32_32x32x16_bf16 ([av]\[\d+:\d+\])", body[i]).group(1))
        assert len(acc) == 24 and sum(a.startswith("a[") for a in acc) == 16
        # the last MFMA of the loop body carries its own wait states, inside the same assembly statement, so that
        # whatever the compiler places at the loop's exit reads retired accumulators
        assert [l.strip() for l in body[mf[-1] + 1:mf[-1] + 4]] == ["s_nop 15", "s_nop 15", ";;#ASMEND"], \
            "no wait states after the last MFMA of the loop"
        found += 1
    assert found == 3        # the symmetric kernel, its paced form and the cross kernel
