"""Instruction-level pin of the paper's claim (Sec. 4.2, Table 2): with integer scales the int32 -> float conversion
leaves the K loop (one per output, in the epilogue), while the float-scale form converts every group's partial sum.
The tiled kernel is compiled to gfx950 assembly (no GPU needed) and the conversions are counted per kernel."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2405_14597_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_conversions_leave_the_k_loop_with_integer_scales():
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "gemm_prefill.s")
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only", "-Xclang",
                        "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                        os.path.join(CSRC, "gemm_prefill.hip"), "-o", asm], check=True, capture_output=True, timeout=600)
        text = open(asm).read()
    kernels = {}
    for m in re.finditer(r"^(_ZN\S*gemm_prefill_kernelILb([01])E\S*):[^\n]*\n(.*?)\n\.Lfunc_end", text, re.S | re.M):
        kernels[m.group(2)] = m.group(3)
    assert set(kernels) == {"0", "1"}, "expected the float-scale (0) and integer-scale (1) instantiations"

    def count(body, pattern):
        return len(re.findall(pattern, body))

    fs, is_ = kernels["0"], kernels["1"]
    outputs_per_lane = 64                      # 4 x 4 sub-tiles x 4 results
    # integer scale: the only conversions are the epilogue's, one per output and variant of the scale step
    assert count(is_, r"v_cvt_f32_i32") <= 2 * outputs_per_lane
    # float scale: one per output and K step in the (twice unrolled) loop, plus none needed in the epilogue
    assert count(fs, r"v_cvt_f32_i32") >= 2 * outputs_per_lane
    # the integer scale step is the 24-bit multiply-add, one per output and K step
    assert count(is_, r"v_mad_i32_i24") >= 2 * outputs_per_lane
    assert count(fs, r"v_mad_i32_i24") == 0
    # both run the same matrix instruction
    assert count(fs, r"v_mfma_i32_16x16x64_i8") > 0 and count(is_, r"v_mfma_i32_16x16x64_i8") > 0
