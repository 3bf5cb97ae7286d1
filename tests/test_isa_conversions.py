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


def _compile_to_asm(source, tmp):
    asm = os.path.join(tmp, os.path.basename(source).replace(".hip", ".s"))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only", "-Xclang",
                    "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                    os.path.join(CSRC, source), "-o", asm], check=True, capture_output=True, timeout=900)
    return open(asm).read()


def _vgprs(text):
    """Vector registers named in an operand string or instruction."""
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        out |= set(range(int(m.group(1)), int(m.group(2)) + 1)) if m.group(1) else {int(m.group(3))}
    return out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_tiled_prepacked_kernel_instruction_level():
    """The benchmarked tiled kernel (gemm_tile_pk.hip), compiled to gfx950 assembly.

    (1) The same claim as above (Sec. 4.2, Table 2) on this kernel: with integer scales no int32 -> float conversion in
    the K loop (only the epilogue's, once per output and copy of the epilogue), with float scales one per output and
    K step.  (2) Two properties of its asm statements that the compiler cannot check: a 16-byte device-scope store is
    followed by two idle cycles before anything may write its data registers (the hardware reads them late), and the
    registers a device-scope load returns into are named by no instruction before the counter wait behind it."""
    with tempfile.TemporaryDirectory() as tmp:
        text = _compile_to_asm("gemm_tile_pk.hip", tmp)
    kernels = {}
    for m in re.finditer(r"^(_ZN\S*19gemm_tile_pk_kernelILb([01])E\S*):[^\n]*\n(.*?)\n\.Lfunc_end", text, re.S | re.M):
        kernels[m.group(2)] = m.group(3)
    assert set(kernels) == {"0", "1"}
    fs, is_ = kernels["0"], kernels["1"]
    outputs_per_lane = 128                     # 8 x 4 sub-tiles x 4 results

    def loops_with_mfma(body):                 # the bodies of the K loops: a label .. the backward branch to it
        lines = body.split("\n")
        labels = {m.group(1): i for i, l in enumerate(lines) if (m := re.match(r"^(\.LBB\d+_\d+):", l))}
        found = []
        for i, l in enumerate(lines):
            m = re.search(r"s_c?branch\w* (\.LBB\d+_\d+)", l)
            if m and m.group(1) in labels and labels[m.group(1)] < i:
                seg = "\n".join(lines[labels[m.group(1)]:i])
                if len(re.findall(r"v_mfma_i32_16x16x64_i8", seg)) >= 64:
                    found.append(seg)
        return found

    is_loops, fs_loops = loops_with_mfma(is_), loops_with_mfma(fs)
    assert is_loops and fs_loops
    for seg in is_loops:                       # (two copies: 24-bit and 32-bit multiplies)
        assert len(re.findall(r"v_cvt_f32_i32", seg)) == 0
        assert len(re.findall(r"v_mad_i32_i24|v_mul_lo_u32", seg)) >= outputs_per_lane
    for seg in fs_loops:
        assert len(re.findall(r"v_cvt_f32_i32", seg)) >= outputs_per_lane
        assert len(re.findall(r"v_mad_i32_i24", seg)) == 0

    lines = [l.strip() for l in text.split("\n")]
    code = [(i, l) for i, l in enumerate(lines) if l and not l.startswith((";", ".")) and not l.endswith(":")]
    stores = loads = 0
    for at, (i, l) in enumerate(code):
        if l.startswith("global_store_dwordx4") and "sc1" in l:
            stores += 1
            assert code[at + 1][1].startswith("s_nop 1"), f"line {i}: no idle cycles behind the 16-byte store"
        if l.startswith("global_load_dwordx4") and "sc1" in l:
            loads += 1
            dst = _vgprs(l.split(None, 1)[1].split(",")[0])
            for j, u in code[at + 1:]:
                if u.startswith("s_waitcnt vmcnt(0)"):
                    break
                assert not (_vgprs(u.split(";")[0]) & dst) or u.startswith("global_load_dwordx4"), \
                    f"line {j}: `{u}` names registers of the load at line {i} before its wait"
    assert stores > 0 and loads > 0


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_producers_round_to_fp32_before_fp16():
    """RMSNorm and SiLU * up are defined with every operation rounded to single precision and the result then rounded
    to fp16 (their codes are compared bit for bit).  The compiler can merge a final multiply into the conversion
    (v_fma_mixlo_f16 / v_fma_mixhi_f16: one rounding of the exact product), which gives the other fp16 neighbour when
    the fp32 product is an fp16 tie: no such instruction may be left in the producers."""
    with tempfile.TemporaryDirectory() as tmp:
        text = _compile_to_asm("act_producers.hip", tmp)
    assert "v_cvt_pk_f16_f32" in text or "v_cvt_f16_f32" in text
    assert not re.search(r"v_fma_mix(lo|hi)_f16", text)
