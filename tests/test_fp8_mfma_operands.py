"""Generated code of the 8-bit attention kernel: no fp8 MFMA writes its result over one of its own operands.

The 32x32x64 fp8 MFMA reads its A and B operands over several passes while it writes the result; a result tuple
that overlaps an operand tuple gives wrong numbers (seen on the GPU with a constant accumulator input, where the
compiler had placed the result on the dying operands).  The kernel always feeds a live accumulator tuple, which the
compiler ties to the result; this test compiles the kernel to assembly and checks every such instruction.
"""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2509_22622_amd", "csrc", "attn_fp8.hip")
PAT = re.compile(r"v_mfma_scale_f32_32x32x64_f8f6f4\s+v\[(\d+):(\d+)\],\s*v\[(\d+):(\d+)\],\s*v\[(\d+):(\d+)\],\s*(\S+?),")


def test_no_result_over_operand():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attn_fp8.s")
        subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-S", "--cuda-device-only", SRC, "-o", out],
                       check=True, capture_output=True)
        text = open(out).read()
    found = PAT.findall(text)
    assert len(found) >= 16, "fp8 MFMAs not found in the generated code"
    for d0, d1, a0, a1, b0, b1, c in found:
        d, a, b = (int(d0), int(d1)), (int(a0), int(a1)), (int(b0), int(b1))
        assert d[1] < a[0] or a[1] < d[0], f"result v[{d0}:{d1}] overlaps operand A v[{a0}:{a1}]"
        assert d[1] < b[0] or b[1] < d[0], f"result v[{d0}:{d1}] overlaps operand B v[{b0}:{b1}]"
        assert c.startswith("v[") or c == "0", f"accumulator input is neither a register tuple nor zero: {c}"
    # the pipelined kernels issue LDS reads whose destination registers stay pending until a counted wait: a spill
    # of such a register in between would store stale data, so these kernels must not spill at all
    spills = dict(re.findall(r"\.name:\s+(\S+)[\s\S]*?\.vgpr_spill_count:\s+(\d+)", text))
    piped = {k: int(v) for k, v in spills.items() if "ll_attn_fp8_kernel" in k and ("ELi1E" in k or "ELi2E" in k)}
    assert len(piped) == 4 and all(v == 0 for v in piped.values()), f"spills in the pipelined kernels: {piped}"


@pytest.mark.parametrize("source, kernel", [("attn_stream.hip", "ll_attn_stream_kernel"),
                                            ("attn_stream16.hip", "ll_attn_stream16_kernel")])
def test_bf16_stream_kernels_do_not_spill(source, kernel):
    """The bf16 software-pipelined kernels (both MFMA shapes) use the same pending LDS reads: they must not spill."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(ROOT, "paper_2509_22622_amd", "csrc", source)
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attn_stream.s")
        subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-S", "--cuda-device-only", src, "-o", out], check=True, capture_output=True)
        text = open(out).read()
    spills = dict(re.findall(r"\.name:\s+(\S+)[\s\S]*?\.vgpr_spill_count:\s+(\d+)", text))
    stream = {k: int(v) for k, v in spills.items() if kernel + "I" in k}
    assert len(stream) >= 6 and all(v == 0 for v in stream.values()), f"spills: {stream}"


def test_backward_kernels_do_not_spill():
    """The two backward kernels of the train-time rule issue their LDS fragment reads by hand, with counted waits:
    a spill of a fragment register between its read and its wait would store stale data."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(ROOT, "paper_2509_22622_amd", "csrc", "attn_bwd.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attn_bwd.s")
        subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-S", "--cuda-device-only", src, "-o", out], check=True, capture_output=True)
        text = open(out).read()
    spills = dict(re.findall(r"\.name:\s+(\S+)[\s\S]*?\.vgpr_spill_count:\s+(\d+)", text))
    kernels = {k: int(v) for k, v in spills.items() if "ll_bwd_dq_kernel" in k or "ll_bwd_dkv_kernel" in k}
    assert len(kernels) == 4 and all(v == 0 for v in kernels.values()), f"spills: {kernels}"
