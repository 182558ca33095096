"""Host-side check of the packed-weight accumulation helper's code (no GPU needed: hipcc cross-compiles).

fma_bf16x8_t<false> multiplies a pair of bf16 values with (w, 0) or (0, w) in one packed dot-product
instruction.  A weight the compiler knows (a literal 1) must not reach that instruction as an inline
constant: the instruction does not read an inline constant as the pair (w, 0), and the sums then come
out wrong without any error.  The helper hides such weights from the compiler; this test compiles a
kernel that passes literal weights and looks at the instructions."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = r"""
#include "ckv_device.h"
using namespace ckv;
__global__ void literal_weights(const uint4* in, float* out) {
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  fma_bf16x8_t<false>(acc, in[threadIdx.x], 1);
  fma_bf16x8_t<false>(acc, in[threadIdx.x + 64], 3);
  fma_bf16x8(acc, in[threadIdx.x + 128], 2);
  for (int i = 0; i < 8; ++i) out[threadIdx.x * 8 + i] = acc[i];
}
"""


def test_literal_weights_never_become_inline_constants(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    src = tmp_path / "literal_weights.hip"
    src.write_text(SRC)
    out = tmp_path / "literal_weights.s"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I",
           os.path.join(ROOT, "paper_2506_11418_amd", "csrc"), "-S", "--cuda-device-only", str(src), "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    dots = [l.split(";")[0].strip() for l in out.read_text().splitlines() if "v_dot2" in l and "bf16" in l]
    assert len(dots) >= 16                                       # the two narrow calls at least
    for line in dots:
        ops = [o.strip() for o in line.split(None, 1)[1].split(",")]
        assert all(re.fullmatch(r"v\d+|v\[\d+:\d+\]", o) for o in ops[:3]), f"operand that is not a register: {line}"
