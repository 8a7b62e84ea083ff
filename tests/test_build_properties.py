"""Properties of the compiled device code that the parity claims rest on
(CPU only: hipcc cross-compiles gfx950 without a GPU)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2304_11277_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_device_code_has_no_packed_fp32_and_no_spills(tmp_path):
    from paper_2304_11277_amd import build as fbuild
    flags = [f for f in fbuild.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    asm = tmp_path / "fsdp_kernels.s"
    subprocess.check_call([HIPCC, *flags, "-x", "hip", os.path.join(CSRC, "fsdp_kernels.hip"), "-I",
                           os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only", "-o", str(asm)],
                          stderr=subprocess.DEVNULL)
    text = asm.read_text()
    kernels = re.findall(r"^\s*\.amdhsa_kernel\s+(\S+)", text, re.M)
    assert len(kernels) > 50, "every template instantiation is a kernel of its own"
    # packed fp32 arithmetic is switched off for the whole library (-packed-fp32-ops)
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", text)
    # the streaming kernels are sized to their register budget: nothing spills to scratch memory
    assert not re.search(r"\bscratch_(load|store)", text)
    for m in re.finditer(r"\.private_segment_fixed_size:\s*(\d+)", text):
        assert int(m.group(1)) == 0
    # -ffp-contract=off is part of the build: the rank-ordered sum must not be fused with the scaling
    assert "-ffp-contract=off" in fbuild.HIPCC_FLAGS and "-fno-fast-math" in fbuild.HIPCC_FLAGS
