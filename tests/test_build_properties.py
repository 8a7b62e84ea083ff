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


def test_library_keeps_no_mutable_state_of_its_own():
    """Writable data of the built library: the HIP toolchain's registration
    objects, the kernels' launch stubs, and the per-thread last-error value.
    Nothing else: no process-wide switch that one caller could flip under
    another (the rank walk is an option of each layout)."""
    from paper_2304_11277_amd import build as fbuild
    lib = fbuild.build_lib(force=False)
    nm = shutil.which("nm")
    if nm is None:
        pytest.skip("needs nm")
    out = subprocess.check_output([nm, "-C", "--defined-only", lib], text=True)
    own = []
    for line in out.splitlines():
        parts = line.split(None, 2)
        if len(parts) < 3 or parts[1] not in "bBdD":
            continue
        name = parts[2]
        if "_kernel" in name and "(" in name:             # device-function handles: written once by the loader
            continue
        if name.startswith(("__hip_", "__do_", "__dso_handle", "__init", "__fini", "_DYNAMIC", "_GLOBAL_OFFSET_TABLE_",
                            "DW.ref.", "completed.", "__TMC_END__", "__frame_dummy", "__JCR")):
            continue
        own.append(name)
    assert own == ["(anonymous namespace)::g_last_hip_error"], own
    tls = subprocess.check_output([shutil.which("readelf") or "readelf", "-sW", lib], text=True)
    assert re.search(r"\bTLS\b.*g_last_hip_error", tls), "the last-error value must be thread-local"
