"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer.

tests/sanitize/host_driver.cpp is built together with the CPU oracle and with
libfsdp_flat's sources, the host side of which is instrumented (the layout
planner, every entry point's argument validation, the batch bookkeeping); the
device code is compiled as usual and never runs: the driver only makes calls
that the host must reject, so no GPU is needed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2304_11277_amd", "csrc")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
HIPCC = shutil.which("hipcc") or os.path.join(ROCM, "bin", "hipcc")
CLANG = os.path.join(ROCM, "llvm", "bin", "clang")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-4000:]}"
    return r.stdout


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="needs the ROCm compilers")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    lib = tmp_path / "libfsdp_flat_san.so"
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san, "-I", os.path.join(ROOT, "include"),
          os.path.join(CSRC, "fsdp_kernels.hip"), os.path.join(CSRC, "fsdp_layout.cpp"), "-o", str(lib)])
    orc = tmp_path / "fsdp_oracle.o"
    _run([CLANG, "-O1", "-g", "-std=gnu99", "-ffp-contract=off", *SAN, "-c",
          os.path.join(ROOT, "oracle", "fsdp_oracle.c"), "-o", str(orc)])
    exe = tmp_path / "host_driver"
    _run([CLANG + "++", "-O1", "-g", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
          os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), str(orc), "-L", str(tmp_path), "-lfsdp_flat_san",
          "-lm", f"-Wl,-rpath,{tmp_path}", "-o", str(exe)])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    out = _run([str(exe)], env=env, timeout=300)
    assert "ALL OK" in out, out[-4000:]
