"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side code: the C oracle, and the host half of
libcommvq (validation, planning, workspace carving) driven through planner handles.  Device code is not
instrumented (sanitizers run on host code only here); nothing in this file touches a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/lib/llvm/bin/clang"


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), res.stdout[-4000:], res.stderr[-4000:])
    return res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-g", "-O1", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
          "-pthread", "-o", exe, os.path.join(ROOT, "oracle", "commvq_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-lm"])
    assert "oracle_driver: ok" in _run([exe])


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if not (os.path.exists(HIPCC) and os.path.exists(CLANG)):
        pytest.skip("no hipcc")
    lib = str(tmp_path / "libcommvq_san.so")
    src = [os.path.join(ROOT, "paper_2506_18879_amd", "csrc", f) for f in ("commvq.hip", "commvq_encode.hip", "commvq_em.hip", "commvq_vbits.hip")]
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
          "-I" + os.path.join(ROOT, "include"), "-o", lib, *src])
    exe = str(tmp_path / "host_driver")
    _run([CLANG, "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-I" + os.path.join(ROOT, "include"),
          "-o", exe, os.path.join(SAN, "host_driver.c"), "-L" + str(tmp_path), "-lcommvq_san", "-Wl,-rpath," + str(tmp_path)])
    assert "host_driver: ok" in _run([exe])


def test_binary_value_row_order_matches_the_kernel_lane_mapping(tmp_path):
    """vbits_code_bit (shared by the value kernel, the output kernels and the codebook packing) against the lane
    mapping written out in the test program: a host-only build of the header."""
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "vbits_rows")
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-std=c++17", "-I" + os.path.join(ROOT, "paper_2506_18879_amd", "csrc"),
          "-o", exe, os.path.join(SAN, "vbits_rows.hip")])
    assert "vbits_rows: ok" in _run([exe])
