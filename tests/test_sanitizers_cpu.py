"""CPU sanitizer job: the fp64 oracle and the host side of libthi (argument validation, workspace layout,
kernel-choice arithmetic) built with -fsanitize=address,undefined and driven over edge-case inputs.

The kernels themselves are not run: the library's launchers are replaced by host stand-ins
(tests/sanitize/api_stubs.cpp), so no GPU is needed.  A finding makes the driver exit non-zero
(halt_on_error / abort) and its report is shown."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ENV = dict(os.environ,
           ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd[:3])} ... failed ({res.returncode}):\n{res.stdout[-3000:]}\n{res.stderr[-6000:]}"
    return res


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fopenmp", "-o", exe,
          os.path.join(ROOT, "oracle", "thi_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-lm"])
    res = _run([exe], env=ENV)
    assert res.stdout.startswith("ok "), res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]


@pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not found")
def test_library_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "api_san")
    csrc = os.path.join(ROOT, "paper_2605_25655_amd", "csrc")
    res = subprocess.run(
        [HIPCC, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
         "-Xarch_host", "-fno-omit-frame-pointer", "-Wno-unused-command-line-argument", "-o", exe,
         os.path.join(csrc, "api.hip"), os.path.join(csrc, "plan.hip"),
         "-x", "hip", os.path.join(SAN, "api_stubs.cpp"), os.path.join(SAN, "api_driver.cpp")],
        capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-6000:]
    syms = subprocess.run(["nm", exe], capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms, "the host code was not instrumented"
    res = _run([exe], env=ENV)
    assert res.stdout.strip().startswith("ok "), res.stdout[-2000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
