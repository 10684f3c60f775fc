"""Host-side sanitizer builds (CPU only, no GPU code is run).

* The CPU oracle, compiled with gcc AddressSanitizer + UndefinedBehaviorSanitizer, is driven through every entry point
  on small exact-size heap buffers (tests/sanitize/oracle_driver.c).
* The host side of the C ABI (csrc/akvq_api.hip: validation, size helpers, descriptor marshalling), compiled with the
  same sanitizers on the host pass only, is driven with the kernel launchers replaced by stubs
  (tests/sanitize/api_driver.cpp); this build found two signed overflows at the top of the int range (workspace sizing
  of the pivot score, the KV-split partition), now computed in 64 bits.
Any report aborts the driver (-fno-sanitize-recover=all), which fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def _run(cmd, exe):
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stdout + build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=600)
    assert run.returncode == 0 and run.stdout.startswith("ok "), run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    return run.stdout


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", *SAN, "-ffp-contract=off", "-fopenmp",
          "-I" + os.path.join(ROOT, "oracle"), os.path.join(ROOT, "oracle", "akvq_oracle.c"),
          os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"], exe)


def test_abi_host_side_under_address_and_ub_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "api_san")
    host_san = [x for flag in SAN for x in ("-Xarch_host", flag)]   # the sanitizers instrument the host pass only
    out = _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *host_san,
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                os.path.join(ROOT, "paper_2501_15021_amd", "csrc", "akvq_api.hip"),
                "-x", "hip", os.path.join(ROOT, "tests", "sanitize", "api_driver.cpp"), "-o", exe], exe)
    assert int(out.split()[1]) >= 30      # the well-formed calls all reached their (stub) launcher
