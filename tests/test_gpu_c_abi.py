"""The C ABI from plain C: tests/c_abi_roundtrip.c (built by __graft_entry__.build()) runs select -> append -> decode
with HIP-runtime memory only and checks the results against the C oracle inside the same process."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_round_trip():
    exe = os.path.join(ROOT, "tests", "c_abi_roundtrip.bin")
    if not os.path.exists(exe):          # normally built by __graft_entry__.build(); gcc only, a second
        import __graft_entry__ as entry
        from oracle import pyoracle
        from paper_2501_15021_amd import binding
        entry.build_c_abi_check(binding.LIB_PATH, pyoracle.build())
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "PASS c_abi_roundtrip" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
