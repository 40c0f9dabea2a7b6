"""The library used from plain C (tests/c_abi/smoke.c), with no Python or PyTorch in the process."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BIN = os.path.join(ROOT, "paper_2412_11741_amd", "csr_c_smoke.bin")


def test_encode_reconstruct_decode_from_a_c_program():
    if not os.path.exists(BIN):
        from paper_2412_11741_amd import build
        build.build_c_smoke()
    r = subprocess.run([BIN], capture_output=True, text=True, timeout=100)
    print(r.stdout)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert "c abi smoke ok" in r.stdout
