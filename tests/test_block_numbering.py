"""Host logic of the update kernels: the map from block number to block of C."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_every_block_gets_exactly_one_number(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = tmp_path / "block_numbering_check"
    src = os.path.join(HERE, "host", "block_numbering_check.hip")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-o", str(exe), src],
                   check=True, capture_output=True, timeout=600)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "bad 0" in out.stdout
