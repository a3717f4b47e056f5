"""The library driven from a plain C program (tests/c_abi_client.c): no PyTorch in the process."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "tests", "c_abi_client")


@pytest.mark.gpu
def test_c_client_runs_the_path_and_matches_the_closed_form():
    if not os.path.exists(CLIENT):                     # normally built beforehand by __graft_entry__.build()
        import __graft_entry__
        __graft_entry__.build_c_client()
    proc = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120)
    assert proc.returncode == 0, proc.stdout + proc.stderr
    assert "c_abi_client ok" in proc.stdout
