"""The library driven from plain C (tests/c_abi_example.c): no Python, no torch in the process that
computes.  The program converts a small matrix, runs SpMM (with a cut window) and SDDMM and compares
both bit for bit with host loops, checks the transposed CSR bit for bit and the fused attention call
against a double-precision loop; exit code 0 means everything matched."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_c_program_runs_the_library_through_its_c_abi():
    exe = os.path.join(HERE, "c_abi_example")
    if not os.path.exists(exe):  # normally built beforehand by python -m paper_2412_11007_amd.build (one gcc call)
        from paper_2412_11007_amd.build import build_c_example
        build_c_example()
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(res.stdout, res.stderr)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("OK")
