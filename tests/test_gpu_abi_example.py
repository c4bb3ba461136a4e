"""The C ABI driven by a plain C program: no Python between the caller and the library."""
import subprocess

import pytest

pytestmark = pytest.mark.gpu


def test_c_program_drives_the_abi(torch_cuda):
    from tests.abi_example import build
    exe = build.build(force=False)  # built with the library; compiled here only if missing
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "abi_example: OK" in run.stdout
