"""The C ABI driven by a plain C program (no Python binding, no torch): tests/abi_c_client.c
allocates device memory with hipMalloc, runs 80 ticks of a seeded 3v3 batch through
tabx_reset / tabx_step / tabx_observe / tabx_step_observe and compares every tick with the CPU
checker bit for bit (needs an MI355X)."""
import subprocess
import sys

import pytest

from tests import c_client

pytestmark = pytest.mark.gpu


def test_plain_c_program_matches_checker():
    if c_client.is_stale():
        c_client.build()
    print("[gpu] tests/abi_c_client", flush=True)
    sys.stdout.flush()
    r = subprocess.run([c_client.BINARY], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi_c_client: PASS" in r.stdout
