"""The C ABI used from plain C: tests/c_abi/abi_check.c links the HIP library and
the oracle, runs Algorithm 1 through include/lasgd.h with buffers from the HIP
runtime (no Python, no torch in that process) and compares every array after
every step, bit for bit.  The program is built by __graft_entry__.build()."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "abi_check")


@pytest.mark.parametrize("K,m,T", [(3, 2, 6), (1, 1, 3), (8, 4, 8), (64, 3, 4)])
def test_plain_c_consumer(K, m, T):
    assert os.path.exists(EXE), "build it first: python __graft_entry__.py"
    r = subprocess.run([EXE, str(K), str(m), str(T)], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stderr
    assert "PASS" in r.stdout
