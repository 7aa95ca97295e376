"""The C ABI used from plain C: tests/c_abi/abi_check.c links the HIP library and
the oracle, runs Algorithm 1 through include/lasgd.h with buffers from the HIP
runtime (no Python, no torch in that process) and compares every array after
every step, bit for bit; with fused = 1 the global update and the next mean go
out as lasgd_step_merge_average, and every run ends with a call of the
allocation-free lasgd_global_update_static checked against the oracle.  The
program is built by __graft_entry__.build()."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "abi_check")


@pytest.mark.parametrize("K,m,T,fused", [(3, 2, 6, 0), (1, 1, 3, 0), (8, 4, 8, 0), (64, 3, 4, 0),
                                         (3, 1, 5, 1), (16, 2, 6, 1), (40, 1, 3, 1)])
def test_plain_c_consumer(K, m, T, fused):
    assert os.path.exists(EXE), "build it first: python __graft_entry__.py"
    r = subprocess.run([EXE, str(K), str(m), str(T), str(fused)], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stderr
    assert "PASS" in r.stdout
