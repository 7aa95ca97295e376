"""Guards on the generated gfx950 code (cross-compiled here, no GPU needed):
the hot kernels keep everything in registers, move 128 bits per access through
GLOBAL instructions, do exactly the pinned arithmetic, and contain no packed
fp32 math.  A regression here (a spill, a scalarised access, an unintended
contraction) would not change results but would cost bandwidth or bit-parity
with the oracle."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def asm():
    from paper_2203_13085_amd import build as b
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "lasgd_dev.s")
        flags = [f for f in b.FLAGS if f not in ("-shared", "-fPIC")]
        subprocess.check_call([os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags +
                              ["--cuda-device-only", "-S", "-o", out, b.SRC], stderr=subprocess.DEVNULL)
        return open(out).read()


def _kernel(asm, mangled):
    start = asm.index(mangled + ":")
    end = asm.index(".end_amdhsa_kernel", start)
    return asm[start:end]


def _fast_path(body):
    """Instructions of the branch-free full-tile path: the basic block holding the 128-bit stores."""
    blocks = re.split(r"\n\.LBB\d+_\d+:", body)
    best = max(blocks, key=lambda b: len(re.findall(r"global_store_dwordx4", b)))
    return best


CASES = {
    # kernel                                              loads x4, stores x4, fma
    "_ZN5lasgd12apply_kernelILi1ELi0ELb0ELi3EEEvNS_9ApplyArgsE": (3, 2, 16),    # local_step: g, x, v -> v, x
    "_ZN5lasgd12apply_kernelILi1ELi2ELb0ELi3EEEvNS_9ApplyArgsE": (4, 3, 16),    # step_merge: g, x, v, s (+z) -> v, x, s
    "_ZN5lasgd12apply_kernelILi1ELi1ELb0ELi3EEEvNS_9ApplyArgsE": (2, 2, 0),     # merge: x, s (+z) -> x, s
    "_ZN5lasgd12apply_kernelILi1ELi3ELb0ELi3EEEvNS_9ApplyArgsE": (1, 1, 0),     # snapshot: x -> s
}


@pytest.mark.parametrize("name", list(CASES))
def test_hot_kernels_keep_their_shape(asm, name):
    loads, stores, fmas = CASES[name]
    body = _kernel(asm, name)
    assert re.search(r"\.amdhsa_private_segment_fixed_size 0\b", body), "scratch memory in use (spill or indexed array)"
    assert not re.search(r"\bscratch_(load|store)", body)
    assert not re.search(r"v_pk_(add|mul|fma)_f32", body), "packed fp32 math must stay off"
    fast = _fast_path(body)
    n_st = len(re.findall(r"global_store_dwordx4", fast))
    n_ld = len(re.findall(r"global_load_dwordx4 .* nt", fast))
    assert n_st == stores, (n_st, stores)
    assert n_ld >= loads, (n_ld, loads)
    assert not re.search(r"flat_(load|store)_dwordx4", body), "128-bit accesses must be GLOBAL, not FLAT"
    if fmas:
        assert len(re.findall(r"v_fma(c|ak|mk)?_f32", fast)) >= fmas - 4   # nesterov's fma may sit behind a select
    vgpr = int(re.search(r"\.amdhsa_next_free_vgpr (\d+)", body).group(1))
    assert vgpr <= 64, f"{vgpr} VGPRs: occupancy would drop below 8 waves per SIMD"


def test_no_kernel_uses_packed_fp32(asm):
    assert not re.search(r"v_pk_(add|mul|fma)_f32", asm)
