"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host build, no GPU).

oracle/sanitize_driver.c walks Algorithm 1 through every function of lasgd_oracle.c
with each (replica, tensor, array) in a heap block of exactly its size; the build
aborts on the first out-of-bounds access, misaligned access, signed overflow or
invalid shift.  Its output must equal, bit for bit, the same schedule run through
the regular build of the oracle that all other tests use.
"""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NUMELS = (5, 1024, 1, 4099, 260, 64)
WD = (0.0, 1e-3, 1e-2, 1e-4, 0.0, 5e-4)


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    d = tmp_path_factory.mktemp("san")
    exe = str(d / "sanitize_driver")
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
                           os.path.join(ROOT, "oracle", "sanitize_driver.c"),
                           os.path.join(ROOT, "oracle", "lasgd_oracle.c"), "-lm"])
    return exe


def _inputs(w, T):
    nt = len(w.numels)
    x0 = np.concatenate([W.initial_tensor(w, t) for t in range(nt)])
    grads = [[np.concatenate([W.gradient_tensor(w, step, k, t) for t in range(nt)]) for k in range(w.K)]
             for step in range(T + 1)]
    if w.storage == "bf16":
        x0 = W.to_bf16_bits(x0)
        grads = [[W.to_bf16_bits(g) for g in gs] for gs in grads]
    return x0, grads


@pytest.mark.parametrize("storage", ["f32", "bf16"])
@pytest.mark.parametrize("alpha,beta", [(1.0, 1.0), (0.5, 0.75)])
@pytest.mark.parametrize("nesterov", [True, False])
def test_oracle_schedule_is_clean_under_asan_and_ubsan(driver, tmp_path, storage, alpha, beta, nesterov):
    K, T, m = 3, 6, 2
    w = W.small(K=K, numels=NUMELS, storage=storage, m=m, T=T, nesterov=nesterov)
    x0, grads = _inputs(w, T)
    elastic = int(alpha != 1.0 or beta != 1.0)
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<8i", K, len(NUMELS), T, m, int(nesterov), int(storage == "bf16"), elastic, 0))
        f.write(struct.pack("<4f", w.lr, w.momentum, alpha, beta))
        f.write(np.asarray(NUMELS, dtype=np.int64).tobytes())
        f.write(np.asarray(WD, dtype=np.float32).tobytes())
        f.write(x0.tobytes())
        for gs in grads:
            for g in gs:
                f.write(g.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([driver, inp, outp], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, f"sanitizer or driver failure:\n{r.stdout}\n{r.stderr}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr

    # the same schedule through the regular build
    o = O32.Oracle(K, NUMELS, w.momentum, nesterov, WD, storage=storage)
    o.set_model(x0)
    o.local_step(grads[0], w.lr); o.snapshot(); o.average(beta=beta)
    tau = 0
    for i in range(1, T + 1):
        o.local_step(grads[i], w.lr)
        tau += 1
        if tau == m:
            o.merge(resnapshot=True, alpha=alpha); o.average(beta=beta)
            tau = 0
    N = sum(NUMELS)
    raw = open(outp, "rb").read()
    pos = 0

    def take(count, dtype):
        nonlocal pos
        a = np.frombuffer(raw, dtype=dtype, count=count, offset=pos)
        pos += a.nbytes
        return a

    def same(a, b, what):
        np.testing.assert_array_equal(a.view(np.uint32) if a.dtype == np.float32 else a,
                                      b.view(np.uint32) if b.dtype == np.float32 else b, err_msg=what)

    for name, arr in (("x", o.x), ("v", o.v), ("s", o.s)):
        for k in range(K):
            same(take(N, np.float32), arr[k], f"{name}[{k}]")
    same(take(N, np.float32), o.z, "z")
    if storage == "bf16":
        for k in range(K):
            same(take(N, np.uint16), o.x16[k], f"x16[{k}]")
    for _ in range(2):
        o.sgd_ar_step(grads[T], w.lr)
    for name, arr in (("x", o.x), ("v", o.v)):
        for k in range(K):
            same(take(N, np.float32), arr[k], f"{name}[{k}] after the comparator steps")
    if storage == "bf16":
        for k in range(K):
            same(take(N, np.uint16), o.x16[k], f"x16[{k}] after the comparator steps")
    r1, r2 = take(2, np.uint16)
    w1 = take(1, np.float32)[0]
    L = O32.lib()
    assert r1 == L.lasgd_oracle_bf16_rne(np.float32(1.00390625) + np.float32(0.001))
    assert r2 == L.lasgd_oracle_bf16_rne(np.float32(1.00390625)) == 0x3F80          # a tie rounds to even
    assert w1 == L.lasgd_oracle_bf16_widen(int(r1))
    assert pos == len(raw)


def test_harness_catches_a_planted_overrun(tmp_path):
    """A copy of the oracle whose snapshot copies one element too many must be stopped by the
    sanitizer build (the planted mistake lives in the copy, on the CPU, only)."""
    src = open(os.path.join(ROOT, "oracle", "lasgd_oracle.c")).read()
    good = "    for (int64_t e = 0; e < n; ++e)\n        s[e] = x[e];"
    assert src.count(good) == 1
    bad_c = tmp_path / "oracle_overrun.c"
    bad_c.write_text(src.replace(good, good.replace("e < n", "e <= n")))
    exe = str(tmp_path / "driver_overrun")
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
                           os.path.join(ROOT, "oracle", "sanitize_driver.c"), str(bad_c), "-lm"])
    w = W.small(K=2, numels=(5, 64), m=1, T=1)
    x0, grads = _inputs(w, 1)
    inp = str(tmp_path / "in.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<8i", 2, 2, 1, 1, 1, 0, 0, 0))
        f.write(struct.pack("<4f", w.lr, w.momentum, 1.0, 1.0))
        f.write(np.asarray((5, 64), dtype=np.int64).tobytes())
        f.write(np.asarray((0.0, 0.0), dtype=np.float32).tobytes())
        f.write(x0.tobytes())
        for gs in grads:
            for g in gs:
                f.write(g.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:abort_on_error=0")
    r = subprocess.run([exe, inp, str(tmp_path / "out.bin")], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "heap-buffer-overflow" in r.stderr
