"""Shared helpers of the GPU parity tests: run Algorithm 1 on the HIP library
and on the CPU oracle with the same seeded inputs and compare state after
every step.

Acceptance bar (stated by the benchmark spec for fp32 parameters, after every step):
    |gpu - oracle| <= 1e-7 + 1e-6 * |oracle|
Both sides pin the same fp32 evaluation order, so x, v and s are also
expected to agree bit for bit, and z too when the kernel sums the replicas in
index order; the tests assert that stronger statement where it is expected.
"""
from __future__ import annotations

import sys
from typing import Optional, Sequence

import numpy as np

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W

RTOL, ATOL = 1e-6, 1e-7


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def within(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    got64, ref64 = got.astype(np.float64), ref.astype(np.float64)
    return np.abs(got64 - ref64) <= ATOL + RTOL * np.abs(ref64)


def assert_close(got, ref, what: str, exact: bool = True) -> int:
    ok = within(got, ref)
    assert ok.all(), (f"{what}: {int((~ok).sum())} of {ok.size} outside 1e-6 rel / 1e-7 abs, "
                      f"max |d| = {np.abs(got.astype(np.float64) - ref.astype(np.float64)).max():.3e}")
    # +0 and -0 compare equal; anything else must match to the bit
    nbits = int(np.sum((got.view(np.uint32) != ref.view(np.uint32)) & ~((got == 0) & (ref == 0))))
    if exact:
        assert nbits == 0, f"{what}: within tolerance but {nbits} of {got.size} differ in bits"
    return nbits


def packed_inputs(w: W.Workload):
    """(x0, grads(step)) over the packed parameter vector; bf16 storage gets bit patterns."""
    nt = len(w.numels)
    x0 = np.concatenate([W.initial_tensor(w, t) for t in range(nt)])

    def grads(step: int):
        out = [np.concatenate([W.gradient_tensor(w, step, k, t) for t in range(nt)]) for k in range(w.K)]
        return [W.to_bf16_bits(g) for g in out] if w.storage == "bf16" else out

    if w.storage == "bf16":
        x0 = W.to_bf16_bits(x0)
    return x0, grads


def compare_state(dev, orc: O32.Oracle, step: int, z_exact: bool = True, z_valid: bool = True) -> int:
    """Every array of every replica, element by element.  Returns the number of
    z elements that differ in bits (0 unless z_exact is False)."""
    w = dev.w
    for k in range(w.K):
        tag = f"step {step} replica {k}"
        assert_close(dev.ctx.read_state(B.STATE_X, k), orc.x[k], f"x {tag}")
        assert_close(dev.ctx.read_state(B.STATE_V, k), orc.v[k], f"v {tag}")
        assert_close(dev.ctx.read_state(B.STATE_S, k), orc.s[k], f"s {tag}")
        if w.storage == "bf16":
            np.testing.assert_array_equal(dev.params(k), orc.x16[k], err_msg=f"x16 {tag}")
        else:
            np.testing.assert_array_equal(dev.params(k).view(np.uint32), dev.ctx.read_state(B.STATE_X, k).view(np.uint32))
    if not z_valid:
        return 0
    return assert_close(dev.ctx.read_state(B.STATE_Z), orc.z, f"z step {step}", exact=z_exact)


def run_parity(w: W.Workload, weight_decay: Optional[Sequence[float]] = None, fused: bool = True,
               tuning: Optional[dict] = None, side_stream: bool = True, z_exact: bool = True,
               every_step: bool = True, fused_mean: bool = False) -> int:
    """Prologue + w.T iterations on both sides; compare after every step."""
    from paper_2203_13085_amd.driver import DeviceReplicas
    wd = list(weight_decay) if weight_decay is not None else [w.weight_decay] * len(w.numels)
    x0, grads = packed_inputs(w)
    orc = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd, storage=w.storage)
    dev = DeviceReplicas(w, weight_decay=wd, side_stream=side_stream)
    zdiff = 0
    try:
        if tuning:
            dev.ctx.set_tuning(**tuning)
        say(f"[parity] {w.name} K={w.K} N={w.N} tensors={len(w.numels)} storage={w.storage} "
            f"fused={fused} fused_mean={fused_mean} nesterov={w.nesterov} tuning={dev.ctx.get_tuning()}")
        orc.set_model(x0)
        dev.load_model(x0)
        g = grads(0)
        orc.prologue(g, w.lr)
        dev.load_grads(g)
        dev.prologue(w.lr)
        zdiff += compare_state(dev, orc, 0, z_exact)
        tau = 0
        for i in range(1, w.T + 1):
            g = grads(i)
            orc.iteration(g, w.lr, w.m)
            dev.load_grads(g)
            tau = dev.iteration(w.lr, tau, w.m, fused=fused, fused_mean=fused_mean)
            if every_step or i == w.T:
                zdiff += compare_state(dev, orc, i, z_exact)
        say(f"[parity] {w.name} done, z bit differences: {zdiff}")
    finally:
        dev.close()
    return zdiff
