"""GPU parity at the benchmark's full sizes and launch configuration.

The whole method is element-wise across parameters (replicas meet only in the
mean of the same element), so the oracle can compute any subset of parameter
columns exactly.  Each test runs Algorithm 1 on the full workload on the GPU
(default launch shape, mean on the side stream, as bench.py times it) and on
the oracle for a sample of columns: the first and last elements of every
tensor, a band around every tile boundary of the largest and smallest
tensors, and random columns.  The caller-visible parameters are compared on
the sample after every step; momentum, sent models, mean (and the fp32
master for bf16 storage) at the end and once mid-run.

Gradients are drawn on the device with a seeded generator (an input recipe,
not part of the method); the sampled columns are copied to the host so both
sides consume the same bits.
"""
import numpy as np
import pytest
import torch

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W
from tests.parity_util import assert_close, say

pytestmark = pytest.mark.gpu


def _sample_columns(numels, rng, n_random):
    off = np.concatenate([[0], np.cumsum(numels)]).astype(np.int64)
    picks = []
    for t, n in enumerate(numels):
        edge = np.unique(np.clip(np.concatenate([np.arange(0, 9), np.arange(n - 9, n)]), 0, n - 1))
        picks.append(off[t] + edge)
    order = np.argsort(numels)
    for t in list(order[:3]) + list(order[-3:]):          # smallest and largest tensors: tile boundaries
        n = numels[t]
        b = np.arange(256, n, 256)
        if b.size > 64:
            b = b[rng.choice(b.size, 64, replace=False)]
        band = (b[:, None] + np.arange(-4, 5)[None, :]).ravel()
        picks.append(off[t] + np.clip(band, 0, n - 1))
    picks.append(rng.integers(0, off[-1], n_random))
    cols = np.unique(np.concatenate(picks))
    tensor_of = np.searchsorted(off, cols, side="right") - 1
    counts = np.bincount(tensor_of, minlength=len(numels))
    assert counts.min() >= 1
    return cols, counts


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_sampled_columns(cfg):
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.config(cfg)
    bf16 = w.storage == "bf16"
    rng = np.random.default_rng(100 + cfg)
    cols, counts = _sample_columns(w.numels, rng, 60000)
    say(f"[full] configs[{cfg}] {w.name}: K={w.K} N={w.N} sample={cols.size} columns, T={w.T}, m={w.m}")
    nt = len(w.numels)
    wd = [w.weight_decay] * nt
    x0 = np.concatenate([W.initial_tensor(w, t) for t in range(nt)])
    if bf16:
        x0 = W.to_bf16_bits(x0)
    dev = DeviceReplicas(w, weight_decay=wd, side_stream=True)
    try:
        say(f"[full] launch shape {dev.ctx.get_tuning()}")
        dcols = dev._idx[torch.from_numpy(cols).to(dev.dev)]            # positions in the padded device buffers
        orc = O32.Oracle(w.K, [int(c) for c in counts], w.momentum, w.nesterov, wd, storage=w.storage)
        orc.set_model(x0[cols])
        dev.load_model(x0)
        gen = torch.Generator(device=dev.dev)

        def new_grads(step):
            dev.ctx.sync()
            out = []
            for k in range(w.K):
                gen.manual_seed(1_000_003 * w.seed + 7919 * step + k)
                g = torch.randn(dev.g[k].numel(), generator=gen, device=dev.dev) * 1e-3
                dev.g[k].copy_(g.to(dev.g[k].dtype))
                s = dev.g[k][dcols]
                out.append(s.view(torch.int16).cpu().numpy().view(np.uint16) if bf16 else s.cpu().numpy())
            torch.cuda.synchronize()
            return out

        def check_params(step):
            dev.ctx.sync()
            for k in range(w.K):
                got = dev.x[k][dcols]
                if bf16:
                    np.testing.assert_array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), orc.x16[k],
                                                  err_msg=f"bf16 params step {step} replica {k}")
                else:
                    assert_close(got.cpu().numpy(), orc.x[k], f"x step {step} replica {k}")

        def check_all(step):
            for k in range(w.K):
                assert_close(dev.ctx.read_state(B.STATE_V, k)[cols], orc.v[k], f"v step {step} replica {k}")
                assert_close(dev.ctx.read_state(B.STATE_S, k)[cols], orc.s[k], f"s step {step} replica {k}")
                if bf16:
                    assert_close(dev.ctx.read_state(B.STATE_X, k)[cols], orc.x[k], f"master step {step} replica {k}")
            assert_close(dev.ctx.read_state(B.STATE_Z)[cols], orc.z, f"z step {step}", exact=False)

        g = new_grads(0)
        orc.prologue(g, w.lr)
        dev.prologue(w.lr)
        check_params(0)
        tau = 0
        for i in range(1, w.T + 1):
            g = new_grads(i)
            orc.iteration(g, w.lr, w.m)
            tau = dev.iteration(w.lr, tau, w.m)
            check_params(i)
            if i == w.m and w.K <= 16:
                check_all(i)
        check_all(w.T)
        say(f"[full] configs[{cfg}] ok")
    finally:
        dev.close()
        del dev
        torch.cuda.empty_cache()


def test_one_huge_tensor_64bit_offsets():
    """A single tensor of 2^30 + 3 elements (4 GiB per array), K = 2: element offsets inside a
    tensor, arena offsets and replica strides all exceed 32 bits' worth of bytes; the tail is
    ragged.  Inputs are drawn on the device; the oracle follows a sample of columns."""
    import dataclasses
    from paper_2203_13085_amd.driver import DeviceReplicas
    n = (1 << 30) + 3
    w = dataclasses.replace(W.small(K=2, numels=(n,), m=2, T=3), name="huge")
    rng = np.random.default_rng(9)
    cols = np.unique(np.concatenate([np.arange(0, 16), np.arange(n - 16, n), rng.integers(0, n, 50000),
                                     (1 << 29) + np.arange(-8, 8), (1 << 30) + np.arange(-8, 3)]))
    wd = [w.weight_decay]
    dev = DeviceReplicas(w, weight_decay=wd)
    try:
        say(f"[huge] N={n} K={w.K} sample={cols.size}")
        dcols = torch.from_numpy(cols).to(dev.dev)
        gen = torch.Generator(device=dev.dev)
        gen.manual_seed(77)
        x0 = torch.randn(n, generator=gen, device=dev.dev) * 0.01
        for k in range(w.K):
            dev.x[k][:n].copy_(x0)
        torch.cuda.synchronize()
        orc = O32.Oracle(w.K, [cols.size], w.momentum, w.nesterov, wd)
        orc.set_model(x0[dcols].cpu().numpy())
        del x0

        def new_grads(step):
            dev.ctx.sync()
            out = []
            for k in range(w.K):
                gen.manual_seed(1000 * step + k)
                dev.g[k][:n].normal_(0.0, 1e-3, generator=gen)
                out.append(dev.g[k][dcols].cpu().numpy())
            torch.cuda.synchronize()
            return out

        def check(step):
            for k in range(w.K):
                dev.ctx.sync()
                assert_close(dev.x[k][dcols].cpu().numpy(), orc.x[k], f"x step {step} replica {k}")
                assert_close(dev.ctx.read_state(B.STATE_V, k)[cols], orc.v[k], f"v step {step} replica {k}")
                assert_close(dev.ctx.read_state(B.STATE_S, k)[cols], orc.s[k], f"s step {step} replica {k}")
            assert_close(dev.ctx.read_state(B.STATE_Z)[cols], orc.z, f"z step {step}")

        g = new_grads(0)
        orc.prologue(g, w.lr); dev.prologue(w.lr)
        check(0)
        tau = 0
        for i in range(1, w.T + 1):
            g = new_grads(i)
            orc.iteration(g, w.lr, w.m)
            tau = dev.iteration(w.lr, tau, w.m)
        check(w.T)
    finally:
        dev.close()
        del dev
        torch.cuda.empty_cache()
