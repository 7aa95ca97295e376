"""The cross-stream ordering of z under the race probe.

With tuning race_probe = 1, lasgd_average fills z with NaN on the side stream
right before the mean rewrites it.  The main stream's next global update must
wait for the end of that mean (the z event); if it did not, it would read NaN
wherever the mean had not arrived yet, and NaN would stay in the parameters for
good.  The probe changes no result when the ordering holds, so the runs are
also compared with the oracle.  Large model, many cycles back to back without
any host synchronisation, global update every step (the mean has no local step
to hide behind: the merge is enqueued while the mean still runs) and every
fourth step."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W
from tests.parity_util import say
from tests.test_gpu_fullsize import HOST_THREADS, assert_same

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("m", [1, 4])
@pytest.mark.parametrize("fused", [True, False])
def test_no_nan_reaches_the_parameters(m, fused):
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = dataclasses.replace(W.config(2), m=m, T=8 * m)          # ResNet-50 list, K = 8: 0.2 ms means, 0.6-0.9 ms steps
    nt = len(w.numels)
    wd = [w.weight_decay] * nt
    x0 = np.concatenate([W.initial_tensor(w, t) for t in range(nt)])
    dev = DeviceReplicas(w, weight_decay=wd, side_stream=True)
    try:
        dev.ctx.set_tuning(race_probe=1, avg_split=1)
        assert dev.ctx.get_tuning()["race_probe"] == 1
        say(f"[race probe] {w.name} m={m} fused={fused}: {w.T} steps without host synchronisation")
        orc = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd, threads=HOST_THREADS)
        orc.set_model(x0)
        dev.load_model(x0)
        gen = torch.Generator(device=dev.dev)
        gen.manual_seed(5)
        g = []
        for k in range(w.K):
            dev.g[k].normal_(0.0, 1e-3, generator=gen)
            g.append(dev._get(dev.g[k]))
        torch.cuda.synchronize()
        dev.prologue(w.lr)
        tau = 0
        for _ in range(w.T):                                     # the same gradients every step: nothing to wait for
            tau = dev.iteration(w.lr, tau, m, fused=fused)
        dev.ctx.sync()
        for k in range(w.K):
            assert not bool(torch.isnan(dev.x[k]).any()), f"NaN in the parameters of replica {k}: a global update read z too early"
        z = dev.ctx.read_state(B.STATE_Z)
        assert not np.isnan(z).any(), "NaN left in z: the mean did not rewrite all of it"
        orc.prologue(g, w.lr)
        for _ in range(w.T):
            orc.iteration(g, w.lr, m)
        for k in range(w.K):
            assert_same(dev.params(k), orc.x[k], f"x replica {k}")
            assert_same(dev.ctx.read_state(B.STATE_S, k), orc.s[k], f"s replica {k}")
        assert_same(z, orc.z, "z")
    finally:
        dev.close()
        del dev
        torch.cuda.empty_cache()


def test_probe_is_off_by_default_and_switches_off_again():
    from paper_2203_13085_amd.driver import DeviceReplicas
    dev = DeviceReplicas(W.small(K=2, numels=(300,)))
    try:
        assert dev.ctx.get_tuning()["race_probe"] == -1
        dev.ctx.set_tuning(race_probe=1)
        assert dev.ctx.get_tuning()["race_probe"] == 1
        dev.ctx.set_tuning(race_probe=-1)
        assert dev.ctx.get_tuning()["race_probe"] == -1
    finally:
        dev.close()
