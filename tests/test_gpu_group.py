"""GPU parity of the replica-group kernels (one workgroup per tile, one wave per
replica, the K values of an element meeting in LDS): lasgd_step_merge_average
against the oracle's global update + mean, and lasgd_sgd_ar_step against the
oracle's mean-gradient step, for every replica count that changes the group's
shape (1 wave, up to 16 waves, two replicas per wave, two passes)."""
import dataclasses

import numpy as np
import pytest

from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W
from tests.parity_util import assert_close, compare_state, packed_inputs, run_parity, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("K", [1, 2, 3, 8, 16, 17, 31, 32, 33, 64])
def test_fused_mean_every_group_shape(K):
    # ragged list: full rows, a scalar tail, a one-element tensor, several tiles
    w = W.small(K=K, numels=(1030, 1, 4, 257, 768), m=2, T=5)
    wd = [0.0, 1e-3, 1e-2, 1e-4, 5e-4]
    assert run_parity(w, weight_decay=wd, fused_mean=True) == 0        # z bit-exact: the sum runs in replica order


@pytest.mark.parametrize("vec", [1, 2, 4])
@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_fused_mean_tile_sizes_and_storage(vec, storage):
    w = W.small(K=5, numels=(3000, 7, 513, 256, 1025, 2), storage=storage, m=1, T=5)
    assert run_parity(w, tuning=dict(vec=vec), fused_mean=True) == 0


def test_fused_mean_bf16_two_passes_heavy_ball():
    w = W.small(K=40, numels=(2048, 12, 999), storage="bf16", m=3, T=6, nesterov=False)
    assert run_parity(w, fused_mean=True, tuning=dict(nontemporal=3)) == 0


def test_fused_mean_grid_cap_and_same_stream():
    w = W.small(K=8, numels=(20000, 33, 4096), m=1, T=4)
    assert run_parity(w, tuning=dict(max_blocks=3), fused_mean=True, side_stream=False) == 0


def test_fused_mean_mobilenet_list_every_step():
    # the workload this call is meant for: K = 16, a global update every step (reduced T)
    w = dataclasses.replace(W.config(3), T=2)
    assert run_parity(w, fused_mean=True) == 0


def test_fused_mean_mixes_with_the_two_stream_calls():
    """Cycles alternate between step_merge + average (side stream) and the fused call;
    average_done works after either; the protocol errors are the documented ones."""
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=6, numels=(5000, 3, 700), m=1, T=8)
    wd = [w.weight_decay] * len(w.numels)
    x0, grads = packed_inputs(w)
    orc = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
    dev = DeviceReplicas(w, weight_decay=wd, side_stream=True)
    c = dev.ctx
    try:
        c.set_tuning(avg_split=1)
        orc.set_model(x0); dev.load_model(x0)
        dev.load_grads(grads(0))
        c.local_step(w.lr)
        with pytest.raises(B.LasgdError) as e:           # nothing sent, no mean pending
            c.step_merge_average(w.lr)
        assert e.value.status == B.ERR_STATE
        c.snapshot(); c.average()
        orc.prologue(grads(0), w.lr)
        compare_state(dev, orc, 0)
        for i in range(1, w.T + 1):
            g = grads(i)
            dev.load_grads(g)
            orc.iteration(g, w.lr, 1)
            if i % 2:
                c.step_merge_average(w.lr)
            else:
                c.step_merge(w.lr, True); c.average()
            c.sync()
            assert c.average_done()
            with pytest.raises(B.LasgdError) as e:       # a mean is pending: s may not be overwritten
                c.snapshot()
            assert e.value.status == B.ERR_STATE
            compare_state(dev, orc, i)
        # partly merged pending mean: the fused call must refuse
        c.merge_ex(0b000111, True)
        with pytest.raises(B.LasgdError) as e:
            c.step_merge_average(w.lr)
        assert e.value.status == B.ERR_STATE
        c.merge_ex(0b111000, True)
        c.average()
        c.set_elastic(0.5, 1.0)
        with pytest.raises(B.LasgdError) as e:
            c.step_merge_average(w.lr)
        assert e.value.status == B.ERR_STATE
    finally:
        dev.close()


@pytest.mark.parametrize("m", [1, 3])
def test_fused_mean_graph_replay_equals_eager(m):
    """m-1 local steps + the fused call captured as one graph and replayed several times, with
    eager library work and host synchronisation between the replays: every replay must give the
    oracle's state (z included: the graph writes it in place)."""
    import torch
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=4, numels=(70000, 5, 1024, 4099), m=m)
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay] * len(w.numels)
    dev = DeviceReplicas(w, weight_decay=wd)
    o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
    try:
        g = grads(1)
        o.set_model(x0); dev.load_model(x0); dev.load_grads(g)
        o.prologue(g, w.lr); dev.prologue(w.lr)
        # one eager cycle through the fused call: from here on z is made on the main stream
        for _ in range(m):
            o.iteration(g, w.lr, m)
        for _ in range(m - 1):
            dev.ctx.local_step(w.lr)
        dev.ctx.step_merge_average(w.lr)
        graph = dev.capture_fused_cycle(w.lr, m)
        with pytest.raises(B.LasgdError) as e:           # recorded, not launched: nothing to poll
            dev.ctx.average_done()
        assert e.value.status == B.ERR_STATE
        for rep in range(5):
            with torch.cuda.stream(dev.main):
                graph.replay()
            for _ in range(m):
                o.iteration(g, w.lr, m)
            compare_state(dev, o, rep)
            if rep % 2 == 0:                             # an eager cycle in between, two-stream calls
                for _ in range(m - 1):
                    dev.ctx.local_step(w.lr)
                dev.ctx.step_merge(w.lr, True)
                dev.ctx.average()
                for _ in range(m):
                    o.iteration(g, w.lr, m)
                dev.ctx.sync()
                assert dev.ctx.average_done()
                # back to "z made on the main stream" before the next replay
                for _ in range(m - 1):
                    dev.ctx.local_step(w.lr)
                dev.ctx.step_merge_average(w.lr)
                for _ in range(m):
                    o.iteration(g, w.lr, m)
        with torch.cuda.stream(dev.main):                # back to back, no host synchronisation
            graph.replay()
            graph.replay()
        for _ in range(2 * m):
            o.iteration(g, w.lr, m)
        compare_state(dev, o, 99)
    finally:
        dev.close()


@pytest.mark.parametrize("storage,K", [("f32", 1), ("f32", 3), ("f32", 8), ("bf16", 16), ("f32", 17), ("bf16", 33),
                                       ("f32", 64)])
def test_sgd_ar_every_group_shape(storage, K):
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=K, numels=(1030, 1, 4, 257, 768), storage=storage)
    wd = [1e-3, 0.0, 1e-2, 1e-4, 0.0]
    x0, grads = packed_inputs(w)
    orc = O32.Oracle(K, w.numels, w.momentum, w.nesterov, wd, storage=storage)
    dev = DeviceReplicas(w, weight_decay=wd)
    try:
        say(f"[sgd-ar] K={K} storage={storage}")
        orc.set_model(x0); dev.load_model(x0)
        for i in range(4):
            g = grads(i)
            dev.load_grads(g)
            orc.sgd_ar_step(g, w.lr)
            dev.ctx.sgd_ar_step(w.lr)
            for k in range(K):
                assert_close(dev.ctx.read_state(B.STATE_X, k), orc.x[k], f"x step {i} replica {k}")
                assert_close(dev.ctx.read_state(B.STATE_V, k), orc.v[k], f"v step {i} replica {k}")
                if storage == "bf16":
                    np.testing.assert_array_equal(dev.params(k), orc.x16[k])
    finally:
        dev.close()
