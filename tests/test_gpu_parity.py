"""GPU parity: the HIP library against the CPU oracle, through the C ABI,
element by element after every step, on the same seeded inputs."""
import dataclasses

import numpy as np
import pytest

from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W
from tests.parity_util import run_parity, say, packed_inputs, assert_close

pytestmark = pytest.mark.gpu


# ---- small ragged lists: several tiles, scalar tails, every launch shape ----
@pytest.mark.parametrize("vec", [1, 2, 4])
@pytest.mark.parametrize("fused", [True, False])
def test_ragged_list_every_tile_shape(vec, fused):
    w = W.small(K=3)
    wd = [0.0 if i % 3 == 0 else 1e-3 * (i + 1) for i in range(len(w.numels))]
    run_parity(w, weight_decay=wd, fused=fused, tuning=dict(vec=vec))


@pytest.mark.parametrize("kper_step,kper_merge", [(1, 1), (2, 3), (5, 5), (3, 2)])
def test_replica_grouping_does_not_change_results(kper_step, kper_merge):
    w = W.small(K=5, numels=(3000, 7, 513, 256, 1025), m=3, T=7)
    run_parity(w, tuning=dict(kper_step=kper_step, kper_merge=kper_merge))


@pytest.mark.parametrize("chunk", [1, 2, 3, 7, 16, 1000, -1])
def test_item_order_does_not_change_results(chunk):
    # 12 + 1 + 3 + 1 + 5 = 22 tiles at vec=1: chunk sizes that divide it, that leave a tail, and beyond it
    w = W.small(K=3, numels=(3000, 7, 513, 256, 1025), m=2, T=4)
    run_parity(w, tuning=dict(chunk_step=chunk, chunk_merge=chunk, kper_merge=2 if chunk == 3 else 1))


def test_heavy_ball_and_plain_sgd():
    run_parity(W.small(K=4, nesterov=False))
    run_parity(W.small(K=4, momentum=0.0, weight_decay=0.0, nesterov=False))


def test_grid_cap_uses_the_stride_loop():
    w = W.small(K=4, numels=(20000, 33, 4096))
    run_parity(w, tuning=dict(max_blocks=3, avg_max_blocks=2, vec=1))


def test_streaming_hints_do_not_change_results():
    for nt in (1, 2, 3):
        run_parity(W.small(K=3), tuning=dict(nontemporal=nt))


def test_same_stream_for_both():
    run_parity(W.small(K=3), side_stream=False)


# ---- degenerate and extreme replica counts -----------------------------------
def test_single_replica():
    # K = 1: the mean is the sent model and the global update is the identity
    run_parity(W.small(K=1, m=1, T=4))


@pytest.mark.parametrize("K", [2, 7, 12, 64])
def test_replica_counts_incl_non_powers_of_two_and_max(K):
    run_parity(W.small(K=K, numels=(1030, 4, 257), m=2, T=4))


def test_merge_every_step():
    run_parity(W.small(K=4, m=1, T=5))


def test_one_element_model():
    run_parity(W.small(K=3, numels=(1,), m=2, T=4))


# ---- the LDS-staged mean -------------------------------------------------------
@pytest.mark.parametrize("K,split", [(16, 2), (16, 4), (32, 4), (5, 4), (3, 2)])
def test_split_mean_staged_through_lds(K, split):
    # summing replica ranges separately changes fp64 rounding only: z may differ
    # from the in-order sum in the last fp32 bit at double-rounding ties, nowhere else
    w = W.small(K=K, numels=(70000, 5, 1024), m=2, T=4)
    ndiff = run_parity(w, tuning=dict(avg_split=split), z_exact=False)
    assert ndiff <= 5


# ---- bf16 storage -----------------------------------------------------------------
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("vec", [1, 2, 4])
def test_bf16_storage(fused, vec):
    # vec 2 and 4: tiles of 512 / 1024 elements, a lane owns 8 consecutive elements of each full
    # 512-element row (128-bit accesses on the bf16 arrays); the sizes below give full tiles,
    # tiles that end inside a row and inside a lane's 8 elements, and tensors smaller than a row
    w = W.small(K=4, numels=(5, 1024, 1, 4099, 260, 64, 2048 + 517, 512), storage="bf16", m=2, T=6)
    wd = [1e-4 if i % 2 else 0.0 for i in range(len(w.numels))]
    run_parity(w, weight_decay=wd, fused=fused, tuning=dict(vec=vec))


def test_bf16_storage_vec4_k32():
    run_parity(W.small(K=32, numels=(2048, 12, 999), storage="bf16", m=3, T=6), tuning=dict(vec=4, avg_split=1))


# ---- configs[0] at full size: the oracle finishes in seconds -----------------------
def test_config0_flat_1m_k4_full():
    run_parity(W.config(0))
    run_parity(W.config(0), fused=False)


# ---- MobileNetV2-shaped list, reduced K: 158 tensors, many tiny ones ---------------
def test_mobilenet_list_k4():
    w = dataclasses.replace(W.config(3), K=4, T=3)
    run_parity(w)


# ---- protocol ------------------------------------------------------------------------
def test_illegal_call_orders_are_refused():
    import torch
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=2, numels=(300,))
    dev = DeviceReplicas(w)
    c = dev.ctx
    try:
        x0, grads = packed_inputs(w)
        dev.load_model(x0)
        dev.load_grads(grads(0))
        for call in (lambda: c.merge(True), lambda: c.step_merge(0.1, True), lambda: c.average(),
                     lambda: c.average_done(), lambda: c.init_master()):
            with pytest.raises(B.LasgdError) as e:
                call()
            assert e.value.status == B.ERR_STATE
        with pytest.raises(B.LasgdError) as e:
            c.local_step(float("nan"))
        assert e.value.status == B.ERR_INVALID
        before = dev.params(0).copy()
        c.local_step(0.1)
        c.snapshot()
        c.average()
        for call in (lambda: c.average(), lambda: c.snapshot()):
            with pytest.raises(B.LasgdError) as e:
                call()
            assert e.value.status == B.ERR_STATE
        c.sync()
        assert c.average_done()
        c.merge(False)
        with pytest.raises(B.LasgdError) as e:
            c.average()           # s was not refreshed by that merge
        assert e.value.status == B.ERR_STATE
        c.snapshot()
        c.average()
        c.step_merge(0.1, True)
        c.average()
        c.sync()
        # refused calls enqueued nothing: state equals the oracle's for the legal calls only
        from oracle import lasgd_oracle as O32
        o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, [w.weight_decay])
        o.set_model(x0)
        g = grads(0)
        o.local_step(g, 0.1); o.snapshot(); o.average(); o.merge(False); o.snapshot(); o.average()
        o.local_step(g, 0.1); o.merge(True); o.average()
        for k in range(w.K):
            assert_close(c.read_state(B.STATE_X, k), o.x[k], f"x[{k}]")
        assert_close(c.read_state(B.STATE_Z), o.z, "z")
        # argument errors of the probe
        for args in ((9, 0, -1), (B.STATE_V, 5, -1), (B.STATE_V, 0, 3)):
            with pytest.raises(B.LasgdError) as e:
                c.read_state(*args)
            assert e.value.status == B.ERR_INVALID
        with pytest.raises(B.LasgdError) as e:
            c.set_tuning(vec=3)
        assert e.value.status == B.ERR_INVALID
    finally:
        dev.close()


def test_unbound_and_misaligned():
    import torch
    c = B.Context(2, [64, 32], momentum=0.9, wd_scalar=0.0)
    try:
        x = torch.zeros(256, device="cuda")
        g = torch.zeros(256, device="cuda")
        with pytest.raises(B.LasgdError) as e:
            c.local_step(0.1)
        assert e.value.status == B.ERR_STATE
        with pytest.raises(B.LasgdError) as e:
            c.bind(0, [x.data_ptr() + 4, x.data_ptr() + 512], [g.data_ptr(), g.data_ptr() + 512])
        assert e.value.status == B.ERR_INVALID
        with pytest.raises(B.LasgdError) as e:
            c.bind(2, [x.data_ptr(), x.data_ptr() + 512], [g.data_ptr(), g.data_ptr() + 512])
        assert e.value.status == B.ERR_INVALID
        c.bind(0, [x.data_ptr(), x.data_ptr() + 512], [g.data_ptr(), g.data_ptr() + 512])
        with pytest.raises(B.LasgdError) as e:
            c.local_step(0.1)     # replica 1 still unbound
        assert e.value.status == B.ERR_STATE
    finally:
        c.close()


def test_overlap_is_race_free_under_load():
    """Local steps keep running on the main stream while the mean is computed
    on the side stream; many cycles back to back without host synchronisation
    must still equal the oracle (which has no concurrency at all)."""
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=8, numels=(1 << 20, 4096, 100), m=3, T=30)
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay] * len(w.numels)
    dev = DeviceReplicas(w, weight_decay=wd)
    try:
        g = grads(1)
        o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
        o.set_model(x0)
        dev.load_model(x0)
        dev.load_grads(g)
        o.prologue(g, w.lr)
        dev.prologue(w.lr)
        tau = 0
        for i in range(1, w.T + 1):          # same gradient buffer every step: no host sync inside the loop
            o.iteration(g, w.lr, w.m)
            tau = dev.iteration(w.lr, tau, w.m)
        for k in range(w.K):
            assert_close(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x[{k}] after {w.T} unsynchronised steps")
            assert_close(dev.ctx.read_state(B.STATE_S, k), o.s[k], f"s[{k}]")
        assert_close(dev.ctx.read_state(B.STATE_Z), o.z, "z")
    finally:
        dev.close()


def test_rebinding_gradient_buffers():
    """A caller may re-point a replica at other buffers (e.g. rotating gradient
    buffers); later steps must read the new ones."""
    import torch
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=2, numels=(1000, 36))
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay] * len(w.numels)
    dev = DeviceReplicas(w, weight_decay=wd)
    o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
    try:
        o.set_model(x0); dev.load_model(x0)
        g0, g1 = grads(0), grads(1)
        dev.load_grads(g0)
        o.local_step(g0, w.lr); dev.ctx.local_step(w.lr)
        alt = [torch.zeros_like(t) for t in dev.g]
        for k in range(w.K):
            alt[k][dev._idx] = torch.from_numpy(g1[k]).to(dev.dev)
            dev.ctx.bind(k, [dev.x[k].data_ptr() + int(off) * 4 for off in dev.off[:-1]],
                         [alt[k].data_ptr() + int(off) * 4 for off in dev.off[:-1]])
        torch.cuda.synchronize()
        o.local_step(g1, w.lr); dev.ctx.local_step(w.lr)
        for k in range(w.K):
            assert_close(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x[{k}] after rebinding")
    finally:
        dev.close()


@pytest.mark.parametrize("m", [1, 3])
def test_graph_replay_equals_eager(m):
    """A captured cycle replayed several times, with eager library work and host
    synchronisation between the replays, must give the oracle's state every time."""
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
        o.local_step(g, w.lr); o.snapshot()
        dev.ctx.local_step(w.lr); dev.ctx.snapshot()
        graph = dev.capture_cycle(w.lr, m)        # capturing does not execute
        # the mean was recorded, not launched: there is nothing this call could poll
        with pytest.raises(B.LasgdError) as e:
            dev.ctx.average_done()
        assert e.value.status == B.ERR_STATE

        def oracle_cycle():
            o.average()
            for _ in range(m):
                o.local_step(g, w.lr)
            o.merge(True)

        for rep in range(5):
            with torch.cuda.stream(dev.main):
                graph.replay()
            oracle_cycle()
            for k in range(w.K):
                assert_close(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x[{k}] after replay {rep}")
                assert_close(dev.ctx.read_state(B.STATE_V, k), o.v[k], f"v[{k}] after replay {rep}")
                assert_close(dev.ctx.read_state(B.STATE_S, k), o.s[k], f"s[{k}] after replay {rep}")
            assert_close(dev.ctx.read_state(B.STATE_Z), o.z, f"z after replay {rep}")
            if rep % 2 == 0:
                # an eager cycle in between, through the ordinary calls
                dev.ctx.average()
                for _ in range(m - 1):
                    dev.ctx.local_step(w.lr)
                dev.ctx.step_merge(w.lr, True)
                oracle_cycle()
                dev.ctx.sync()
                assert dev.ctx.average_done()        # an eager mean can be polled again
        # two replays back to back without host synchronisation
        with torch.cuda.stream(dev.main):
            graph.replay()
            graph.replay()
        oracle_cycle(); oracle_cycle()
        for k in range(w.K):
            assert_close(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x[{k}] after back-to-back replays")
        assert_close(dev.ctx.read_state(B.STATE_Z), o.z, "z after back-to-back replays")
    finally:
        dev.close()


def test_graph_survives_a_change_of_tile_size():
    """A cycle captured with 256-element tiles is replayed after the context has moved on to
    1024-element tiles (and back): the graph still points at a live tile table."""
    import torch
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=3, numels=(9000, 5, 1024, 4099), m=2)
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay] * len(w.numels)
    dev = DeviceReplicas(w, weight_decay=wd)
    o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
    try:
        g = grads(1)
        o.set_model(x0); dev.load_model(x0); dev.load_grads(g)
        o.local_step(g, w.lr); o.snapshot()
        dev.ctx.set_tuning(vec=1)
        dev.ctx.local_step(w.lr); dev.ctx.snapshot()
        graph = dev.capture_cycle(w.lr, w.m)

        def oracle_cycle():
            o.average()
            for _ in range(w.m):
                o.local_step(g, w.lr)
            o.merge(True)

        for vec in (4, 2, 1, 4):
            dev.ctx.set_tuning(vec=vec)
            with torch.cuda.stream(dev.main):
                graph.replay()                       # recorded with vec = 1
            oracle_cycle()
            dev.ctx.average()                        # and an eager cycle with the current tile size
            dev.ctx.local_step(w.lr)
            dev.ctx.step_merge(w.lr, True)
            oracle_cycle()
            for k in range(w.K):
                assert_close(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x[{k}] at vec {vec}")
                assert_close(dev.ctx.read_state(B.STATE_S, k), o.s[k], f"s[{k}] at vec {vec}")
            assert_close(dev.ctx.read_state(B.STATE_Z), o.z, f"z at vec {vec}")
    finally:
        dev.close()


def _same_special(got, ref, what):
    """Finite values and infinities bit for bit (+0 == -0 aside); NaN where the oracle has NaN
    (payload and sign of a generated NaN are the processor's business)."""
    gn, rn = np.isnan(got), np.isnan(ref)
    np.testing.assert_array_equal(gn, rn, err_msg=f"{what}: NaN positions")
    ok = ~rn
    same = (got.view(np.uint32)[ok] == ref.view(np.uint32)[ok]) | ((got[ok] == 0) & (ref[ok] == 0))
    assert same.all(), f"{what}: {int((~same).sum())} finite values differ"


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_denormals_zeros_infinities_and_nans_are_not_special_cased(storage):
    """No flushing, no clamping, no checks: denormal parameters and gradients keep their
    bits, NaN and Inf propagate exactly where the oracle's do."""
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=3, numels=(1024, 37), storage=storage, m=2, T=4)
    n = w.N
    rng = np.random.default_rng(11)
    x0 = (rng.standard_normal(n) * 0.01).astype(np.float32)
    x0[0:64] = (rng.standard_normal(64) * 1e-41).astype(np.float32)      # denormals
    x0[100:164] = (rng.standard_normal(64) * 1e-41).astype(np.float32)   # ... that meet denormal gradients
    x0[64:70] = [0.0, -0.0, 1e30, -1e30, 3e38, 1e-38]
    x0[70] = np.inf
    x0[71] = np.nan
    x0[1030] = -np.inf

    def grads(step):
        out = []
        for k in range(w.K):
            g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
            g[100:164] = (rng.standard_normal(64) * 1e-42).astype(np.float32)
            g[164] = np.nan if (step == 2 and k == 1) else 0.0
            g[165] = 3e38                                                  # overflows with momentum
            out.append(g)
        return [W.to_bf16_bits(g) for g in out] if storage == "bf16" else out

    if storage == "bf16":
        x0 = W.to_bf16_bits(x0)
    wd = [1e-4, 0.0]
    dev = DeviceReplicas(w, weight_decay=wd)
    o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd, storage=storage)
    try:
        o.set_model(x0); dev.load_model(x0)
        g = grads(0)
        dev.load_grads(g); o.prologue(g, w.lr); dev.prologue(w.lr)
        tau = 0
        for i in range(1, w.T + 1):
            g = grads(i)
            dev.load_grads(g)
            o.iteration(g, w.lr, w.m)
            tau = dev.iteration(w.lr, tau, w.m)
            for k in range(w.K):
                _same_special(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x step {i} replica {k}")
                _same_special(dev.ctx.read_state(B.STATE_V, k), o.v[k], f"v step {i} replica {k}")
                _same_special(dev.ctx.read_state(B.STATE_S, k), o.s[k], f"s step {i} replica {k}")
                if storage == "bf16":
                    got, ref = dev.params(k), o.x16[k]
                    nan = (ref & 0x7fff) > 0x7f80
                    np.testing.assert_array_equal(got[~nan], ref[~nan])
                    assert np.all((got[nan] & 0x7fff) > 0x7f80)
            _same_special(dev.ctx.read_state(B.STATE_Z), o.z, f"z step {i}")
        # the run did exercise what it claims to
        assert np.isnan(o.z).sum() >= 3 and np.isnan(o.x[1]).sum() >= 4
        if storage == "f32":
            for arr in (o.x[0][100:164], o.v[0][100:164], o.z[100:164]):
                assert np.all(np.abs(arr) < 1.2e-38) and np.any(arr != 0)
    finally:
        dev.close()


def test_two_hundred_steps_stay_bit_identical():
    """Rounding differences would random-walk over a long run; with the operation order pinned
    on both sides there are none to accumulate."""
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=4, numels=(6000, 130), m=3, T=200)
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay] * len(w.numels)
    dev = DeviceReplicas(w, weight_decay=wd)
    o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
    try:
        o.set_model(x0); dev.load_model(x0)
        g = grads(0)
        dev.load_grads(g); o.prologue(g, w.lr); dev.prologue(w.lr)
        tau = 0
        for i in range(1, w.T + 1):
            g = grads(i)
            dev.load_grads(g)
            o.iteration(g, w.lr, w.m)
            tau = dev.iteration(w.lr, tau, w.m)
            if i % 50 == 0:
                for k in range(w.K):
                    assert_close(dev.ctx.read_state(B.STATE_X, k), o.x[k], f"x step {i} replica {k}")
                    assert_close(dev.ctx.read_state(B.STATE_V, k), o.v[k], f"v step {i} replica {k}")
                assert_close(dev.ctx.read_state(B.STATE_Z), o.z, f"z step {i}")
    finally:
        dev.close()


def test_k64_masks_reach_the_top_bit():
    from oracle import lasgd_oracle as O32
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=64, numels=(300, 5))
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay] * len(w.numels)
    dev = DeviceReplicas(w, weight_decay=wd)
    o = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd)
    c = dev.ctx
    try:
        o.set_model(x0); dev.load_model(x0)
        g = grads(0)
        dev.load_grads(g)
        full = (1 << 64) - 1
        top = (1 << 63) | (1 << 62) | 1
        o.local_step(g, w.lr); c.local_step_ex(w.lr, full)
        o.snapshot(); c.snapshot_ex(full)
        o.average(mask=top); c.average_ex(top)
        o.local_step(g, 0.01, mask=top); c.local_step_ex(0.01, top)
        o.merge(True, mask=top); c.merge_ex(top, True)
        o.average(); c.average()
        for k in (0, 1, 62, 63):
            assert_close(c.read_state(B.STATE_X, k), o.x[k], f"x[{k}]")
            assert_close(c.read_state(B.STATE_S, k), o.s[k], f"s[{k}]")
        assert_close(c.read_state(B.STATE_Z), o.z, "z")
    finally:
        dev.close()


def test_allocation_failure_is_reported_not_fatal():
    """State that cannot fit the GPU (64 replicas of 2^31 - 2^21 parameters: 1.1 TB) is
    refused with ERR_ALLOC; the library keeps working afterwards."""
    with pytest.raises(B.LasgdError) as e:
        B.Context(64, [(1 << 31) - (1 << 21)], momentum=0.9)
    assert e.value.status == B.ERR_ALLOC, str(e.value)
    run_parity(W.small(K=2, numels=(300,), m=1, T=2))


def test_create_destroy_returns_all_device_memory():
    import torch

    def cycle(i):
        c = B.Context(4, [1 << 20, 1000, 7], momentum=0.9, storage=B.BF16 if i % 2 else B.F32)
        c.set_tuning(vec=1 + (i % 2))            # also replaces the tile table once
        c.close()

    cycle(0); cycle(1)                           # first use loads code objects and runtime pools
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for i in range(40):
        cycle(i)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert abs(free0 - free1) <= 8 << 20, (free0, free1)
