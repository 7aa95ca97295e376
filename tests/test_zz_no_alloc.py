"""The allocation-free entry point, lasgd_global_update_static, against the
context calls it is a variant of (lasgd_average + lasgd_merge) and against the
oracle: bit for bit, on two calls in a row that share the library's static
device buffer, the second on a smaller, ragged vector.  Device memory in use
must not change across either call."""
import numpy as np
import pytest
import torch

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W
from tests.parity_util import packed_inputs, say

pytestmark = pytest.mark.gpu


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def _one_call(K, n, resnapshot, seed):
    """Bring a context and the oracle to 'mean pending, one local step of progress',
    then take the global update three ways."""
    from paper_2203_13085_amd.driver import DeviceReplicas
    w = W.small(K=K, numels=(n,), m=2, T=1, seed=seed)
    x0, grads = packed_inputs(w)
    wd = [w.weight_decay]
    orc = O32.Oracle(K, [n], w.momentum, w.nesterov, wd)
    dev = DeviceReplicas(w, weight_decay=wd, side_stream=True)
    try:
        dev.ctx.set_tuning(avg_split=1)                  # the in-order mean: bit-exact z
        orc.set_model(x0)
        dev.load_model(x0)
        g = grads(0)
        orc.local_step(g, w.lr); orc.snapshot()
        dev.load_grads(g); dev.ctx.local_step(w.lr); dev.ctx.snapshot()
        g = grads(1)
        orc.local_step(g, w.lr)                          # progress while the All-Reduce is in flight
        dev.load_grads(g); dev.ctx.local_step(w.lr)
        dev.ctx.sync()
        # the static call works on copies of the same device state
        xs = [dev.x[k][:n].clone() for k in range(K)]
        ss = [torch.from_numpy(dev.ctx.read_state(B.STATE_S, k)).to(dev.dev) for k in range(K)]
        stream = torch.cuda.Stream(device=dev.dev)
        with torch.cuda.stream(stream):                  # a stream's first launch creates its hardware queue:
            torch.zeros(8, device=dev.dev).add_(1.0)     # keep that out of the measurement below
        torch.cuda.synchronize()
        free0, _ = torch.cuda.mem_get_info()
        say(f"[no-alloc] K={K} n={n} resnapshot={resnapshot}: calling lasgd_global_update_static")
        B.global_update_static([t.data_ptr() for t in xs], [t.data_ptr() for t in ss], n, resnapshot,
                               stream.cuda_stream)
        stream.synchronize()
        free1, _ = torch.cuda.mem_get_info()
        assert free1 == free0, f"device memory in use changed across the call: {free0} -> {free1}"
        # the existing entry points
        dev.ctx.average()
        dev.ctx.merge(resnapshot)
        dev.ctx.sync()
        orc.average()
        orc.merge(resnapshot=resnapshot)
        for k in range(K):
            got_x = xs[k].cpu().numpy()
            got_s = ss[k].cpu().numpy()
            np.testing.assert_array_equal(_bits(got_x), _bits(dev.params(k)), err_msg=f"x replica {k} vs context")
            np.testing.assert_array_equal(_bits(got_s), _bits(dev.ctx.read_state(B.STATE_S, k)),
                                          err_msg=f"sent replica {k} vs context")
            np.testing.assert_array_equal(_bits(got_x), _bits(orc.x[k]), err_msg=f"x replica {k} vs oracle")
            np.testing.assert_array_equal(_bits(got_s), _bits(orc.s[k]), err_msg=f"sent replica {k} vs oracle")
    finally:
        dev.close()
        del dev
        torch.cuda.empty_cache()


def test_static_global_update_two_calls_second_smaller():
    _one_call(K=8, n=1_000_003, resnapshot=True, seed=21)
    _one_call(K=3, n=4_098, resnapshot=False, seed=22)       # smaller; stale z beyond n must not matter


def test_static_global_update_at_the_maximum_size():
    """n = LASGD_STATIC_MAX_N exactly (the whole static buffer), K = 2, inputs drawn on the device."""
    n, K = B.STATIC_MAX_N, 2
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(3)
    xs = [torch.randn(n, generator=gen, device="cuda:0") * 0.01 for _ in range(K)]
    ss = [x + torch.randn(n, generator=gen, device="cuda:0") * 1e-3 for x in xs]
    hx = [t.cpu().numpy() for t in xs]
    hs = [t.cpu().numpy() for t in ss]
    say(f"[no-alloc] K={K} n={n} (maximum)")
    B.global_update_static([t.data_ptr() for t in xs], [t.data_ptr() for t in ss], n, True)
    torch.cuda.synchronize()
    orc = O32.Oracle(K, [n], 0.9, True, [0.0], threads=2)
    for k in range(K):
        orc.x[k][:] = hx[k]
        orc.s[k][:] = hs[k]
    orc.average()
    orc.merge(resnapshot=True)
    for k in range(K):
        np.testing.assert_array_equal(_bits(xs[k].cpu().numpy()), _bits(orc.x[k]), err_msg=f"x replica {k}")
        np.testing.assert_array_equal(_bits(ss[k].cpu().numpy()), _bits(orc.s[k]), err_msg=f"sent replica {k}")
    del xs, ss
    torch.cuda.empty_cache()


def test_static_global_update_refuses_bad_arguments():
    t = torch.zeros(64, device="cuda:0")
    u = torch.zeros(64, device="cuda:0")
    with pytest.raises(B.LasgdError) as e:
        B.global_update_static([t.data_ptr()], [u.data_ptr()], B.STATIC_MAX_N + 1)
    assert e.value.status == B.ERR_UNSUPPORTED and "LASGD_STATIC_MAX_N" in str(e.value)
    with pytest.raises(B.LasgdError) as e:
        B.global_update_static([t.data_ptr() + 4], [u.data_ptr()], 8)
    assert e.value.status == B.ERR_INVALID
    with pytest.raises(B.LasgdError) as e:
        B.global_update_static([t.data_ptr(), t.data_ptr()], [u.data_ptr(), u.data_ptr() + 128], 8)
    assert e.value.status == B.ERR_INVALID
    with pytest.raises(B.LasgdError) as e:
        B.global_update_static([t.data_ptr()], [u.data_ptr()], 0)
    assert e.value.status == B.ERR_INVALID
    torch.cuda.synchronize()
    assert float(t.abs().sum()) == 0.0 and float(u.abs().sum()) == 0.0
