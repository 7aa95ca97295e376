"""GPU parity of the extended entry points (replicas at their own pace, partial
All-Reduce, elastic alpha/beta, SGD-AR) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import lasgd_oracle as O32
from paper_2203_13085_amd import binding as B
from paper_2203_13085_amd import workloads as W
from tests.parity_util import assert_close, compare_state, packed_inputs, say

pytestmark = pytest.mark.gpu


def _pair(w, wd=None):
    from paper_2203_13085_amd.driver import DeviceReplicas
    wd = list(wd) if wd is not None else [w.weight_decay] * len(w.numels)
    x0, grads = packed_inputs(w)
    orc = O32.Oracle(w.K, w.numels, w.momentum, w.nesterov, wd, storage=w.storage)
    dev = DeviceReplicas(w, weight_decay=wd)
    orc.set_model(x0)
    dev.load_model(x0)
    return orc, dev, grads


def _tau5_counts(rng, K, tau_max=5):
    """Local steps per All-Reduce drawn from the shape of the paper's histogram
    (communication-intensive experiment: 11.2 / 72.8 / 11.1 / 0.2 / 0.6 / 3.9 %
    of All-Reduces took 1 / 2 / 3 / 4 / 5 / 6+ gradient computations), capped
    at tau_max, with per-replica jitter: some nodes are up to twice as slow
    (Sec. 2), so a node may take fewer steps than the fastest one."""
    p = np.array([11.2, 72.8, 11.1, 0.2, 0.6, 3.9])
    base = min(int(rng.choice(6, p=p / p.sum())) + 1, tau_max)
    return [max(1, int(round(base * rng.uniform(0.5, 1.0)))) if rng.random() < 0.4 else base for _ in range(K)]


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_adaptive_cadence_scripted_from_the_papers_histogram(storage):
    w = W.small(K=6, numels=(3000, 7, 513, 256, 1025), storage=storage)
    rng = np.random.default_rng(5)
    rounds = [_tau5_counts(rng, w.K) for _ in range(8)] + [[1, 5, 2, 3, 1, 4]]
    lr = lambda k, c: float(np.float32(0.05 / (1 + 0.1 * c)))      # eta indexed by the node's own clock
    orc, dev, grads = _pair(w)
    c = dev.ctx
    full = (1 << w.K) - 1
    try:
        say(f"[dyn] rounds = {rounds}")
        rec = {}
        O32.run_dynamic(orc, orc.x16[0].copy() if storage == "bf16" else orc.x[0].copy(), grads, lr, rounds,
                        after=lambda t, o: rec.__setitem__(t, ([a.copy() for a in o.x], [a.copy() for a in o.v],
                                                               [a.copy() for a in o.s], o.z.copy(),
                                                               [a.copy() for a in o.x16] if o.x16 else None)))
        # device: same script; the last tick of a round is the fused step + global update
        clock = [0] * w.K
        tick = 0
        dev.load_grads(grads(0))
        c.local_step_ex([lr(k, 0) for k in range(w.K)], full)
        clock = [1] * w.K
        c.snapshot(); c.average()

        def check(t):
            x, v, s, z, x16 = rec[t]
            for k in range(w.K):
                assert_close(c.read_state(B.STATE_X, k), x[k], f"x tick {t} replica {k}")
                assert_close(c.read_state(B.STATE_V, k), v[k], f"v tick {t} replica {k}")
                assert_close(c.read_state(B.STATE_S, k), s[k], f"s tick {t} replica {k}")
                if x16 is not None:
                    np.testing.assert_array_equal(dev.params(k), x16[k])
            assert_close(c.read_state(B.STATE_Z), z, f"z tick {t}")
        check(0)
        for counts in rounds:
            for j in range(max(counts)):
                tick += 1
                dev.load_grads(grads(tick))
                mask = sum(1 << k for k in range(w.K) if counts[k] > j)
                lrs = [lr(k, clock[k]) for k in range(w.K)]
                if j == max(counts) - 1:
                    assert c.average_done() in (True, False)
                    c.step_merge_ex(lrs, mask, full, True)
                    c.average()
                else:
                    c.local_step_ex(lrs, mask)
                for k in range(w.K):
                    if counts[k] > j:
                        clock[k] += 1
                check(tick)
    finally:
        dev.close()


def test_partial_all_reduce():
    """Each round only some replicas take part in the All-Reduce; the others
    keep stepping and join later (Sec. 6).  Participants merge at different
    ticks, in two groups."""
    w = W.small(K=5, numels=(2000, 5, 700))
    orc, dev, grads = _pair(w)
    c = dev.ctx
    K, full = w.K, (1 << w.K) - 1
    rounds = [0b11111, 0b01011, 0b10110, 0b00001, 0b11101, 0b11111]
    try:
        g = grads(0)
        dev.load_grads(g)
        orc.local_step(g, w.lr); c.local_step(w.lr)
        orc.snapshot(); c.snapshot()
        tick = 0
        for r, part in enumerate(rounds):
            orc.average(mask=part); c.average_ex(part)
            members = [k for k in range(K) if (part >> k) & 1]
            first = sum(1 << k for k in members[: (len(members) + 1) // 2])
            second = part & ~first
            for j in range(2):
                tick += 1
                g = grads(tick)
                dev.load_grads(g)
                if j == 0:
                    # everyone steps; the first group merges in the same pass
                    orc.local_step(g, w.lr); orc.merge(True, mask=first)
                    c.step_merge_ex(w.lr, full, first, True)
                else:
                    orc.local_step(g, w.lr)
                    c.local_step_ex(w.lr, full)
                    if second:
                        orc.merge(True, mask=second); c.merge_ex(second, True)
            nxt = rounds[r + 1] if r + 1 < len(rounds) else 0
            late = nxt & ~part                      # replicas that sat this round out send before joining
            if late:
                orc.snapshot(mask=late); c.snapshot_ex(late)
            compare_state(dev, orc, tick)
    finally:
        dev.close()


@pytest.mark.parametrize("alpha,beta", [(0.5, 0.75), (1.0, 0.5), (0.25, 1.0), (0.0, 0.0)])
@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_elastic_coefficients(alpha, beta, storage):
    w = W.small(K=4, storage=storage, m=2, T=6)
    orc, dev, grads = _pair(w)
    c = dev.ctx
    try:
        c.set_elastic(alpha, beta)
        g = grads(0)
        dev.load_grads(g)
        orc.local_step(g, w.lr); c.local_step(w.lr)
        orc.snapshot(); c.snapshot()
        orc.average(beta=beta); c.average()
        compare_state(dev, orc, 0)
        tau = 0
        for i in range(1, w.T + 1):
            g = grads(i)
            dev.load_grads(g)
            tau += 1
            orc.local_step(g, w.lr)
            if tau == w.m:
                orc.merge(True, alpha=alpha); orc.average(beta=beta)
                if i % 4 == 0:
                    c.local_step(w.lr); c.merge(True)
                else:
                    c.step_merge(w.lr, True)
                c.average()
                tau = 0
            else:
                c.local_step(w.lr)
            compare_state(dev, orc, i)
    finally:
        dev.close()


@pytest.mark.parametrize("storage,K,vec", [("f32", 4, 1), ("f32", 7, 2), ("bf16", 16, 1), ("f32", 1, 4)])
def test_sgd_ar_step(storage, K, vec):
    w = W.small(K=K, numels=(3000, 7, 513, 256, 1025), storage=storage)
    orc, dev, grads = _pair(w, wd=[1e-3, 0.0, 1e-2, 1e-4, 0.0])
    try:
        dev.ctx.set_tuning(vec=vec)
        for i in range(5):
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


def test_mask_order_rules():
    w = W.small(K=4, numels=(300,))
    orc, dev, grads = _pair(w)
    c = dev.ctx
    try:
        dev.load_grads(grads(0))
        c.local_step(0.1)

        def refused(call, status=B.ERR_STATE):
            with pytest.raises(B.LasgdError) as e:
                call()
            assert e.value.status == status

        refused(lambda: c.average_ex(0b0011))                 # nobody has sent yet
        refused(lambda: c.snapshot_ex(0), B.ERR_INVALID)
        refused(lambda: c.snapshot_ex(1 << 4), B.ERR_INVALID)  # beyond K
        refused(lambda: c.local_step_ex([0.1, float("inf"), 0.1, 0.1], 0b0010), B.ERR_INVALID)
        c.local_step_ex([0.1, float("inf"), 0.1, 0.1], 0b0101)  # entries of idle replicas are not read
        c.local_step_ex([0.1] * 4, 0)                          # nobody steps: accepted, nothing happens
        c.snapshot_ex(0b0011)
        refused(lambda: c.average_ex(0b0111))                 # replica 2 has not sent
        c.average_ex(0b0011)
        refused(lambda: c.snapshot_ex(0b0001))                # its s may still be read
        c.snapshot_ex(0b1100)                                 # bystanders may send meanwhile
        refused(lambda: c.average_ex(0b1100))                 # z still owed to replicas 0, 1
        refused(lambda: c.merge_ex(0b0100, True))             # not a participant
        c.merge_ex(0b0001, True)
        refused(lambda: c.merge_ex(0b0001, True))             # merged already
        refused(lambda: c.average_ex(0b1100))                 # replica 1 has not merged yet
        c.step_merge_ex([0.1] * 4, 0b1111, 0b0010, False)
        refused(lambda: c.average_ex(0b0010))                 # that merge did not re-send
        c.average_ex(0b1101)
        c.merge_ex(0b1101, True)
        refused(lambda: c.set_elastic(1.5, 0.5), B.ERR_INVALID)
        refused(lambda: c.set_elastic(float("nan"), 0.5), B.ERR_INVALID)
        c.sync()
    finally:
        dev.close()


@pytest.mark.parametrize("tau_max", [1, 3, 5])
@pytest.mark.parametrize("fused_mean", [False, True])
def test_live_polling_replayed_through_the_oracle(tau_max, fused_mean):
    """The real adaptive rule: poll "All Reduce done" on the device, cap at
    tau_max.  Which iterations fire depends on timing, so the decisions are
    recorded and replayed through the oracle; whatever they were, the states
    must agree, and no replica may take more than tau_max steps per All-Reduce."""
    w = W.small(K=8, numels=(1 << 18, 4096, 100), T=24)
    orc, dev, grads = _pair(w)
    try:
        g = grads(1)
        dev.load_grads(g)              # one gradient set for every step: no host sync inside the loop
        orc.prologue(g, w.lr)
        dev.prologue(w.lr)
        tau, fired_at, since = 0, [], 0
        for i in range(1, w.T + 1):
            tau, fired = dev.adaptive_iteration(w.lr, tau, tau_max, fused_mean=fused_mean)
            since += 1
            if fired:
                fired_at.append(i)
                assert since <= tau_max
                since = 0
        say(f"[live] tau_max={tau_max} fused_mean={fused_mean}: global updates fired at iterations {fired_at}")
        if tau_max == 1:
            assert fired_at == list(range(1, w.T + 1))
        for i in range(1, w.T + 1):
            orc.local_step(g, w.lr)
            if i in fired_at:
                orc.merge(True)
                orc.average()
        compare_state(dev, orc, w.T)
    finally:
        dev.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_legal_call_sequences(seed):
    """Randomly drawn, legal sequences of the extended calls (masked steps with
    per-replica step sizes, partial means, staggered partial merges with and
    without re-sending, late snapshots, elastic coefficients, the fused
    step + global update + next mean where it is legal): device and oracle
    must agree after every call group."""
    r = np.random.default_rng(500 + seed)
    K = int(r.integers(1, 9))
    storage = "bf16" if seed % 3 == 2 else "f32"
    numels = tuple(int(n) for n in r.choice([1, 3, 64, 255, 256, 257, 1000, 2049], size=int(r.integers(1, 5))))
    w = W.small(K=K, numels=numels, storage=storage, momentum=float(r.choice([0.0, 0.9])),
                nesterov=bool(r.integers(0, 2)))
    if w.momentum == 0.0:
        w = __import__("dataclasses").replace(w, nesterov=False)
    alpha = float(np.float32(r.choice([1.0, 1.0, 0.5])))
    beta = float(np.float32(r.choice([1.0, 1.0, 0.25])))
    orc, dev, grads = _pair(w, wd=[float(np.float32(x)) for x in r.choice([0.0, 1e-3], size=len(numels))])
    c = dev.ctx
    full = (1 << K) - 1
    say(f"[fuzz] seed={seed} K={K} numels={numels} storage={storage} alpha={alpha} beta={beta}")
    try:
        c.set_elastic(alpha, beta)
        pending = sent = 0
        for step in range(12):
            g = grads(step)
            dev.load_grads(g)
            lrs = [float(np.float32(v)) for v in r.uniform(0.01, 0.2, size=K)]
            mask = int(r.integers(0, full + 1))
            part = 0
            if pending == full and alpha == 1.0 and beta == 1.0 and r.random() < 0.35:
                # everybody steps, merges, re-sends and the next mean is taken in the same pass
                orc.local_step(g, lrs[0]); orc.merge(True); orc.average()
                c.step_merge_average(lrs[0])
                sent = full
                compare_state(dev, orc, step, z_exact=False)
                continue
            if pending and r.random() < 0.6:
                part = (int(r.integers(1, pending + 1)) & pending) or pending
                resnap = bool(r.integers(0, 2))
            if part and r.random() < 0.5:
                orc.local_step(g, lrs, mask=mask); orc.merge(resnap, mask=part, alpha=alpha)
                c.step_merge_ex(lrs, mask, part, resnap)
            else:
                orc.local_step(g, lrs, mask=mask); c.local_step_ex(lrs, mask)
                if part:
                    orc.merge(resnap, mask=part, alpha=alpha); c.merge_ex(part, resnap)
            if part:
                pending &= ~part
                sent = (sent | part) if resnap else (sent & ~part)
            if not pending:
                late = full & ~sent
                if late and r.random() < 0.7:
                    orc.snapshot(mask=late); c.snapshot_ex(late)
                    sent |= late
                if sent and r.random() < 0.8:
                    p2 = (int(r.integers(1, full + 1)) & sent) or sent
                    orc.average(mask=p2, beta=beta); c.average_ex(p2)
                    pending = p2
            compare_state(dev, orc, step, z_exact=False)
    finally:
        dev.close()
