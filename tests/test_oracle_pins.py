"""Pins for the CPU oracles: what the paper and the mathematics fix.

Each check takes a factory `make(K, numels, mu, nesterov, wd)` and is applied
to (a) the fp32 C oracle, (b) the fp64 numpy reference and (c) a set of
deliberately wrong variants of the reference, each of which has to be caught
by at least one check.  No expected value here comes from a GPU.

    P1  K = 1: the global update leaves the local model unchanged
    P2  no local progress: the global update returns the mean
    P3  the global update preserves the replica mean; the mean of equal models is that model
    P4  exact-rational brute force of Algorithm 1 on tiny vectors, and the closed
        form "average model plus the local gradient steps taken meanwhile" (Sec. 4)
    P5  cadence 1, plain SGD: Sec. 3 Eq. 7-8
    P6  identical gradients everywhere: the run is single-model momentum SGD (torch.optim.SGD)
    P7  the replica mean follows large-batch momentum SGD on the mean gradient
    P8  after a global update, deviations from the mean equal deviations of local progress
    P9  bf16 rounding equals torch's conversion
    P10 the mean equals the exactly rounded sum (math.fsum) divided by K
    hand-worked values from tests/golden/alg1_hand_worked.json
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import lasgd_oracle as O32
from oracle import lasgd_ref64 as O64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- adapters
def make32(K, numels, mu, nesterov, wd):
    return O32.Oracle(K, numels, mu, nesterov, wd)


def make64(K, numels, mu, nesterov, wd):
    return O64.Ref64(K, numels, mu, nesterov, wd)


def X(o):
    return np.stack([np.asarray(a, dtype=np.float64) for a in o.x])


def V(o):
    return np.stack([np.asarray(a, dtype=np.float64) for a in o.v])


def S(o):
    return np.stack([np.asarray(a, dtype=np.float64) for a in o.s])


def Z(o):
    return np.asarray(o.z, dtype=np.float64)


def put(o, name, k, values):
    """Write one replica's state array, whatever the container type."""
    arr = getattr(o, name)
    arr[k][:] = values


def is32(o):
    return isinstance(o, O32.Oracle)


def tol(o, steps=1):
    """(rtol, atol) for comparing an implementation with exact mathematics."""
    if is32(o):
        return 2e-6 * max(1, steps) ** 0.5, 2e-7 * max(1, steps) ** 0.5
    return 1e-11, 1e-13


def close(o, a, b, steps=1, what=""):
    r, t = tol(o, steps)
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    bad = np.abs(a - b) > t + r * np.abs(b)
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} differ, max |d|={np.abs(a - b).max():.3e}"


def draws(seed, K, N, scale=1.0):
    """fp32-representable random values, so both precisions see equal inputs."""
    r = np.random.default_rng(seed)
    return (r.standard_normal((K, N)) * scale).astype(np.float32)


def run(o, x0, g, lr, m, T, after=None):
    """Algorithm 1 on either implementation; g[step][k] is a flat gradient."""
    mod = O32 if is32(o) else O64
    return mod.run_schedule(o, x0, lambda i: [g[i][k] for k in range(o.K)], lr, m, T, after)


# ------------------------------------------------------------------- checks
def check_p1_k1_identity(make):
    N = 257
    o = make(1, [N], 0.9, True, [1e-4])
    x0 = draws(1, 1, N, 0.05)[0]
    g = draws(2, 12, N, 1e-3)[:, None, :]
    def after(i, o):
        # with one replica the mean is the sent model itself
        close(o, Z(o), S(o)[0], what="K=1 mean")
    run(o, x0, g, 0.1, 3, 9, after)
    # one more local step, then merge must not move x
    o.local_step([g[10][0]], 0.1)
    before, sent = X(o).copy(), S(o)[0].copy()
    o.merge(True)
    close(o, X(o), before, what="K=1 merge identity")
    if is32(o):
        # x - s is exact whenever s/2 <= x <= 2s (Sterbenz), then z + (x - s) = x bit for bit
        xs, ss = before[0], sent
        st = (np.sign(xs) == np.sign(ss)) & (np.abs(xs) <= 2 * np.abs(ss)) & (np.abs(ss) <= 2 * np.abs(xs))
        assert st.sum() > N // 2
        np.testing.assert_array_equal(X(o)[0][st], before[0][st])


def check_p2_zero_progress(make):
    K, N = 4, 130
    o = make(K, [N], 0.9, True, [0.0])
    xs = draws(3, K, N, 0.1)
    for k in range(K):
        put(o, "x", k, xs[k])
    o.snapshot()
    o.average()
    zexp = xs.astype(np.float64).mean(axis=0)
    close(o, Z(o), zexp, what="mean")
    o.merge(True)
    # x == s, so x - s = 0 exactly and the result is z itself, in any precision
    for k in range(K):
        np.testing.assert_array_equal(X(o)[k], Z(o))
        np.testing.assert_array_equal(S(o)[k], Z(o))


def check_p3_mean_preserved(make):
    K, N = 5, 96
    o = make(K, [N], 0.0, False, [0.0])
    same = draws(4, 1, N, 0.3)[0]
    for k in range(K):
        put(o, "x", k, same)
    o.snapshot()
    o.average()
    close(o, Z(o), same, what="mean of identical replicas")
    if is32(o):
        np.testing.assert_array_equal(Z(o).astype(np.float32), same)
    xs, ss = draws(5, K, N, 0.2), draws(6, K, N, 0.2)
    for k in range(K):
        put(o, "x", k, ss[k])
    o.snapshot()
    for k in range(K):
        put(o, "x", k, xs[k])
    o.average()          # the All-Reduce sees the sent models, not the ones still moving
    close(o, Z(o), ss.astype(np.float64).mean(axis=0), what="mean is over the sent models")
    o.merge(False)
    close(o, X(o).mean(axis=0), xs.astype(np.float64).mean(axis=0), what="replica mean across merge")
    # without re-snapshot the sent models are untouched
    np.testing.assert_array_equal(S(o), ss.astype(np.float64))


def _alg1_rational(x0, g, lr, mu, wd, nesterov, m, T):
    """Algorithm 1 in exact rational arithmetic, one scalar parameter per
    replica-element, straight from the definitions.  Returns per-step
    (x, v, s, z) lists of Fractions."""
    K, N = len(g[0]), len(x0)
    F = Fraction
    lr, mu = F(lr), F(mu)
    x = [[F(float(a)) for a in x0] for _ in range(K)]
    v = [[F(0)] * N for _ in range(K)]
    s = [[F(0)] * N for _ in range(K)]
    z = [F(0)] * N
    hist = []

    def step(i):
        for k in range(K):
            for e in range(N):
                gg = F(float(g[i][k][e])) + F(wd[e]) * x[k][e]
                v[k][e] = mu * v[k][e] + gg
                d = gg + mu * v[k][e] if nesterov else v[k][e]
                x[k][e] = x[k][e] - lr * d

    def send():
        for k in range(K):
            s[k] = list(x[k])
        for e in range(N):
            z[e] = sum(s[k][e] for k in range(K)) / K

    step(0)
    send()
    hist.append(([list(r) for r in x], [list(r) for r in v], [list(r) for r in s], list(z)))
    tau = 0
    for i in range(1, T + 1):
        step(i)
        tau += 1
        if tau == m:
            for k in range(K):
                for e in range(N):
                    x[k][e] = z[e] + (x[k][e] - s[k][e])
            send()
            tau = 0
        hist.append(([list(r) for r in x], [list(r) for r in v], [list(r) for r in s], list(z)))
    return hist


def _fr(a):
    return np.array([[float(c) for c in row] for row in a]) if isinstance(a[0], list) else np.array([float(c) for c in a])


def check_p4_bruteforce(make):
    for (K, numels, mu, nes, wdt, m, T, lr) in (
            (3, [2, 3], 0.5, True, [0.25, 0.0], 2, 6, 0.125),
            (4, [8], 0.9, False, [1e-2], 3, 6, 0.1),
            (2, [1, 1, 2], 0.0, False, [0.0, 0.5, 0.0], 1, 4, 0.3),
            (3, [4], 0.75, True, [0.1], 4, 6, 0.05)):
        N = sum(numels)
        wd_e = np.repeat(np.asarray(wdt, dtype=np.float32).astype(np.float64), numels)
        lr32, mu32 = float(np.float32(lr)), float(np.float32(mu))
        o = make(K, numels, mu32, nes, [float(np.float32(w)) for w in wdt])
        x0 = draws(10 + K, 1, N, 0.5)[0]
        g = draws(20 + K, (T + 1) * K, N, 0.1).reshape(T + 1, K, N)
        hist = _alg1_rational(x0, g, lr32, mu32, wd_e, nes, m, T)

        def after(i, o):
            hx, hv, hs, hz = hist[i]
            close(o, X(o), _fr(hx), steps=i + 1, what=f"x step {i}")
            close(o, V(o), _fr(hv), steps=i + 1, what=f"v step {i}")
            close(o, S(o), _fr(hs), steps=i + 1, what=f"s step {i}")
            close(o, Z(o), _fr(hz), steps=i + 1, what=f"z step {i}")
        run(o, x0, g, lr32, m, T, after)


def check_p4_closed_form(make):
    """Plain SGD: after a global update the model is the mean of the sent
    models minus eta times the gradients applied while the All-Reduce ran."""
    K, N, m, T, lr = 4, 33, 3, 9, 0.25
    o = make(K, [N], 0.0, False, [0.0])
    x0 = draws(30, 1, N, 0.5)[0]
    g = draws(31, (T + 1) * K, N, 0.1).reshape(T + 1, K, N).astype(np.float32)
    g64 = g.astype(np.float64)
    seen = {}

    def after(i, o):
        seen[i] = (X(o).copy(), S(o).copy(), Z(o).copy())
    run(o, x0, g, lr, m, T, after)
    # prologue: sent model = x0 - lr*g0; z = its mean
    sent = x0.astype(np.float64)[None, :] - lr * g64[0]
    close(o, seen[0][1], sent, what="sent model after prologue")
    z = sent.mean(axis=0)
    close(o, seen[0][2], z, what="first mean")
    for cyc in range(T // m):
        steps = range(cyc * m + 1, (cyc + 1) * m + 1)
        expect = z[None, :] - lr * sum(g64[i] for i in steps)
        got = seen[(cyc + 1) * m][0]
        close(o, got, expect, steps=(cyc + 1) * m, what=f"closed form, cycle {cyc}")
        z = expect.mean(axis=0)           # what was sent is what was merged
        close(o, seen[(cyc + 1) * m][2], z, steps=(cyc + 1) * m, what="next mean")


def check_p5_alpha_beta_one(make):
    """Cadence 1 and plain SGD: x_{t+1}^i = z_t - eta g_t^i, z_t = mean_i x_t^i."""
    K, N, T, lr = 3, 40, 6, 0.5
    o = make(K, [N], 0.0, False, [0.0])
    x0 = draws(40, 1, N, 1.0)[0]
    g = draws(41, (T + 1) * K, N, 0.2).reshape(T + 1, K, N)
    g64 = g.astype(np.float64)
    xt = x0.astype(np.float64)[None, :] - lr * g64[0]      # x_1^i (all start equal: z_0 = x0)
    rec = {}
    run(o, x0, g, lr, 1, T, lambda i, o: rec.__setitem__(i, (X(o).copy(), Z(o).copy())))
    close(o, rec[0][0], xt, what="x_1")
    for t in range(1, T + 1):
        z = xt.mean(axis=0)
        xt = z[None, :] - lr * g64[t]
        close(o, rec[t][0], xt, steps=t + 1, what=f"Eq.7 at t={t}")
        close(o, rec[t][1], xt.mean(axis=0), steps=t + 1, what=f"Eq.8 at t={t}")


def _torch_sgd(x0, grads, lr, mu, wd, nesterov, dtype):
    p = torch.nn.Parameter(torch.tensor(np.asarray(x0), dtype=dtype))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd, nesterov=nesterov, dampening=0.0)
    out = []
    for g in grads:
        p.grad = torch.tensor(np.asarray(g), dtype=dtype)
        opt.step()
        out.append(p.detach().to(torch.float64).numpy().copy())
    return out


def check_p6_identical_gradients(make):
    for nes, mu, wd in ((True, 0.9, 1e-2), (False, 0.8, 0.0), (False, 0.0, 0.05)):
        K, N, m, T, lr = 3, 50, 2, 8, 0.1
        o = make(K, [N], mu, nes, [wd])
        x0 = draws(50, 1, N, 0.5)[0]
        gs = draws(51, T + 1, N, 0.1)
        g = np.repeat(gs[:, None, :], K, axis=1)
        # torch needs momentum > 0 for nesterov; mu = 0 is run without it
        ref = _torch_sgd(x0, gs, float(np.float32(lr)) if is32(o) else lr, mu, wd, nes and mu > 0,
                         torch.float32 if is32(o) else torch.float64)

        def after(i, o):
            for k in range(K):
                close(o, X(o)[k], ref[i], steps=4 * (i + 1), what=f"torch SGD step {i} replica {k}")
        run(o, x0, g, lr, m, T, after)


def check_p7_mean_is_large_batch_sgd(make):
    K, N, T, lr, mu, wd = 4, 64, 30, 0.05, 0.9, 1e-3
    x0 = draws(60, 1, N, 0.5)[0]
    g = draws(61, (T + 1) * K, N, 0.1).reshape(T + 1, K, N)
    gbar = g.astype(np.float64).mean(axis=1)
    ref = _torch_sgd(x0, gbar, lr, mu, wd, True, torch.float64)
    for m in (1, 3, 5):
        o = make(K, [N], mu, True, [wd])

        def after(i, o):
            close(o, X(o).mean(axis=0), ref[i], steps=8 * (i + 1), what=f"mean trajectory m={m} step {i}")
        run(o, x0, g, lr, m, T, after)


def check_p8_deviation(make):
    K, N = 4, 77
    o = make(K, [N], 0.9, True, [1e-3])
    x0 = draws(70, 1, N, 0.5)[0]
    g = draws(71, 4 * K, N, 0.1).reshape(4, K, N)
    o.set_model(x0)
    o.prologue([g[0][k] for k in range(K)], 0.1)
    o.local_step([g[1][k] for k in range(K)], 0.1)
    o.local_step([g[2][k] for k in range(K)], 0.1)
    prog = X(o) - S(o)
    zt = Z(o).copy()
    o.merge(True)
    x1 = X(o)
    close(o, x1 - x1.mean(axis=0), prog - prog.mean(axis=0), steps=4, what="deviation = deviation of progress")
    close(o, x1, zt[None, :] + prog, steps=4, what="x = z + progress")
    # momentum is local state: the global update must not touch it
    vb = V(o).copy()
    o.local_step([g[3][k] for k in range(K)], 0.0)      # lr = 0: x frozen, v advances
    assert not np.array_equal(V(o), vb)


def check_momentum_untouched_by_merge(make):
    K, N = 3, 20
    o = make(K, [N], 0.9, True, [0.0])
    x0 = draws(80, 1, N, 0.5)[0]
    g = draws(81, 2 * K, N, 0.1).reshape(2, K, N)
    o.set_model(x0)
    o.prologue([g[0][k] for k in range(K)], 0.1)
    o.local_step([g[1][k] for k in range(K)], 0.1)
    vb = V(o).copy()
    o.merge(True)
    o.average()
    np.testing.assert_array_equal(V(o), vb)


def check_hand_worked(make):
    with open(os.path.join(GOLDEN, "alg1_hand_worked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        K, N = c["K"], c["N"]
        o = make(K, [N], c["mu"], c["nesterov"], [c["wd"]])
        g = np.asarray(c["g"], dtype=np.float32)                 # [T+1][K][N]
        rec = {}
        run(o, np.asarray(c["x0"], dtype=np.float32), g, c["lr"], c["m"], c["T"],
            lambda i, o: rec.__setitem__(i, (X(o).copy(), V(o).copy(), S(o).copy(), Z(o).copy())))
        for step, exp in c["expect"].items():
            x, v, s, z = rec[int(step)]
            for name, got in (("x", x), ("v", v), ("s", s), ("z", z)):
                if name in exp:
                    # all values are small dyadic rationals: exact in fp32 and fp64
                    np.testing.assert_array_equal(got, np.asarray(exp[name], dtype=np.float64),
                                                  err_msg=f"{c['name']} step {step} {name}")


CHECKS = [check_p1_k1_identity, check_p2_zero_progress, check_p3_mean_preserved,
          check_p4_bruteforce, check_p4_closed_form, check_p5_alpha_beta_one,
          check_p6_identical_gradients, check_p7_mean_is_large_batch_sgd,
          check_p8_deviation, check_momentum_untouched_by_merge, check_hand_worked]


@pytest.mark.parametrize("check", CHECKS, ids=lambda f: f.__name__)
@pytest.mark.parametrize("make", [make32, make64], ids=["c_fp32", "numpy_fp64"])
def test_pin(make, check):
    check(make)


# -------------------------------------------------- planted mistakes (CPU)
def _mutant(name):
    """A wrong variant of the reference; each plants one plausible slip."""
    class M(O64.Ref64):
        def local_step(self, grads, lr):
            g = np.stack([np.asarray(a, dtype=np.float64) for a in grads])
            g1 = g + self.wd[None, :] * self.x
            if name == "wd_dropped":
                g1 = g
            if name == "wd_sign":
                g1 = g - self.wd[None, :] * self.x
            vold = self.v
            if name == "dampening":
                self.v = self.mu * self.v + (1 - self.mu) * g1
            elif name == "v_from_raw_g":
                self.v = self.mu * self.v + g
            else:
                self.v = self.mu * self.v + g1
            if name == "nesterov_old_v":
                d = g1 + self.mu * vold if self.nesterov else self.v
            elif name == "nesterov_ignored":
                d = self.v
            elif name == "nesterov_always":
                d = g1 + self.mu * self.v
            elif name == "nesterov_raw_g":
                d = g + self.mu * self.v if self.nesterov else self.v
            else:
                d = g1 + self.mu * self.v if self.nesterov else self.v
            if name == "lr_sign":
                self.x = self.x + lr * d
            elif name == "wd_decoupled":
                gg = g
                self.v = self.mu * vold + gg
                d = gg + self.mu * self.v if self.nesterov else self.v
                self.x = self.x * (1 - lr * self.wd[None, :]) - lr * d
            else:
                self.x = self.x - lr * d

        def average(self):
            if name == "sum_not_mean":
                self.z = self.s.sum(axis=0)
            elif name == "drops_last_replica":
                self.z = self.s[:-1].sum(axis=0) / max(1, self.K - 1)
            elif name == "mean_of_x_not_s":
                self.z = self.x.sum(axis=0) / self.K
            else:
                super().average()

        def merge(self, resnapshot=True):
            if name == "merge_sign":
                self.x = self.z[None, :] - (self.x - self.s)
            elif name == "merge_swapped":
                self.x = self.z[None, :] + (self.s - self.x)
            elif name == "merge_drops_s":
                self.x = self.z[None, :] + self.x
            elif name == "merge_is_reset":
                self.x = np.repeat(self.z[None, :], self.K, axis=0)
            elif name == "merge_half":
                self.x = 0.5 * self.z[None, :] + 0.5 * self.x
            elif name == "merge_resets_v":
                self.x = self.z[None, :] + (self.x - self.s)
                self.v = np.zeros_like(self.v)
            elif name == "merge_averages_v":
                self.x = self.z[None, :] + (self.x - self.s)
                self.v = np.repeat(self.v.mean(axis=0)[None, :], self.K, axis=0)
            else:
                self.x = self.z[None, :] + (self.x - self.s)
            if name == "merge_always_resnaps":
                self.s = self.x.copy()
            elif resnapshot and name != "merge_never_resnaps":
                self.s = self.x.copy()

        def prologue(self, grads0, lr):
            if name == "sent_is_x0":
                # the other reading of x^i_0 in step 9a: the initial weights
                self.snapshot()
                self.local_step(grads0, lr)
                self.average()
                self.tau = 0
            else:
                super().prologue(grads0, lr)

        def iteration(self, grads, lr, m):
            if name == "cadence_off_by_one":
                return super().iteration(grads, lr, m + 1)
            if name == "merge_before_step":
                self.tau += 1
                fired = self.tau == m
                if fired:
                    self.merge(True)
                    self.average()
                    self.tau = 0
                self.local_step(grads, lr)
                return fired
            return super().iteration(grads, lr, m)
    return lambda K, numels, mu, nes, wd: M(K, numels, mu, nes, wd)


MUTANTS = ["wd_dropped", "wd_sign", "dampening", "v_from_raw_g", "nesterov_old_v",
           "nesterov_ignored", "nesterov_always", "nesterov_raw_g", "lr_sign", "wd_decoupled",
           "sum_not_mean", "drops_last_replica", "mean_of_x_not_s",
           "merge_sign", "merge_swapped", "merge_drops_s", "merge_is_reset", "merge_half",
           "merge_resets_v", "merge_averages_v", "merge_always_resnaps", "merge_never_resnaps",
           "sent_is_x0", "cadence_off_by_one", "merge_before_step"]


@pytest.mark.parametrize("name", MUTANTS)
def test_planted_mistake_is_caught(name):
    make = _mutant(name)
    caught = []
    for check in CHECKS:
        try:
            check(make)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"


def test_unmutated_reference_passes_mutant_harness():
    make = _mutant("none")
    for check in CHECKS:
        check(make)


# ------------------------------------------------------------ P9, P10, misc
def test_p9_bf16_rounding_matches_torch():
    L = O32.lib()
    r = np.random.default_rng(0)
    bits = r.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0x00000000, 0x80000000, 0x7f800000, 0xff800000, 0x7f7fffff, 0x3f808000,
                        0x3f818000, 0x3f808001, 0x3f807fff, 0x00000001, 0x00008000, 0x00018000,
                        0x7f7f8000, 0x7f7f7fff, 0x33800000], dtype=np.uint32)
    bits = np.concatenate([bits, special])
    f = bits.view(np.float32)
    finite = np.isfinite(f) | np.isinf(f)
    f = f[finite]
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.lasgd_oracle_bf16_rne(float(a)) for a in f[:20000]], dtype=np.uint16)
    np.testing.assert_array_equal(got, want[:20000])
    got_s = np.array([L.lasgd_oracle_bf16_rne(float(a)) for a in f[-len(special):]], dtype=np.uint16)
    np.testing.assert_array_equal(got_s, want[-len(special):])
    # NaN stays NaN
    h = L.lasgd_oracle_bf16_rne(float("nan"))
    assert (h & 0x7f80) == 0x7f80 and (h & 0x7f) != 0
    # widening is the exact inverse on bf16 values
    back = np.array([L.lasgd_oracle_bf16_widen(int(b)) for b in want[:5000]], dtype=np.float32)
    np.testing.assert_array_equal(back.view(np.uint32), want[:5000].astype(np.uint32) << 16)


def test_p9_bf16_storage_tracks_master():
    K, N = 2, 300
    o = O32.Oracle(K, [N], 0.9, True, [1e-4], storage="bf16")
    from paper_2203_13085_amd import workloads as W
    x0 = W.to_bf16_bits(draws(90, 1, N, 0.1)[0])
    g = [[W.to_bf16_bits(a) for a in draws(91 + i, K, N, 1e-3)] for i in range(5)]
    def after(i, o):
        for k in range(K):
            want = torch.from_numpy(o.x[k].copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
            np.testing.assert_array_equal(o.x16[k], want)
    O32.run_schedule(o, x0, lambda i: g[i], 0.1, 2, 4, after)
    # bf16 run == f32 run fed the widened inputs (storage only changes what is stored)
    o2 = O32.Oracle(K, [N], 0.9, True, [1e-4])
    O32.run_schedule(o2, W.bf16_bits_to_f32(x0), lambda i: [W.bf16_bits_to_f32(a) for a in g[i]], 0.1, 2, 4)
    for k in range(K):
        np.testing.assert_array_equal(o.x[k], o2.x[k])
        np.testing.assert_array_equal(o.v[k], o2.v[k])
    np.testing.assert_array_equal(o.z, o2.z)


def test_p10_mean_is_exactly_rounded():
    for K in (2, 3, 7, 8, 32):
        N = 4000
        o = O32.Oracle(K, [N], 0.0, False, [0.0])
        vals = draws(100 + K, K, N, 1.0) * np.float32(10.0) ** np.random.default_rng(K).integers(-3, 3, (K, 1)).astype(np.float32)
        for k in range(K):
            o.x[k][:] = vals[k]
        o.snapshot()
        o.average()
        exact = np.array([Fraction(math.fsum(float(vals[k, e]) for k in range(K))) / K for e in range(N)],
                         dtype=object)
        want = np.array([np.float32(float(q)) for q in exact])
        ulp = np.spacing(np.abs(want))
        assert np.all(np.abs(o.z - want) <= ulp)
        assert np.mean(o.z == want) > 0.999


def test_fp32_oracle_tracks_fp64_reference_on_ragged_list():
    """Two separately written codes, per-tensor weight decay, both momentum forms."""
    from paper_2203_13085_amd import workloads as W
    for nes in (True, False):
        w = W.small(K=3, nesterov=nes)
        wd = [0.0 if i % 3 == 0 else 1e-3 * (i + 1) for i in range(len(w.numels))]
        x0 = np.concatenate([W.initial_tensor(w, t) for t in range(len(w.numels))])
        def grads(i):
            return [np.concatenate([W.gradient_tensor(w, i, k, t) for t in range(len(w.numels))])
                    for k in range(w.K)]
        a = O32.Oracle(w.K, w.numels, w.momentum, nes, wd)
        b = O64.Ref64(w.K, w.numels, float(np.float32(w.momentum)), nes, [float(np.float32(x)) for x in wd])
        recA = {}
        O32.run_schedule(a, x0, grads, w.lr, w.m, w.T,
                         lambda i, o: recA.__setitem__(i, (X(o).copy(), V(o).copy(), S(o).copy(), Z(o).copy())))
        def after(i, o):
            for got, ref, nm in zip(recA[i], (X(o), V(o), S(o), Z(o)), "xvsz"):
                assert np.all(np.abs(got - ref) <= 1e-7 + 1e-6 * np.abs(ref)), (i, nm)
        O64.run_schedule(b, x0, grads, float(np.float32(w.lr)), w.m, w.T, after)


def test_threads_do_not_change_results():
    from paper_2203_13085_amd import workloads as W
    w = W.small(K=4)
    x0 = np.concatenate([W.initial_tensor(w, t) for t in range(len(w.numels))])
    grads = lambda i: [np.concatenate([W.gradient_tensor(w, i, k, t) for t in range(len(w.numels))])
                       for k in range(w.K)]
    wd = [w.weight_decay] * len(w.numels)
    a = O32.run_schedule(O32.Oracle(w.K, w.numels, w.momentum, True, wd), x0, grads, w.lr, w.m, w.T)
    b = O32.run_schedule(O32.Oracle(w.K, w.numels, w.momentum, True, wd, threads=3), x0, grads, w.lr, w.m, w.T)
    for k in range(w.K):
        np.testing.assert_array_equal(a.x[k], b.x[k])
    np.testing.assert_array_equal(a.z, b.z)
