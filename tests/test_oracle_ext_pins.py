"""Pins for the oracle's extensions: adaptive per-replica step counts (Sec. 4),
elastic coefficients alpha/beta (Sec. 3 Eq. 5-6), the partial All-Reduce
(Sec. 6) and the SGD All-Reduce comparator (Sec. 2).  Same scheme as
test_oracle_pins.py: every check runs on the fp32 C oracle, on the fp64
reference and on planted-mistake variants that must each be caught.

    E1  a full mask equals no mask; replicas outside a mask are untouched, bit for bit
    E2  the partial mean is the exactly rounded mean over the participants (divisor = their number)
    E3  a partial global update preserves the participants' mean and leaves the others alone
    E4  scripted step counts that are all equal reproduce the fixed cadence
    E5  exact-rational brute force of the scripted schedule (per-replica counts and step sizes)
    E6  plain SGD closed form: after a global update x_k = z - sum of eta*g over k's own steps
    E7  alpha = beta = 1 is Algorithm 1
    E8  cadence 1, plain SGD: the recurrences of Eq. 5-6 in their printed form
    E9  alpha = 0 decouples the replicas (each is torch.optim.SGD on its own gradients);
        beta = 0 freezes the centre after its initialisation
    E10 zero gradients: every global update shrinks deviations from the mean by (1 - alpha)
    E11 exact-rational brute force with alpha, beta
    E12 SGD-AR: every replica follows torch.optim.SGD on the mean gradient; K = 1 is the local update
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import lasgd_oracle as O32
from oracle import lasgd_ref64 as O64
from tests.test_oracle_pins import (X, V, S, Z, close, draws, is32, make32, make64, put, run, tol,
                                    _torch_sgd)


def run_dyn(o, x0, g, lr, rounds, after=None):
    mod = O32 if is32(o) else O64
    return mod.run_dynamic(o, x0, lambda i: [g[i][k] for k in range(o.K)], lr, rounds, after)


# ------------------------------------------------------------------ masks
def check_e1_masks(make):
    K, N = 4, 70
    g = draws(1, K, N, 0.1)
    xs = draws(2, K, N, 0.5)
    a, b = make(K, [N], 0.9, True, [1e-2]), make(K, [N], 0.9, True, [1e-2])
    for o in (a, b):
        for k in range(K):
            put(o, "x", k, xs[k])
    a.local_step(list(g), 0.1)
    b.local_step(list(g), 0.1, mask=(1 << K) - 1)
    np.testing.assert_array_equal(X(a), X(b))
    a.snapshot(); b.snapshot(mask=(1 << K) - 1)
    a.average(); b.average(mask=(1 << K) - 1)
    np.testing.assert_array_equal(Z(a), Z(b))
    a.local_step(list(g), 0.1); b.local_step(list(g), [0.1] * K)
    a.merge(True); b.merge(True, mask=(1 << K) - 1)
    np.testing.assert_array_equal(X(a), X(b))
    np.testing.assert_array_equal(S(a), S(b))
    # a partial mask touches only its members
    before = (X(b).copy(), V(b).copy(), S(b).copy())
    mask = 0b0101
    b.local_step(list(g), [0.3, 0.0, 0.2, 0.0], mask=mask)
    for k in range(K):
        same = np.array_equal(X(b)[k], before[0][k]) and np.array_equal(V(b)[k], before[1][k])
        assert same == (k in (1, 3)), f"replica {k}"
    np.testing.assert_array_equal(S(b), before[2])
    # per-replica step sizes: replica 0 moved by 0.3*d, replica 2 by 0.2*d
    c = make(K, [N], 0.9, True, [1e-2])
    for k in range(K):
        put(c, "x", k, before[0][k]); put(c, "v", k, before[1][k])
    c.local_step(list(g), 0.3)
    close(b, X(b)[0], X(c)[0], what="lr of replica 0")
    assert not np.allclose(X(b)[2], X(c)[2], rtol=1e-9, atol=0)
    b.snapshot(mask=0b1000)
    for k in range(K):
        assert np.array_equal(S(b)[k], X(b)[k]) == (k == 3) or np.array_equal(before[2][k], X(b)[k])


def check_e2_partial_mean(make):
    K, N = 6, 500
    o = make(K, [N], 0.0, False, [0.0])
    vals = draws(3, K, N, 1.0) * np.float32(10.0) ** np.random.default_rng(3).integers(-2, 3, (K, 1)).astype(np.float32)
    for k in range(K):
        put(o, "x", k, vals[k])
    o.snapshot()
    for mask in (0b000001, 0b101010, 0b011111, 0b100001):
        ks = [k for k in range(K) if (mask >> k) & 1]
        o.average(mask=mask)
        exact = [Fraction(math.fsum(float(vals[k, e]) for k in ks)) / len(ks) for e in range(N)]
        if is32(o):
            want = np.array([np.float32(float(q)) for q in exact])
            assert np.all(np.abs(Z(o) - want.astype(np.float64)) <= np.spacing(np.abs(want)).astype(np.float64))
        else:
            close(o, Z(o), np.array([float(q) for q in exact]), what=f"partial mean {mask:b}")


def check_e3_partial_merge(make):
    K, N = 5, 64
    o = make(K, [N], 0.0, False, [0.0])
    ss, xs = draws(4, K, N, 0.3), draws(5, K, N, 0.3)
    for k in range(K):
        put(o, "x", k, ss[k])
    o.snapshot()
    mask = 0b01101
    ks = [0, 2, 3]
    for k in range(K):
        put(o, "x", k, xs[k])
    o.average(mask=mask)
    close(o, Z(o), ss[ks].astype(np.float64).mean(axis=0), what="mean over participants")
    o.merge(True, mask=mask)
    close(o, X(o)[ks].mean(axis=0), xs[ks].astype(np.float64).mean(axis=0), what="participants' mean preserved")
    for k in (1, 4):
        np.testing.assert_array_equal(X(o)[k], xs[k].astype(np.float64))
        np.testing.assert_array_equal(S(o)[k], ss[k].astype(np.float64))
    for k in ks:
        np.testing.assert_array_equal(S(o)[k], X(o)[k])


# ------------------------------------------------------- adaptive cadence
def check_e4_equal_counts_are_fixed_cadence(make):
    K, N, n, R = 3, 40, 3, 3
    x0 = draws(10, 1, N, 0.5)[0]
    g = draws(11, (n * R + 1) * K, N, 0.1).reshape(n * R + 1, K, N)
    a = run(make(K, [N], 0.9, True, [1e-3]), x0, g, 0.05, n, n * R)
    rec = {}
    b = run_dyn(make(K, [N], 0.9, True, [1e-3]), x0, g, lambda k, c: 0.05, [[n] * K] * R)
    np.testing.assert_array_equal(X(a), X(b))
    np.testing.assert_array_equal(V(a), V(b))
    np.testing.assert_array_equal(Z(a), Z(b))


def _dyn_rational(x0, g, lr, mu, wd, nesterov, rounds, alpha=1, beta=1):
    K, N = len(g[0]), len(x0)
    F = Fraction
    mu, alpha, beta = F(mu), F(alpha), F(beta)
    x = [[F(float(a)) for a in x0] for _ in range(K)]
    v = [[F(0)] * N for _ in range(K)]
    s = [[F(0)] * N for _ in range(K)]
    z = [F(0)] * N
    clock = [0] * K
    first = [True]

    def step(tick, ks):
        for k in ks:
            eta = F(lr(k, clock[k]))
            for e in range(N):
                gg = F(float(g[tick][k][e])) + F(wd) * x[k][e]
                v[k][e] = mu * v[k][e] + gg
                d = gg + mu * v[k][e] if nesterov else v[k][e]
                x[k][e] -= eta * d
            clock[k] += 1

    def send():
        for k in range(K):
            s[k] = list(x[k])
        b = F(1) if first[0] else beta
        first[0] = False
        for e in range(N):
            z[e] = (1 - b) * z[e] + b * sum(s[k][e] for k in range(K)) / K

    step(0, range(K))
    send()
    tick = 0
    for counts in rounds:
        for j in range(max(counts)):
            tick += 1
            step(tick, [k for k in range(K) if counts[k] > j])
        for k in range(K):
            for e in range(N):
                x[k][e] = x[k][e] + alpha * (z[e] - s[k][e])
        send()
    return x, v, s, z


def _f(a):
    return np.array([[float(c) for c in r] for r in a]) if isinstance(a[0], list) else np.array([float(c) for c in a])


def check_e5_dynamic_bruteforce(make):
    K, N = 3, 5
    rounds = [[2, 1, 3], [1, 1, 1], [4, 2, 1], [1, 5, 2]]
    ticks = 1 + sum(max(c) for c in rounds)
    mu, wd = 0.5, 0.125
    lr = lambda k, c: float(np.float32(0.1 / (1 + c) + 0.01 * k))
    x0 = draws(20, 1, N, 0.5)[0]
    g = draws(21, ticks * K, N, 0.1).reshape(ticks, K, N)
    for nes in (True, False):
        o = run_dyn(make(K, [N], mu, nes, [wd]), x0, g, lr, rounds)
        x, v, s, z = _dyn_rational(x0, g, lr, mu, wd, nes, rounds)
        close(o, X(o), _f(x), steps=ticks, what="x")
        close(o, V(o), _f(v), steps=ticks, what="v")
        close(o, S(o), _f(s), steps=ticks, what="s")
        close(o, Z(o), _f(z), steps=ticks, what="z")


def check_e6_dynamic_closed_form(make):
    K, N = 4, 16
    rounds = [[1, 2, 3, 1], [5, 1, 1, 2]]
    ticks = 1 + sum(max(c) for c in rounds)
    eta = 0.25
    x0 = draws(30, 1, N, 0.5)[0]
    g = draws(31, ticks * K, N, 0.1).reshape(ticks, K, N)
    g64 = g.astype(np.float64)
    rec = {}
    run_dyn(make(K, [N], 0.0, False, [0.0]), x0, g, lambda k, c: eta, rounds,
            after=lambda t, o: rec.__setitem__(t, (X(o).copy(), Z(o).copy())))
    sent = x0.astype(np.float64)[None, :] - eta * g64[0]
    z = sent.mean(axis=0)
    tick = 0
    for counts in rounds:
        prog = np.zeros((K, N))
        for j in range(max(counts)):
            tick += 1
            for k in range(K):
                if counts[k] > j:
                    prog[k] -= eta * g64[tick][k]
        expect = z[None, :] + prog
        o_x, o_z = rec[tick]
        dummy = make(1, [1], 0.0, False, [0.0])
        close(dummy, o_x, expect, steps=tick, what=f"x after round ending at tick {tick}")
        z = expect.mean(axis=0)
        close(dummy, o_z, z, steps=tick, what="next mean")


# ------------------------------------------------------------ alpha, beta
def _elastic_run(o, x0, g, lr, m, T, alpha, beta, after=None):
    K = o.K
    o.set_model(x0)
    o.local_step([g[0][k] for k in range(K)], lr)
    o.snapshot()
    o.average(beta=beta)
    if after:
        after(0, o)
    tau = 0
    for i in range(1, T + 1):
        o.local_step([g[i][k] for k in range(K)], lr)
        tau += 1
        if tau == m:
            o.merge(True, alpha=alpha)
            o.average(beta=beta)
            tau = 0
        if after:
            after(i, o)
    return o


def check_e7_alpha_beta_one_is_algorithm_1(make):
    K, N, m, T = 3, 30, 2, 6
    x0 = draws(40, 1, N, 0.5)[0]
    g = draws(41, (T + 1) * K, N, 0.1).reshape(T + 1, K, N)
    a = run(make(K, [N], 0.9, True, [1e-3]), x0, g, 0.1, m, T)
    b = _elastic_run(make(K, [N], 0.9, True, [1e-3]), x0, g, 0.1, m, T, 1.0, 1.0)
    np.testing.assert_array_equal(X(a), X(b))
    np.testing.assert_array_equal(Z(a), Z(b))
    # and the general formula evaluated just off 1 stays close to it
    c = _elastic_run(make(K, [N], 0.9, True, [1e-3]), x0, g, 0.1, m, T, 1.0 - 2.0 ** -20, 1.0 - 2.0 ** -20)
    assert np.max(np.abs(X(c) - X(a))) < 1e-4


def check_e8_printed_recurrences(make):
    """Cadence 1, plain SGD.  With x_t the sent models and z_t the centre that
    includes their mean:  z_t = (1-beta) z_{t-1} + beta mean_i x_t^i   (Eq. 5)
                          x_{t+1}^i = alpha z_t + (1-alpha) x_t^i - eta g_t^i   (Eq. 6)"""
    K, N, T, eta = 3, 24, 7, 0.3
    x0 = draws(50, 1, N, 1.0)[0]
    g = draws(51, (T + 1) * K, N, 0.2).reshape(T + 1, K, N)
    g64 = g.astype(np.float64)
    for alpha, beta in ((0.5, 0.75), (0.25, 1.0), (1.0, 0.5), (0.9, 0.1)):
        rec = {}
        o = make(K, [N], 0.0, False, [0.0])
        _elastic_run(o, x0, g, eta, 1, T, alpha, beta, after=lambda i, o: rec.__setitem__(i, (X(o).copy(), Z(o).copy())))
        xt = x0.astype(np.float64)[None, :] - eta * g64[0]          # the first sent models
        z = xt.mean(axis=0)                                         # first mean initialises the centre
        close(o, rec[0][1], z, what="centre after the prologue")
        for t in range(1, T + 1):
            xt = alpha * z[None, :] + (1 - alpha) * xt - eta * g64[t]
            z = (1 - beta) * z + beta * xt.mean(axis=0)
            close(o, rec[t][0], xt, steps=t + 1, what=f"Eq.6 alpha={alpha} t={t}")
            close(o, rec[t][1], z, steps=t + 1, what=f"Eq.5 beta={beta} t={t}")


def check_e9_decoupling_limits(make):
    K, N, T, eta, mu, wd = 3, 20, 6, 0.1, 0.9, 1e-2
    x0 = draws(60, 1, N, 0.5)[0]
    g = draws(61, (T + 1) * K, N, 0.1).reshape(T + 1, K, N)
    rec = {}
    o = make(K, [N], mu, True, [wd])
    _elastic_run(o, x0, g, eta, 2, T, 0.0, 1.0, after=lambda i, o: rec.__setitem__(i, X(o).copy()))
    for k in range(K):
        ref = _torch_sgd(x0, g[:, k, :], eta, mu, wd, True, torch.float32 if is32(o) else torch.float64)
        for i in range(T + 1):
            close(o, rec[i][k], ref[i], steps=4 * (i + 1), what=f"alpha=0: replica {k} is plain SGD, step {i}")
    zs = {}
    o = make(K, [N], mu, True, [wd])
    _elastic_run(o, x0, g, eta, 2, T, 1.0, 0.0, after=lambda i, o: zs.__setitem__(i, Z(o).copy()))
    for i in range(1, T + 1):
        np.testing.assert_array_equal(zs[i], zs[0])


def check_e10_contraction(make):
    K, N = 4, 32
    for alpha in (0.25, 0.5, 1.0):
        o = make(K, [N], 0.0, False, [0.0])
        xs = draws(70, K, N, 1.0)
        for k in range(K):
            put(o, "x", k, xs[k])
        o.snapshot()
        o.average()
        mean = xs.astype(np.float64).mean(axis=0)
        dev = xs.astype(np.float64) - mean
        for r in range(3):
            o.merge(True, alpha=alpha)
            o.average()
            dev = (1 - alpha) * dev
            close(o, X(o) - mean[None, :], dev, steps=4 * (r + 1), what=f"alpha={alpha} round {r}")
            close(o, Z(o), mean, steps=4 * (r + 1), what="centre stays at the mean")


def check_e11_elastic_bruteforce(make):
    K, N, m, R = 3, 4, 2, 3
    T = m * R
    mu, wd, eta = 0.5, 0.25, 0.125
    alpha, beta = 0.375, 0.625
    x0 = draws(80, 1, N, 0.5)[0]
    g = draws(81, (T + 1) * K, N, 0.1).reshape(T + 1, K, N)
    o = _elastic_run(make(K, [N], mu, True, [wd]), x0, g, eta, m, T, alpha, beta)
    x, v, s, z = _dyn_rational(x0, g, lambda k, c: eta, mu, wd, True, [[m] * K] * R, alpha, beta)
    close(o, X(o), _f(x), steps=T, what="x")
    close(o, V(o), _f(v), steps=T, what="v")
    close(o, Z(o), _f(z), steps=T, what="z")


# ------------------------------------------------------------------ SGD-AR
def check_e12_sgd_ar(make):
    K, N, T, eta, mu, wd = 4, 48, 10, 0.1, 0.9, 1e-2
    x0 = draws(90, 1, N, 0.5)[0]
    g = draws(91, T * K, N, 0.1).reshape(T, K, N)
    o = make(K, [N], mu, True, [wd])
    o.set_model(x0)
    gbar = g.astype(np.float64).mean(axis=1)
    ref = _torch_sgd(x0, gbar, eta, mu, wd, True, torch.float64)
    for i in range(T):
        o.sgd_ar_step([g[i][k] for k in range(K)], eta)
        for k in range(K):
            close(o, X(o)[k], ref[i], steps=4 * (i + 1), what=f"SGD-AR step {i} replica {k}")
            np.testing.assert_array_equal(X(o)[k], X(o)[0])
    a, b = make(1, [N], mu, True, [wd]), make(1, [N], mu, True, [wd])
    a.set_model(x0); b.set_model(x0)
    for i in range(3):
        a.sgd_ar_step([g[i][0]], eta)
        b.local_step([g[i][0]], eta)
    np.testing.assert_array_equal(X(a), X(b))
    np.testing.assert_array_equal(V(a), V(b))


CHECKS = [check_e1_masks, check_e2_partial_mean, check_e3_partial_merge,
          check_e4_equal_counts_are_fixed_cadence, check_e5_dynamic_bruteforce,
          check_e6_dynamic_closed_form, check_e7_alpha_beta_one_is_algorithm_1,
          check_e8_printed_recurrences, check_e9_decoupling_limits, check_e10_contraction,
          check_e11_elastic_bruteforce, check_e12_sgd_ar]


@pytest.mark.parametrize("check", CHECKS, ids=lambda f: f.__name__)
@pytest.mark.parametrize("make", [make32, make64], ids=["c_fp32", "numpy_fp64"])
def test_ext_pin(make, check):
    check(make)


# ------------------------------------------------- planted mistakes (CPU)
def _mutant(name):
    class M(O64.Ref64):
        def local_step(self, grads, lr, mask=None):
            if name == "mask_ignored_in_step":
                mask = None
            if name == "lr_not_per_replica" and not np.isscalar(lr):
                lr = float(np.asarray(lr)[0])
            super().local_step(grads, lr, mask)

        def snapshot(self, mask=None):
            super().snapshot(None if name == "mask_ignored_in_snapshot" else mask)

        def average(self, mask=None, beta=1.0):
            sel = self._sel(mask)
            if name == "partial_mean_divides_by_K":
                mean = self.s[sel].sum(axis=0) / self.K
            elif name == "partial_mean_over_everyone":
                mean = self.s.sum(axis=0) / self.K
            else:
                mean = self.s[sel].sum(axis=0) / int(sel.sum())
            first = not self.center_valid
            self.center_valid = True
            if first and name != "centre_not_initialised":
                beta = 1.0
            if name == "beta_swapped":
                self.z = beta * self.z + (1.0 - beta) * mean
            elif name == "beta_ignored":
                self.z = mean
            else:
                self.z = (1.0 - beta) * self.z + beta * mean

        def merge(self, resnapshot=True, mask=None, alpha=1.0):
            if name == "mask_ignored_in_merge":
                mask = None
            sel = self._sel(mask)
            if name == "pull_from_current_model":
                x = self.x + alpha * (self.z[None, :] - self.x)
            elif name == "alpha_ignored":
                x = self.z[None, :] + (self.x - self.s)
            elif name == "alpha_on_progress":
                x = self.z[None, :] + alpha * (self.x - self.s)
            elif name == "eq6_without_progress":
                x = alpha * self.z[None, :] + (1 - alpha) * self.s
            else:
                x = self.x + alpha * (self.z[None, :] - self.s) if alpha != 1.0 else self.z[None, :] + (self.x - self.s)
            self.x = np.where(sel[:, None], x, self.x)
            if resnapshot:
                if name == "resnapshot_everyone":
                    self.s = self.x.copy()
                else:
                    self.s = np.where(sel[:, None], self.x, self.s)

        def sgd_ar_step(self, grads, lr):
            g = np.stack([np.asarray(a, dtype=np.float64) for a in grads])
            if name == "sgd_ar_sum":
                super().local_step([g.sum(axis=0)] * self.K, lr)
            elif name == "sgd_ar_own_gradient":
                super().local_step(list(g), lr)
            elif name == "sgd_ar_first_gradient":
                super().local_step([g[0]] * self.K, lr)
            else:
                super().sgd_ar_step(grads, lr)
    return lambda K, numels, mu, nes, wd: M(K, numels, mu, nes, wd)


MUTANTS = ["mask_ignored_in_step", "lr_not_per_replica", "mask_ignored_in_snapshot",
           "partial_mean_divides_by_K", "partial_mean_over_everyone", "centre_not_initialised",
           "beta_swapped", "beta_ignored", "mask_ignored_in_merge", "pull_from_current_model",
           "alpha_ignored", "alpha_on_progress", "eq6_without_progress", "resnapshot_everyone",
           "sgd_ar_sum", "sgd_ar_own_gradient", "sgd_ar_first_gradient"]


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


def test_dynamic_clock_mistake_is_caught():
    """A driver that indexes eta by the global tick instead of each replica's own
    clock must disagree with the brute force."""
    def bad_run_dynamic(o, x0, grads, lr, rounds, after=None):
        K = o.K
        o.set_model(x0)
        tick = 0
        o.local_step(grads(0), [lr(k, 0) for k in range(K)])
        o.snapshot(); o.average()
        for counts in rounds:
            for j in range(max(counts)):
                tick += 1
                o.local_step(grads(tick), [lr(k, tick) for k in range(K)],
                             mask=sum(1 << k for k in range(K) if counts[k] > j))
            o.merge(True); o.average()
        return o
    good = O64.run_dynamic
    try:
        O64.run_dynamic = bad_run_dynamic
        with pytest.raises(AssertionError):
            check_e5_dynamic_bruteforce(make64)
    finally:
        O64.run_dynamic = good
    check_e5_dynamic_bruteforce(make64)


def test_bf16_storage_variants_of_the_extensions():
    """bf16 storage changes what is stored, never the arithmetic: the elastic and
    SGD-AR paths on bf16 inputs equal the fp32 paths fed the widened inputs, and
    the stored bf16 parameters are torch's rounding of the master."""
    from paper_2203_13085_amd import workloads as W
    K, N = 3, 200
    x0 = W.to_bf16_bits(draws(200, 1, N, 0.1)[0])
    g = [[W.to_bf16_bits(a) for a in draws(201 + i, K, N, 1e-2)] for i in range(6)]
    wide = lambda b: W.bf16_bits_to_f32(b)

    def rne(a):
        return torch.from_numpy(a.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)

    # elastic
    a = O32.Oracle(K, [N], 0.9, True, [1e-3], storage="bf16")
    b = O32.Oracle(K, [N], 0.9, True, [1e-3])
    a.set_model(x0); b.set_model(wide(x0))
    for o, gg in ((a, g), (b, [[wide(t) for t in row] for row in g])):
        o.local_step(gg[0], 0.1); o.snapshot(); o.average(beta=0.5)
        for i in range(1, 5):
            o.local_step(gg[i], 0.1)
            if i % 2 == 0:
                o.merge(True, alpha=0.25); o.average(beta=0.5)
    for k in range(K):
        np.testing.assert_array_equal(a.x[k], b.x[k])
        np.testing.assert_array_equal(a.s[k], b.s[k])
        np.testing.assert_array_equal(a.x16[k], rne(a.x[k]))
    np.testing.assert_array_equal(a.z, b.z)
    # SGD-AR
    a = O32.Oracle(K, [N], 0.9, True, [1e-3], storage="bf16")
    b = O32.Oracle(K, [N], 0.9, True, [1e-3])
    a.set_model(x0); b.set_model(wide(x0))
    for i in range(4):
        a.sgd_ar_step(g[i], 0.1)
        b.sgd_ar_step([wide(t) for t in g[i]], 0.1)
    for k in range(K):
        np.testing.assert_array_equal(a.x[k], b.x[k])
        np.testing.assert_array_equal(a.v[k], b.v[k])
        np.testing.assert_array_equal(a.x16[k], rne(a.x[k]))


@pytest.mark.parametrize("seed", range(24))
def test_random_schedules_two_codes_agree(seed):
    """Randomly drawn replica counts, parameter lists, optimizer settings, elastic
    coefficients, participant sets and per-replica step counts: the fp32 C oracle
    must track the separately written fp64 reference through the whole run."""
    r = np.random.default_rng(1000 + seed)
    K = int(r.integers(1, 9))
    numels = [int(n) for n in r.integers(1, 40, size=int(r.integers(1, 5)))]
    N = sum(numels)
    mu = float(np.float32(r.choice([0.0, 0.5, 0.9])))
    nes = bool(r.integers(0, 2)) and mu > 0
    wd = [float(np.float32(w)) for w in r.choice([0.0, 1e-4, 1e-2], size=len(numels))]
    alpha = float(np.float32(r.choice([1.0, 1.0, 0.5, 0.125])))
    beta = float(np.float32(r.choice([1.0, 1.0, 0.75, 0.25])))
    a = O32.Oracle(K, numels, mu, nes, wd)
    b = O64.Ref64(K, numels, mu, nes, wd)
    x0 = draws(seed, 1, N, 0.3)[0]
    a.set_model(x0); b.set_model(x0)
    full = (1 << K) - 1
    pending = 0
    sent = 0
    for step in range(14):
        g = list(draws(100 * seed + step, K, N, 0.05))
        lrs = [float(np.float32(v)) for v in r.uniform(0.01, 0.2, size=K)]
        mask = int(r.integers(0, full + 1))
        for o in (a, b):
            o.local_step(g, lrs, mask=mask)
        if pending and r.random() < 0.6:
            part = int(r.integers(1, pending + 1)) & pending or pending
            resnap = bool(r.integers(0, 2))
            for o in (a, b):
                o.merge(resnap, mask=part, alpha=alpha)
            pending &= ~part
            sent = (sent | part) if resnap else (sent & ~part)
        if not pending:
            late = full & ~sent
            if late and r.random() < 0.7:
                for o in (a, b):
                    o.snapshot(mask=late)
                sent |= late
            if sent and r.random() < 0.8:
                part = int(r.integers(1, full + 1)) & sent or sent
                for o in (a, b):
                    o.average(mask=part, beta=beta)
                pending = part
        for got, ref, nm in ((X(a), X(b), "x"), (V(a), V(b), "v"), (S(a), S(b), "s"), (Z(a)[None], Z(b)[None], "z")):
            bad = np.abs(got - ref) > 3e-7 + 3e-6 * np.abs(ref)
            assert not bad.any(), (seed, step, nm, float(np.abs(got - ref).max()))
