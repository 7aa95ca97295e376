"""LASGD reference in fp64 numpy -- TEST INFRASTRUCTURE, not the product.

The definitions of the paper written out with whole-array numpy expressions in
double precision, independently of lasgd_oracle.c.  It serves two purposes:
the invariants of the method are checked on it to ~1e-12, and the fp32 oracle
is checked against it within the fp32 tolerance, so that a slip in either one
shows up as a disagreement between two separately written codes.

    local update   Algorithm 1 steps 3, 7 with the optimizer of Sec. 5.2
    send           Algorithm 1 steps 4, 9c
    mean           Sec. 3, Eq. 8
    global update  Algorithm 1 step 9a-b
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np


class Ref64:
    def __init__(self, K: int, numels: Sequence[int], momentum: float, nesterov: bool,
                 weight_decay: Sequence[float]):
        self.K = K
        self.numels = [int(n) for n in numels]
        self.N = sum(self.numels)
        self.mu, self.nesterov = float(momentum), bool(nesterov)
        # weight decay is per tensor; spread it per element once
        self.wd = np.repeat(np.asarray(weight_decay, dtype=np.float64), self.numels)
        self.x = np.zeros((K, self.N))
        self.v = np.zeros((K, self.N))
        self.s = np.zeros((K, self.N))
        self.z = np.zeros(self.N)
        self.center_valid = False
        self.tau = 0
        self.t = 0

    def set_model(self, x0: np.ndarray) -> None:
        self.x[:] = np.asarray(x0, dtype=np.float64)[None, :]
        self.v[:] = 0.0

    def _sel(self, mask) -> np.ndarray:
        """Boolean selector of the replicas taking part (all when mask is None)."""
        if mask is None:
            return np.ones(self.K, dtype=bool)
        return np.array([(int(mask) >> k) & 1 == 1 for k in range(self.K)])

    def local_step(self, grads: Sequence[np.ndarray], lr, mask=None) -> None:
        sel = self._sel(mask)
        lrs = np.full(self.K, float(lr)) if np.isscalar(lr) else np.asarray(lr, dtype=np.float64)
        g = np.stack([np.asarray(a, dtype=np.float64) for a in grads])
        g = g + self.wd[None, :] * self.x           # L2 decay joins the gradient
        v = self.mu * self.v + g                    # momentum buffer, zero dampening
        d = g + self.mu * v if self.nesterov else v
        x = self.x - lrs[:, None] * d
        self.v = np.where(sel[:, None], v, self.v)  # idle replicas keep their state
        self.x = np.where(sel[:, None], x, self.x)

    def snapshot(self, mask=None) -> None:
        sel = self._sel(mask)
        self.s = np.where(sel[:, None], self.x, self.s)

    def average(self, mask=None, beta: float = 1.0) -> None:
        sel = self._sel(mask)
        mean = self.s[sel].sum(axis=0) / int(sel.sum())
        if not self.center_valid:
            beta = 1.0                              # the first mean initialises the centre
        self.center_valid = True
        self.z = (1.0 - beta) * self.z + beta * mean

    def merge(self, resnapshot: bool = True, mask=None, alpha: float = 1.0) -> None:
        sel = self._sel(mask)
        if alpha == 1.0:
            x = self.z[None, :] + (self.x - self.s)
        else:
            x = self.x + alpha * (self.z[None, :] - self.s)
        self.x = np.where(sel[:, None], x, self.x)
        if resnapshot:
            self.s = np.where(sel[:, None], self.x, self.s)

    def sgd_ar_step(self, grads: Sequence[np.ndarray], lr: float) -> None:
        gbar = np.stack([np.asarray(a, dtype=np.float64) for a in grads]).mean(axis=0)
        self.local_step([gbar] * self.K, lr)

    def prologue(self, grads0, lr: float) -> None:
        self.local_step(grads0, lr)
        self.snapshot()
        self.average()
        self.tau = 0

    def iteration(self, grads, lr: float, m: int) -> bool:
        self.local_step(grads, lr)
        self.tau += 1
        if self.tau == m:
            self.merge(True)
            self.average()
            self.t += 1
            self.tau = 0
            return True
        return False


def run_schedule(o: Ref64, x0: np.ndarray, grads: Callable[[int], List[np.ndarray]],
                 lr: float, m: int, T: int,
                 after: Optional[Callable[[int, Ref64], None]] = None) -> Ref64:
    o.set_model(x0)
    o.prologue(grads(0), lr)
    if after:
        after(0, o)
    for i in range(1, T + 1):
        o.iteration(grads(i), lr, m)
        if after:
            after(i, o)
    return o


def run_dynamic(o: Ref64, x0, grads, lr, rounds, after=None) -> Ref64:
    """Algorithm 1 with scripted per-replica step counts per All-Reduce; see the
    fp32 oracle's run_dynamic for the meaning of the arguments."""
    K = o.K
    o.set_model(x0)
    tick = 0
    o.local_step(grads(0), [lr(k, 0) for k in range(K)])
    clock = [1] * K
    o.snapshot()
    o.average()
    if after:
        after(tick, o)
    for counts in rounds:
        last = max(counts) - 1
        for j in range(last + 1):
            tick += 1
            active = [k for k in range(K) if counts[k] > j]
            o.local_step(grads(tick), [lr(k, clock[k]) for k in range(K)], mask=sum(1 << k for k in active))
            for k in active:
                clock[k] += 1
            if j == last:
                o.merge(True)
                o.average()
                o.t += 1
            if after:
                after(tick, o)
    return o
