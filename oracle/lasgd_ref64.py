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
        self.tau = 0
        self.t = 0

    def set_model(self, x0: np.ndarray) -> None:
        self.x[:] = np.asarray(x0, dtype=np.float64)[None, :]
        self.v[:] = 0.0

    def local_step(self, grads: Sequence[np.ndarray], lr: float) -> None:
        g = np.stack([np.asarray(a, dtype=np.float64) for a in grads])
        g = g + self.wd[None, :] * self.x           # L2 decay joins the gradient
        self.v = self.mu * self.v + g               # momentum buffer, zero dampening
        d = g + self.mu * self.v if self.nesterov else self.v
        self.x = self.x - lr * d

    def snapshot(self) -> None:
        self.s = self.x.copy()

    def average(self) -> None:
        self.z = self.s.sum(axis=0) / self.K

    def merge(self, resnapshot: bool = True) -> None:
        self.x = self.z[None, :] + (self.x - self.s)
        if resnapshot:
            self.s = self.x.copy()

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
