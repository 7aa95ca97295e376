"""LASGD CPU oracle, fp32 pinned order -- TEST INFRASTRUCTURE, not the product.

Python driver around lasgd_oracle.c: it holds the state of K replicas and
walks Algorithm 1 of the paper (Sec. 4) with a fixed merge cadence.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it.
It imports nothing from the HIP package.

State per replica k (flat fp32 arrays over all tensors, concatenated):
    x[k]  local model x^i                     (Algorithm 1, steps 1, 3, 7, 9b)
    v[k]  momentum buffer                     (Sec. 5.2: Nesterov momentum)
    s[k]  the model last sent to All-Reduce, x^i_t   (steps 4, 9c; used in 9a)
    z     the All-Reduce result z_t           (Sec. 3, Eq. 8)
bf16 storage adds x16[k], the bf16 copy of x[k] the user sees; x[k] is then
the fp32 master.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from typing import Callable, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lasgd_oracle.c")
_LIB = os.path.join(_HERE, "liblasgd_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with the host compiler (contraction off)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        f32p = ctypes.POINTER(ctypes.c_float)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i64, f32, i32 = ctypes.c_int64, ctypes.c_float, ctypes.c_int32
        L.lasgd_oracle_bf16_rne.argtypes = [f32]
        L.lasgd_oracle_bf16_rne.restype = ctypes.c_uint16
        L.lasgd_oracle_bf16_widen.argtypes = [ctypes.c_uint16]
        L.lasgd_oracle_bf16_widen.restype = f32
        L.lasgd_oracle_local_step_f32.argtypes = [f32p, f32p, f32p, i64, f32, f32, f32, i32]
        L.lasgd_oracle_local_step_bf16.argtypes = [f32p, u16p, f32p, u16p, i64, f32, f32, f32, i32]
        L.lasgd_oracle_snapshot.argtypes = [f32p, f32p, i64]
        L.lasgd_oracle_average.argtypes = [f32p, ctypes.POINTER(f32p), i32, i64]
        L.lasgd_oracle_merge_f32.argtypes = [f32p, f32p, f32p, i64, i32]
        L.lasgd_oracle_merge_bf16.argtypes = [f32p, u16p, f32p, f32p, i64, i32]
        L.lasgd_oracle_widen_bf16.argtypes = [f32p, u16p, i64]
        L.lasgd_oracle_average_elastic.argtypes = [f32p, ctypes.POINTER(f32p), i32, i64, f32]
        L.lasgd_oracle_merge_elastic_f32.argtypes = [f32p, f32p, f32p, i64, f32, i32]
        L.lasgd_oracle_merge_elastic_bf16.argtypes = [f32p, u16p, f32p, f32p, i64, f32, i32]
        L.lasgd_oracle_mean_gradient_f32.argtypes = [f32p, ctypes.POINTER(f32p), i32, i64]
        L.lasgd_oracle_mean_gradient_bf16.argtypes = [f32p, ctypes.POINTER(u16p), i32, i64]
        L.lasgd_oracle_local_step_bf16_g32.argtypes = [f32p, u16p, f32p, f32p, i64, f32, f32, f32, i32]
        for name in ("local_step_f32", "local_step_bf16", "snapshot", "average",
                     "merge_f32", "merge_bf16", "widen_bf16", "average_elastic",
                     "merge_elastic_f32", "merge_elastic_bf16", "mean_gradient_f32",
                     "mean_gradient_bf16", "local_step_bf16_g32"):
            getattr(L, "lasgd_oracle_" + name).restype = None
        _lib = L
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _u16(a: np.ndarray):
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


class Oracle:
    """K replicas of a parameter list, updated by the C oracle.

    numels        element count of each tensor
    weight_decay  one value per tensor
    threads       replicas are independent in every step but the mean, so the
                  replica loop may be spread over this many host threads
                  (the C calls release the GIL); 1 = plain sequential.
    """

    def __init__(self, K: int, numels: Sequence[int], momentum: float, nesterov: bool,
                 weight_decay: Sequence[float], storage: str = "f32", threads: int = 1):
        assert K >= 1 and len(numels) == len(weight_decay)
        self.K, self.numels = K, [int(n) for n in numels]
        self.off = np.concatenate([[0], np.cumsum(self.numels)]).astype(np.int64)
        self.N = int(self.off[-1])
        self.mu, self.nesterov = float(momentum), bool(nesterov)
        self.wd = [float(w) for w in weight_decay]
        self.storage = storage
        self.x = [np.zeros(self.N, np.float32) for _ in range(K)]
        self.v = [np.zeros(self.N, np.float32) for _ in range(K)]
        self.s = [np.zeros(self.N, np.float32) for _ in range(K)]
        self.z = np.zeros(self.N, np.float32)
        self.x16 = [np.zeros(self.N, np.uint16) for _ in range(K)] if storage == "bf16" else None
        self.threads = max(1, int(threads))
        self._pool = ThreadPoolExecutor(self.threads) if self.threads > 1 else None
        self.center_valid = False   # has z been computed at least once
        self.tau = 0      # local steps since the last global update (tau_i)
        self.t = 0        # global clock (number of global updates)

    # -- helpers ----------------------------------------------------------
    def _members(self, mask) -> List[int]:
        """Replicas taking part: all of them, or those whose bit is set in `mask`."""
        if mask is None:
            return list(range(self.K))
        return [k for k in range(self.K) if (int(mask) >> k) & 1]

    def _each_replica(self, fn: Callable[[int], None], mask=None) -> None:
        ks = self._members(mask)
        if self._pool is None:
            for k in ks:
                fn(k)
        else:
            list(self._pool.map(fn, ks))

    def set_model(self, x0: np.ndarray) -> None:
        """Step 1: every replica starts from the same model (Sec. 4).
        f32: x0 is fp32.  bf16: x0 holds bf16 bit patterns; the master is
        their exact widening."""
        L = lib()
        for k in range(self.K):
            if self.storage == "bf16":
                self.x16[k][:] = x0
                L.lasgd_oracle_widen_bf16(_f32(self.x[k]), _u16(self.x16[k]), self.N)
            else:
                self.x[k][:] = x0
            self.v[k][:] = 0.0

    # -- the four operations ------------------------------------------------
    def local_step(self, grads: Sequence[np.ndarray], lr, mask=None) -> None:
        """Algorithm 1 steps 3 / 7; grads[k] is flat over all tensors (fp32, or
        bf16 bit patterns in bf16 storage).  `lr` is one value or one per
        replica (eta is indexed by each node's local clock); with `mask`, only
        the replicas whose bit is set take the step (nodes run at their own pace)."""
        L = lib()
        lrs = [float(lr)] * self.K if np.isscalar(lr) else [float(a) for a in lr]

        def one(k: int) -> None:
            for t, n in enumerate(self.numels):
                a, b = int(self.off[t]), int(self.off[t + 1])
                if self.storage == "bf16":
                    L.lasgd_oracle_local_step_bf16(
                        _f32(self.x[k][a:b]), _u16(self.x16[k][a:b]), _f32(self.v[k][a:b]),
                        _u16(grads[k][a:b]), n, lrs[k], self.mu, self.wd[t], int(self.nesterov))
                else:
                    L.lasgd_oracle_local_step_f32(
                        _f32(self.x[k][a:b]), _f32(self.v[k][a:b]), _f32(grads[k][a:b]),
                        n, lrs[k], self.mu, self.wd[t], int(self.nesterov))

        self._each_replica(one, mask)

    def snapshot(self, mask=None) -> None:
        """Steps 4 / 9c: keep the model that goes to the All-Reduce."""
        L = lib()
        self._each_replica(lambda k: L.lasgd_oracle_snapshot(_f32(self.s[k]), _f32(self.x[k]), self.N), mask)

    def average(self, mask=None, beta: float = 1.0) -> None:
        """Eq. 8: z is the mean of the sent models -- of all replicas, or of
        the subset `mask` (partial All-Reduce, Sec. 6: the divisor is the number
        of participants).  beta != 1: the elastic centre of Eq. 5; the very
        first mean initialises the centre (there is no earlier z to keep)."""
        L = lib()
        ks = self._members(mask)
        assert ks, "an All-Reduce needs at least one participant"
        if not self.center_valid:
            beta = 1.0
        self.center_valid = True

        def run(zs, ss, n):
            ptrs = (ctypes.POINTER(ctypes.c_float) * len(ks))(*[_f32(a) for a in ss])
            if beta == 1.0:
                L.lasgd_oracle_average(_f32(zs), ptrs, len(ks), n)
            else:
                L.lasgd_oracle_average_elastic(_f32(zs), ptrs, len(ks), n, beta)

        if self._pool is None:
            run(self.z, [self.s[k] for k in ks], self.N)
            return
        # element ranges are independent; split them, not the replica sum
        cuts = np.linspace(0, self.N, self.threads + 1).astype(np.int64)

        def part(i: int) -> None:
            a, b = int(cuts[i]), int(cuts[i + 1])
            if b > a:
                run(self.z[a:b], [self.s[k][a:b] for k in ks], b - a)

        list(self._pool.map(part, range(self.threads)))

    def merge(self, resnapshot: bool = True, mask=None, alpha: float = 1.0) -> None:
        """Steps 9a-b (and 9c when resnapshot) for all replicas or the subset
        `mask`.  alpha != 1: the elastic pull of Eq. 6, x <- x + alpha (z - s)."""
        L = lib()

        def one(k: int) -> None:
            if self.storage == "bf16":
                if alpha == 1.0:
                    L.lasgd_oracle_merge_bf16(_f32(self.x[k]), _u16(self.x16[k]), _f32(self.s[k]),
                                              _f32(self.z), self.N, int(resnapshot))
                else:
                    L.lasgd_oracle_merge_elastic_bf16(_f32(self.x[k]), _u16(self.x16[k]), _f32(self.s[k]),
                                                      _f32(self.z), self.N, alpha, int(resnapshot))
            elif alpha == 1.0:
                L.lasgd_oracle_merge_f32(_f32(self.x[k]), _f32(self.s[k]), _f32(self.z),
                                         self.N, int(resnapshot))
            else:
                L.lasgd_oracle_merge_elastic_f32(_f32(self.x[k]), _f32(self.s[k]), _f32(self.z),
                                                 self.N, alpha, int(resnapshot))

        self._each_replica(one, mask)

    def sgd_ar_step(self, grads: Sequence[np.ndarray], lr: float) -> None:
        """The SGD All-Reduce comparator (Sec. 2): average the K gradients, then
        every replica takes the same local update with the mean gradient."""
        L = lib()
        gbar = np.empty(self.N, np.float32)
        if self.storage == "bf16":
            ptrs = (ctypes.POINTER(ctypes.c_uint16) * self.K)(*[_u16(a) for a in grads])
            L.lasgd_oracle_mean_gradient_bf16(_f32(gbar), ptrs, self.K, self.N)
        else:
            ptrs = (ctypes.POINTER(ctypes.c_float) * self.K)(*[_f32(a) for a in grads])
            L.lasgd_oracle_mean_gradient_f32(_f32(gbar), ptrs, self.K, self.N)

        def one(k: int) -> None:
            for t, n in enumerate(self.numels):
                a, b = int(self.off[t]), int(self.off[t + 1])
                if self.storage == "bf16":
                    L.lasgd_oracle_local_step_bf16_g32(
                        _f32(self.x[k][a:b]), _u16(self.x16[k][a:b]), _f32(self.v[k][a:b]),
                        _f32(gbar[a:b]), n, lr, self.mu, self.wd[t], int(self.nesterov))
                else:
                    L.lasgd_oracle_local_step_f32(
                        _f32(self.x[k][a:b]), _f32(self.v[k][a:b]), _f32(gbar[a:b]),
                        n, lr, self.mu, self.wd[t], int(self.nesterov))

        self._each_replica(one)

    # -- Algorithm 1 with a fixed cadence ------------------------------------
    def prologue(self, grads0: Sequence[np.ndarray], lr: float) -> None:
        """Steps 2-5: first local update, send, start the All-Reduce."""
        self.local_step(grads0, lr)
        self.snapshot()
        self.average()
        self.tau = 0

    def iteration(self, grads: Sequence[np.ndarray], lr: float, m: int) -> bool:
        """Steps 6-9 for one value of the local clock.  The global update fires
        when tau reaches m (= tau_max; the early "All-Reduce done" exit is not
        taken, so the run is deterministic).  Returns True if it fired."""
        self.local_step(grads, lr)
        self.tau += 1
        if self.tau == m:
            self.merge(resnapshot=True)
            self.average()
            self.t += 1
            self.tau = 0
            return True
        return False


def run_schedule(o: Oracle, x0: np.ndarray, grads: Callable[[int], List[np.ndarray]],
                 lr: float, m: int, T: int,
                 after: Optional[Callable[[int, Oracle], None]] = None) -> Oracle:
    """Algorithm 1: prologue, then T loop iterations; `grads(step)` returns the
    K flat gradients of that step (step 0 = prologue); `after(step, o)` sees
    the state after each step."""
    o.set_model(x0)
    o.prologue(grads(0), lr)
    if after:
        after(0, o)
    for i in range(1, T + 1):
        o.iteration(grads(i), lr, m)
        if after:
            after(i, o)
    return o


def run_dynamic(o: Oracle, x0: np.ndarray, grads: Callable[[int], List[np.ndarray]],
                lr: Callable[[int, int], float], rounds: Sequence[Sequence[int]],
                after: Optional[Callable[[int, Oracle], None]] = None) -> Oracle:
    """Algorithm 1 with the adaptive synchronisation rate scripted from outside.

    rounds[r][k] = number of local updates replica k performs while All-Reduce r
    is in flight (1 <= n <= tau_max: every node takes at least one step per
    loop iteration before it can notice that the All-Reduce is done, and at
    most tau_max).  Nodes run concurrently, so tick j of a round is taken by
    every replica with n > j at once; `grads(tick)` gives that tick's K
    gradients (entries of idle replicas are ignored) and `lr(k, local_clock)`
    the step size of replica k at its own local clock t^i.
    """
    K = o.K
    clock = [0] * K
    o.set_model(x0)
    tick = 0
    o.local_step(grads(tick), [lr(k, 0) for k in range(K)])
    clock = [1] * K
    o.snapshot()
    o.average()
    if after:
        after(tick, o)
    for counts in rounds:
        assert len(counts) == K and min(counts) >= 1
        for j in range(max(counts)):
            tick += 1
            mask = sum(1 << k for k in range(K) if counts[k] > j)
            o.local_step(grads(tick), [lr(k, clock[k]) for k in range(K)], mask=mask)
            for k in range(K):
                if counts[k] > j:
                    clock[k] += 1
            if j == max(counts) - 1:
                o.merge(resnapshot=True)     # every node has seen the All-Reduce end by now
                o.average()
                o.t += 1
            if after:
                after(tick, o)
    return o
