"""ctypes binding of the LASGD HIP library: argument marshalling only.

Every operation runs in the library's kernels; this module converts Python
values to the C ABI of include/lasgd.h and turns status codes into
exceptions.  PyTorch appears only as the provider of device buffers and
streams.  There is no CPU fallback: if the shared library is missing, loading
fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblasgd_hip.so")

OK, ERR_INVALID, ERR_STATE, ERR_ALLOC, ERR_HIP, ERR_UNSUPPORTED = range(6)
F32, BF16 = 0, 1
STATE_X, STATE_V, STATE_S, STATE_Z = range(4)
_STATUS_NAMES = ["OK", "ERR_INVALID", "ERR_STATE", "ERR_ALLOC", "ERR_HIP", "ERR_UNSUPPORTED"]

EXPORTS = ["lasgd_create", "lasgd_bind", "lasgd_init_master", "lasgd_local_step", "lasgd_snapshot",
           "lasgd_average", "lasgd_average_done", "lasgd_merge", "lasgd_step_merge",
           "lasgd_read_state", "lasgd_sync", "lasgd_set_tuning", "lasgd_get_tuning",
           "lasgd_last_error", "lasgd_destroy", "lasgd_local_step_ex", "lasgd_snapshot_ex",
           "lasgd_average_ex", "lasgd_merge_ex", "lasgd_step_merge_ex", "lasgd_set_elastic",
           "lasgd_sgd_ar_step", "lasgd_global_update_static", "lasgd_step_merge_average"]


class LasgdError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{_STATUS_NAMES[status] if 0 <= status < 6 else status}: {text}")
        self.status = status


class Config(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("n_tensors", ctypes.c_int32),
                ("numel", ctypes.POINTER(ctypes.c_int64)), ("storage", ctypes.c_int),
                ("momentum", ctypes.c_float), ("nesterov", ctypes.c_int32),
                ("weight_decay", ctypes.POINTER(ctypes.c_float)), ("wd_scalar", ctypes.c_float),
                ("main_stream", ctypes.c_void_p), ("side_stream", ctypes.c_void_p)]


class Tuning(ctypes.Structure):
    _fields_ = [("vec", ctypes.c_int32), ("kper_step", ctypes.c_int32), ("kper_merge", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("avg_split", ctypes.c_int32),
                ("avg_max_blocks", ctypes.c_int32), ("nontemporal", ctypes.c_int32),
                ("chunk_step", ctypes.c_int32), ("chunk_merge", ctypes.c_int32),
                ("waves_per_block", ctypes.c_int32), ("race_probe", ctypes.c_int32),
                ("group_r", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None


def load() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2203_13085_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.c_void_p
    i32, f32, i64 = ctypes.c_int32, ctypes.c_float, ctypes.c_int64
    L.lasgd_create.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(P)]
    L.lasgd_bind.argtypes = [P, i32, ctypes.POINTER(P), ctypes.POINTER(P)]
    L.lasgd_init_master.argtypes = [P]
    L.lasgd_local_step.argtypes = [P, f32]
    L.lasgd_snapshot.argtypes = [P]
    L.lasgd_average.argtypes = [P]
    L.lasgd_average_done.argtypes = [P, ctypes.POINTER(i32)]
    L.lasgd_merge.argtypes = [P, i32]
    L.lasgd_step_merge.argtypes = [P, f32, i32]
    L.lasgd_step_merge_average.argtypes = [P, f32]
    L.lasgd_read_state.argtypes = [P, i32, i32, i32, ctypes.POINTER(f32), i64]
    L.lasgd_sync.argtypes = [P]
    L.lasgd_set_tuning.argtypes = [P, ctypes.POINTER(Tuning)]
    L.lasgd_get_tuning.argtypes = [P, ctypes.POINTER(Tuning)]
    u64, f32p = ctypes.c_uint64, ctypes.POINTER(ctypes.c_float)
    L.lasgd_local_step_ex.argtypes = [P, f32p, u64]
    L.lasgd_snapshot_ex.argtypes = [P, u64]
    L.lasgd_average_ex.argtypes = [P, u64]
    L.lasgd_merge_ex.argtypes = [P, u64, i32]
    L.lasgd_step_merge_ex.argtypes = [P, f32p, u64, u64, i32]
    L.lasgd_set_elastic.argtypes = [P, f32, f32]
    L.lasgd_sgd_ar_step.argtypes = [P, f32]
    L.lasgd_global_update_static.argtypes = [i32, i64, ctypes.POINTER(P), ctypes.POINTER(P), i32, P]
    L.lasgd_last_error.argtypes = [P]
    L.lasgd_last_error.restype = ctypes.c_char_p
    L.lasgd_destroy.argtypes = [P]
    L.lasgd_destroy.restype = None
    for name in EXPORTS:
        if name not in ("lasgd_last_error", "lasgd_destroy"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


STATIC_MAX_N = 32 << 20


def global_update_static(x: Sequence[int], sent: Sequence[int], n: int, resnapshot: bool = True,
                         stream: Optional[int] = None) -> None:
    """lasgd_global_update_static: x / sent are device addresses, one per replica."""
    L = load()
    K = len(x)
    assert len(sent) == K
    xa = (ctypes.c_void_p * max(K, 1))(*x)
    sa = (ctypes.c_void_p * max(K, 1))(*sent)
    st = L.lasgd_global_update_static(K, int(n), xa, sa, int(bool(resnapshot)), stream or None)
    if st != OK:
        raise LasgdError(st, L.lasgd_last_error(None).decode())


class Context:
    """One LASGD context: K replicas of a parameter list on the current GPU.

    Method names are the C entry points without the prefix.  Streams are raw
    hipStream_t handles (e.g. torch.cuda.Stream().cuda_stream); 0 / None is
    the default stream.
    """

    def __init__(self, K: int, numels: Sequence[int], *, storage: int = F32, momentum: float = 0.9,
                 nesterov: bool = True, weight_decay=None, wd_scalar: float = 0.0,
                 main_stream: Optional[int] = None, side_stream: Optional[int] = None):
        self._L = load()
        self.K, self.numels = int(K), [int(n) for n in numels]
        self.N = sum(self.numels)
        self.storage = storage
        arr = (ctypes.c_int64 * len(self.numels))(*self.numels)
        wd = None
        if weight_decay is not None:
            assert len(weight_decay) == len(self.numels)
            wd = (ctypes.c_float * len(self.numels))(*[float(w) for w in weight_decay])
        cfg = Config(self.K, len(self.numels), arr, storage, float(momentum), int(bool(nesterov)),
                     wd, float(wd_scalar), main_stream or None, side_stream or None)
        h = ctypes.c_void_p()
        st = self._L.lasgd_create(ctypes.byref(cfg), ctypes.byref(h))
        if st != OK:
            raise LasgdError(st, self._L.lasgd_last_error(None).decode())
        self._h = h

    # -- plumbing ---------------------------------------------------------
    def _check(self, st: int) -> None:
        if st != OK:
            raise LasgdError(st, self._L.lasgd_last_error(self._h).decode())

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._L.lasgd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C entry points -------------------------------------------------
    def bind(self, k: int, params: Sequence[int], grads: Sequence[int]) -> None:
        """params / grads: device addresses (e.g. tensor.data_ptr()), one per tensor."""
        n = len(self.numels)
        assert len(params) == n and len(grads) == n
        pa = (ctypes.c_void_p * n)(*params)
        ga = (ctypes.c_void_p * n)(*grads)
        self._check(self._L.lasgd_bind(self._h, k, pa, ga))

    def init_master(self) -> None:
        self._check(self._L.lasgd_init_master(self._h))

    def local_step(self, lr: float) -> None:
        self._check(self._L.lasgd_local_step(self._h, lr))

    def snapshot(self) -> None:
        self._check(self._L.lasgd_snapshot(self._h))

    def average(self) -> None:
        self._check(self._L.lasgd_average(self._h))

    def average_done(self) -> bool:
        d = ctypes.c_int32(0)
        self._check(self._L.lasgd_average_done(self._h, ctypes.byref(d)))
        return bool(d.value)

    def merge(self, resnapshot: bool = True) -> None:
        self._check(self._L.lasgd_merge(self._h, int(resnapshot)))

    def step_merge(self, lr: float, resnapshot: bool = True) -> None:
        self._check(self._L.lasgd_step_merge(self._h, lr, int(resnapshot)))

    def step_merge_average(self, lr: float) -> None:
        self._check(self._L.lasgd_step_merge_average(self._h, lr))

    def _lrs(self, lr):
        vals = [float(lr)] * self.K if np.isscalar(lr) else [float(a) for a in lr]
        assert len(vals) == self.K
        return (ctypes.c_float * self.K)(*vals)

    def local_step_ex(self, lr, mask: int) -> None:
        self._check(self._L.lasgd_local_step_ex(self._h, self._lrs(lr), mask))

    def snapshot_ex(self, mask: int) -> None:
        self._check(self._L.lasgd_snapshot_ex(self._h, mask))

    def average_ex(self, mask: int) -> None:
        self._check(self._L.lasgd_average_ex(self._h, mask))

    def merge_ex(self, mask: int, resnapshot: bool = True) -> None:
        self._check(self._L.lasgd_merge_ex(self._h, mask, int(resnapshot)))

    def step_merge_ex(self, lr, step_mask: int, merge_mask: int, resnapshot: bool = True) -> None:
        self._check(self._L.lasgd_step_merge_ex(self._h, self._lrs(lr), step_mask, merge_mask, int(resnapshot)))

    def set_elastic(self, alpha: float, beta: float) -> None:
        self._check(self._L.lasgd_set_elastic(self._h, alpha, beta))

    def sgd_ar_step(self, lr: float) -> None:
        self._check(self._L.lasgd_sgd_ar_step(self._h, lr))

    def read_state(self, which: int, k: int = 0, tensor: int = -1) -> np.ndarray:
        # an out-of-range tensor index is the library's to refuse
        n = self.N if tensor < 0 else self.numels[tensor] if tensor < len(self.numels) else 1
        out = np.empty(n, dtype=np.float32)
        self._check(self._L.lasgd_read_state(self._h, which, k, tensor,
                                             out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), n))
        return out

    def sync(self) -> None:
        self._check(self._L.lasgd_sync(self._h))

    def set_tuning(self, **kw) -> None:
        t = Tuning(**{k: int(v) for k, v in kw.items()})
        self._check(self._L.lasgd_set_tuning(self._h, ctypes.byref(t)))

    def get_tuning(self) -> dict:
        t = Tuning()
        self._check(self._L.lasgd_get_tuning(self._h, ctypes.byref(t)))
        return {f: getattr(t, f) for f, _ in Tuning._fields_}
