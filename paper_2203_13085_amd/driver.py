"""Device-side plumbing around the binding: buffers, streams, Algorithm 1's loop.

PyTorch is used for device memory and streams only.  Parameters and gradients
of each replica live in one flat device buffer per replica, each tensor
starting on a 1 KiB boundary, so that the KiB a wave moves per access is one
aligned KiB (measured: tensors that start 256 or 512 bytes off such a boundary
cost 3-5 % of the streaming rate on MI355X).  The gradient buffer starts 4 KiB
into its allocation: separately allocated tensors of a real model sit at
unrelated phases, whereas two identically laid-out buffers that both start on
an allocator boundary would send every wave's parameter and gradient accesses
to the same memory channels at the same moment.  The library sees per-tensor
pointers, exactly as it would see a real model's parameter list.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .workloads import Workload

_ALIGN = 256          # elements: every tensor starts on 1 KiB (fp32) / 512 B (bf16)
_GRAD_LEAD_BYTES = 4096  # the gradient buffer's offset inside its allocation


def _offsets(numels: Sequence[int]) -> np.ndarray:
    off, out = 0, []
    for n in numels:
        out.append(off)
        off += (int(n) + _ALIGN - 1) // _ALIGN * _ALIGN
    out.append(off)
    return np.asarray(out, dtype=np.int64)


class DeviceReplicas:
    """K replicas' parameters and gradients on the GPU, bound to a LASGD context."""

    def __init__(self, w: Workload, weight_decay: Optional[Sequence[float]] = None,
                 side_stream: bool = True, device: str = "cuda:0", grad_lead_bytes: int = _GRAD_LEAD_BYTES):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the LASGD path runs only on the device")
        self.w = w
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.numels = w.numels
        self.off = _offsets(self.numels)
        self.bf16 = w.storage == "bf16"
        dt = torch.bfloat16 if self.bf16 else torch.float32
        self.esize = 2 if self.bf16 else 4
        self.main = torch.cuda.Stream(device=self.dev)
        self.side = torch.cuda.Stream(device=self.dev) if side_stream else self.main
        total = int(self.off[-1])
        lead = int(grad_lead_bytes) // self.esize
        self.x = [torch.zeros(total, dtype=dt, device=self.dev) for _ in range(w.K)]
        self._g_alloc = [torch.zeros(total + lead, dtype=dt, device=self.dev) for _ in range(w.K)]
        self.g = [t[lead:] for t in self._g_alloc]
        torch.cuda.synchronize()
        wd = list(weight_decay) if weight_decay is not None else [w.weight_decay] * len(self.numels)
        self.ctx = B.Context(w.K, self.numels, storage=B.BF16 if self.bf16 else B.F32,
                             momentum=w.momentum, nesterov=w.nesterov, weight_decay=wd,
                             main_stream=self.main.cuda_stream, side_stream=self.side.cuda_stream)
        for k in range(w.K):
            self.ctx.bind(k, [self.x[k].data_ptr() + int(o) * self.esize for o in self.off[:-1]],
                          [self.g[k].data_ptr() + int(o) * self.esize for o in self.off[:-1]])
        # packed <-> padded index map for uploads and downloads
        idx = np.concatenate([np.arange(n, dtype=np.int64) + o for n, o in zip(self.numels, self.off[:-1])])
        self._idx = torch.from_numpy(idx).to(self.dev)
        self._contig = bool((idx == np.arange(idx.size)).all())

    # ---- host <-> device (untimed plumbing) ---------------------------------
    def _put(self, dst: torch.Tensor, flat: np.ndarray) -> None:
        """flat: packed values over all tensors; fp32, or uint16 bf16 patterns."""
        if self.bf16:
            src = torch.from_numpy(np.ascontiguousarray(flat).view(np.int16)).to(self.dev).view(torch.bfloat16)
        else:
            src = torch.from_numpy(np.ascontiguousarray(flat, dtype=np.float32)).to(self.dev)
        if self._contig:
            dst[: src.numel()].copy_(src)
        else:
            dst[self._idx] = src

    def _get(self, src: torch.Tensor) -> np.ndarray:
        t = src[: self._idx.numel()] if self._contig else src[self._idx]
        if self.bf16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    def load_model(self, x0: np.ndarray) -> None:
        """Every replica starts from the same model (Sec. 4)."""
        self.ctx.sync()
        for k in range(self.w.K):
            self._put(self.x[k], x0)
        torch.cuda.synchronize()
        if self.bf16:
            self.ctx.init_master()

    def load_grads(self, grads: Sequence[np.ndarray]) -> None:
        self.ctx.sync()
        for k in range(self.w.K):
            self._put(self.g[k], grads[k])
        torch.cuda.synchronize()

    def params(self, k: int) -> np.ndarray:
        """The caller-visible parameters of replica k (fp32, or bf16 patterns)."""
        self.ctx.sync()
        return self._get(self.x[k])

    # ---- Algorithm 1 with a fixed cadence ------------------------------------
    def prologue(self, lr: float) -> None:
        self.ctx.local_step(lr)      # steps 2-3
        self.ctx.snapshot()          # step 4: send
        self.ctx.average()           #         the All-Reduce starts on the side stream

    def iteration(self, lr: float, tau: int, m: int, fused: bool = True, fused_mean: bool = False) -> int:
        """Steps 6-9 for one tick of the local clock; returns the new tau.
        fused_mean: the global update and the next All-Reduce go out as one pass on the
        main stream (lasgd_step_merge_average) instead of step_merge + average."""
        tau += 1
        if tau == m:
            if fused_mean:
                self.ctx.step_merge_average(lr)
                return 0
            if fused:
                self.ctx.step_merge(lr, True)
            else:
                self.ctx.local_step(lr)
                self.ctx.merge(True)
            self.ctx.average()
            return 0
        self.ctx.local_step(lr)
        return tau

    def adaptive_iteration(self, lr: float, tau: int, tau_max: int, fused_mean: bool = False) -> tuple:
        """Steps 6-9 with the paper's adaptive rule: the global update fires as
        soon as the All-Reduce is found finished, or when tau reaches tau_max (then
        the main stream waits for it on the device; the host never blocks).  The
        poll happens before the step is enqueued so that step and global update
        can go out as one fused pass.  fused_mean: the next All-Reduce is taken in that
        same pass (lasgd_step_merge_average).  Returns (new tau, fired)."""
        tau += 1
        if tau >= tau_max or self.ctx.average_done():
            if fused_mean:
                self.ctx.step_merge_average(lr)
            else:
                self.ctx.step_merge(lr, True)
                self.ctx.average()
            return 0, True
        self.ctx.local_step(lr)
        return tau, False

    def capture_cycle(self, lr: float, m: int):
        """Record one closed cycle as a HIP graph (for workloads whose kernels are so
        short that launch latency dominates):

            mean (forks to the side stream)  ||  m-1 local steps   ->   fused step + global update (joins)

        The cycle starts from "models sent, no mean pending" (after the prologue's
        step and snapshot, or after any step_merge) and ends in the same state, so the
        graph can be replayed back to back; lr is frozen into it.  Replay with
        `with torch.cuda.stream(self.main): graph.replay()`."""
        graph = torch.cuda.CUDAGraph()
        self.ctx.sync()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=self.main):
            self.ctx.average()
            for _ in range(m - 1):
                self.ctx.local_step(lr)
            self.ctx.step_merge(lr, True)
        return graph

    def capture_fused_cycle(self, lr: float, m: int):
        """Record m-1 local steps + lasgd_step_merge_average as a HIP graph on the main stream.
        Call it when the pending mean was itself made by lasgd_step_merge_average (or with one
        stream for everything): the graph then contains no wait on an event recorded outside it.
        It starts and ends in the state "models sent, mean pending", so it replays back to back."""
        graph = torch.cuda.CUDAGraph()
        self.ctx.sync()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=self.main):
            for _ in range(m - 1):
                self.ctx.local_step(lr)
            self.ctx.step_merge_average(lr)
        return graph

    def close(self) -> None:
        self.ctx.close()
