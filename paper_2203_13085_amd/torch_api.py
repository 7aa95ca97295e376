"""LASGD for K torch models that live on one GPU.

A thin convenience over the binding for callers who already have K replicas of a
torch module (the paper's P workers, Sec. 4): it binds every replica's parameter
and gradient tensors to a LASGD context once and then runs one iteration of
Algorithm 1 per `step()` -- a local update of all replicas, and every m-th
call the fused global update followed by the launch of the next mean on the
side stream.  All arithmetic happens in the library's kernels; torch supplies
the tensors, the autograd gradients and the streams.

Gradient tensors are allocated here once and attached to the parameters
(`p.grad`), so that autograd accumulates into buffers whose addresses never
change; clear them with `zero_grad()` of this class (or
`module.zero_grad(set_to_none=False)`), never by dropping them.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


class LASGD:
    def __init__(self, replicas: Sequence[torch.nn.Module], lr: float, momentum: float = 0.9,
                 nesterov: bool = True, weight_decay: float = 0.0, m: int = 1,
                 no_decay_1d: bool = False, side_stream: bool = True):
        """replicas: K modules with identical parameter lists on the same GPU, already
        holding the same initial weights (every node starts from the same model).
        m: local steps per global update (tau_max with the early exit disabled).
        no_decay_1d: apply no weight decay to 1-D tensors (norm scales, biases)."""
        assert len(replicas) >= 1 and m >= 1
        self.replicas = list(replicas)
        self.params: List[List[torch.nn.Parameter]] = [[p for p in r.parameters() if p.requires_grad] for r in self.replicas]
        first = self.params[0]
        assert first, "no trainable parameters"
        dev = first[0].device
        assert dev.type == "cuda", "the LASGD path runs only on the GPU"
        dtype = first[0].dtype
        assert dtype in (torch.float32, torch.bfloat16)
        for ps in self.params:
            assert len(ps) == len(first)
            for p, q in zip(ps, first):
                assert p.shape == q.shape and p.dtype == dtype and p.device == dev and p.is_contiguous()
        self.lr, self.m, self.tau, self.t = float(lr), int(m), 0, 0
        self.device = dev
        self.main = torch.cuda.Stream(device=dev)
        self.side = torch.cuda.Stream(device=dev) if side_stream else self.main
        wd = [0.0 if (no_decay_1d and p.dim() <= 1) else float(weight_decay) for p in first]
        with torch.cuda.device(dev):
            self.ctx = B.Context(len(self.replicas), [p.numel() for p in first],
                                 storage=B.BF16 if dtype == torch.bfloat16 else B.F32,
                                 momentum=momentum, nesterov=nesterov, weight_decay=wd,
                                 main_stream=self.main.cuda_stream, side_stream=self.side.cuda_stream)
            for k, ps in enumerate(self.params):
                for p in ps:
                    if p.grad is None or not p.grad.is_contiguous():
                        p.grad = torch.zeros_like(p, memory_format=torch.contiguous_format)
                self.ctx.bind(k, [p.data_ptr() for p in ps], [p.grad.data_ptr() for p in ps])
            torch.cuda.synchronize(dev)
            if dtype == torch.bfloat16:
                self.ctx.init_master()
        self._started = False

    def zero_grad(self) -> None:
        for ps in self.params:
            for p in ps:
                p.grad.zero_()

    def _check_bound(self) -> None:
        # a dropped or replaced .grad would leave the library reading a stale buffer
        for ps in self.params:
            for p in ps:
                assert p.grad is not None, "a gradient buffer was dropped (use zero_grad(set_to_none=False))"

    @torch.no_grad()
    def step(self, lr: Optional[float] = None) -> bool:
        """One iteration of Algorithm 1 for all replicas, after their backward passes.
        Returns True if a global update happened in this call."""
        self._check_bound()
        lr = self.lr if lr is None else float(lr)
        cur = torch.cuda.current_stream(self.device)
        self.main.wait_stream(cur)                  # gradients are complete before the update reads them
        fired = False
        if not self._started:                       # steps 2-5: first update, send, start the All-Reduce
            self.ctx.local_step(lr)
            self.ctx.snapshot()
            self.ctx.average()
            self._started = True
            self.tau = 0
        else:                                       # steps 6-9
            self.tau += 1
            if self.tau >= self.m:
                self.ctx.step_merge(lr, True)
                self.ctx.average()
                self.tau, self.t, fired = 0, self.t + 1, True
            else:
                self.ctx.local_step(lr)
        cur.wait_stream(self.main)                  # the next forward sees the new parameters
        return fired

    def center(self) -> torch.Tensor:
        """The current mean model z (flat, fp32), e.g. for evaluation."""
        import numpy as np
        return torch.from_numpy(np.ascontiguousarray(self.ctx.read_state(B.STATE_Z)))

    def close(self) -> None:
        self.ctx.close()
