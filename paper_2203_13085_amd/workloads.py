"""Seeded synthetic workloads: parameter-shape lists and input generators.

This module holds none of the method's arithmetic.  It only produces the
inputs both the CPU oracle and the HIP path consume: parameter shapes of the
networks the paper trains or cites (Sec. 5.1.1: ResNet-50; Sec. 1: MobileNetV2),
initial weights and per-step gradients.  Every array is a pure function of
(seed, step, replica, tensor), drawn from a counter-based Philox stream, so the
two sides can regenerate identical bits independently and at any subset.

Shape lists are produced by rule from the published architectures, never read
from a model library.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]


# --------------------------------------------------------------------------
# shape lists
# --------------------------------------------------------------------------
def _bn(c: int) -> List[Tuple[str, Shape]]:
    return [("bn_gamma", (c,)), ("bn_beta", (c,))]


def _conv(cout: int, cin: int, k: int) -> Tuple[str, Shape]:
    return ("conv", (cout, cin, k, k))


def resnet_shapes(depth: int) -> List[Tuple[str, Shape]]:
    """Trainable tensors of an ImageNet ResNet-18 or ResNet-50, in module order.

    Stem 7x7 conv + BN, four stages of planes 64/128/256/512, a projection
    shortcut wherever the block input and output widths differ, a 1000-way
    classifier.  Convolutions carry no bias; BN running statistics are buffers,
    not parameters, and are left out.
    """
    if depth == 18:
        blocks, bottleneck = (2, 2, 2, 2), False
    elif depth == 50:
        blocks, bottleneck = (3, 4, 6, 3), True
    else:
        raise ValueError("depth must be 18 or 50")
    out: List[Tuple[str, Shape]] = [_conv(64, 3, 7)] + _bn(64)
    width = 64
    for stage, nblk in enumerate(blocks):
        p = 64 << stage
        wout = 4 * p if bottleneck else p
        for b in range(nblk):
            if bottleneck:
                out += [_conv(p, width, 1)] + _bn(p)
                out += [_conv(p, p, 3)] + _bn(p)
                out += [_conv(wout, p, 1)] + _bn(wout)
            else:
                out += [_conv(p, width, 3)] + _bn(p)
                out += [_conv(p, p, 3)] + _bn(p)
            if b == 0 and width != wout:
                out += [_conv(wout, width, 1)] + _bn(wout)
            width = wout
    out += [("fc_weight", (1000, width)), ("fc_bias", (1000,))]
    return out


def mobilenet_v2_shapes() -> List[Tuple[str, Shape]]:
    """Trainable tensors of MobileNetV2 (width 1.0, 1000 classes), module order."""
    out: List[Tuple[str, Shape]] = [_conv(32, 3, 3)] + _bn(32)
    width = 32
    for t, c, n in ((1, 16, 1), (6, 24, 2), (6, 32, 3), (6, 64, 4),
                    (6, 96, 3), (6, 160, 3), (6, 320, 1)):
        for _ in range(n):
            hidden = t * width
            if t != 1:
                out += [_conv(hidden, width, 1)] + _bn(hidden)
            out += [("dwconv", (hidden, 1, 3, 3))] + _bn(hidden)
            out += [_conv(c, hidden, 1)] + _bn(c)
            width = c
    out += [_conv(1280, width, 1)] + _bn(1280)
    out += [("fc_weight", (1000, 1280)), ("fc_bias", (1000,))]
    return out


def numel(shape: Shape) -> int:
    return int(np.prod(shape, dtype=np.int64))


# --------------------------------------------------------------------------
# configurations (the five synthetic workloads this build is measured on)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    K: int                       # replicas resident on the GPU (the paper's P nodes)
    tensors: Tuple[Tuple[str, Shape], ...]
    lr: float
    momentum: float = 0.9
    weight_decay: float = 1e-4
    nesterov: bool = True
    m: int = 1                   # local steps per merge (fixed cadence, tau_max)
    T: int = 3                   # loop iterations for parity runs
    storage: str = "f32"         # "f32" | "bf16" (dtype of user-visible params/grads)
    init: str = "he"             # "he" | "flat"
    seed: int = 0
    side_stream: bool = False

    @property
    def numels(self) -> List[int]:
        return [numel(s) for _, s in self.tensors]

    @property
    def N(self) -> int:
        return sum(self.numels)


def config(index: int) -> Workload:
    """The benchmark configurations, by position in the baseline's list."""
    if index == 0:
        return Workload("flat-1M-K4", 4, (("flat", (1 << 20,)),), lr=0.1, m=2, T=10,
                        init="flat", seed=0)
    if index == 1:
        return Workload("resnet18-K8", 8, tuple(resnet_shapes(18)), lr=0.4, m=4, T=12)
    if index == 2:
        return Workload("resnet50-K8", 8, tuple(resnet_shapes(50)), lr=0.8, m=4, T=12,
                        side_stream=True)
    if index == 3:
        return Workload("mobilenetv2-K16", 16, tuple(mobilenet_v2_shapes()), lr=0.4, m=1, T=3)
    if index == 4:
        return Workload("resnet50-bf16-K32", 32, tuple(resnet_shapes(50)), lr=0.8, m=8, T=24,
                        storage="bf16", side_stream=True)
    raise IndexError(index)


def small(K: int = 3, numels: Sequence[int] = (5, 1024, 1, 4099, 260, 64), **kw) -> Workload:
    """A ragged little list for parity tests: odd sizes, scalar tails, several tiles."""
    tensors = tuple(("conv" if i % 2 else "bn_beta", (int(n),)) for i, n in enumerate(numels))
    base = dict(lr=0.05, m=2, T=6, init="flat", seed=7)
    base.update(kw)
    return Workload("small", K, tensors, **base)


# --------------------------------------------------------------------------
# seeded values
# --------------------------------------------------------------------------
_STREAM_INIT = 0
_STREAM_GRAD = 1


def _rng(seed: int, stream: int, step: int, replica: int, tensor: int) -> np.random.Generator:
    # Philox-4x64: the 128-bit key carries (seed, stream), the counter's upper
    # words carry (step, replica, tensor); word 0 counts the draws.
    bits = np.random.Philox(key=np.array([seed, stream], dtype=np.uint64),
                            counter=np.array([0, step, replica, tensor], dtype=np.uint64))
    return np.random.Generator(bits)


def init_std(kind: str, shape: Shape, mode: str) -> float | None:
    """Standard deviation of the initial draw; None means a constant tensor."""
    if mode == "flat":
        return 0.01
    if kind in ("conv", "dwconv"):
        fan_in = shape[1] * shape[2] * shape[3]
        return math.sqrt(2.0 / fan_in)
    if kind == "fc_weight":
        return math.sqrt(2.0 / shape[1])
    return None


def initial_tensor(w: Workload, tensor: int) -> np.ndarray:
    """x_0 for one tensor, flat fp32.  One draw, shared by all K replicas
    (every node starts from the same model, Sec. 4)."""
    kind, shape = w.tensors[tensor]
    n = numel(shape)
    std = init_std(kind, shape, w.init)
    if std is None:
        const = 1.0 if kind == "bn_gamma" else 0.0
        return np.full(n, const, dtype=np.float32)
    r = _rng(w.seed, _STREAM_INIT, 0, 0, tensor)
    return (r.standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float32)


def gradient_tensor(w: Workload, step: int, replica: int, tensor: int,
                    std: float = 1e-3) -> np.ndarray:
    """Synthetic mini-batch gradient for (step, replica, tensor), flat fp32,
    N(0, std^2); step 0 is the prologue's gradient."""
    n = w.numels[tensor]
    r = _rng(w.seed, _STREAM_GRAD, step, replica, tensor)
    return (r.standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Input preparation only: round fp32 inputs to bf16 (nearest-even) and
    return the 16-bit patterns.  Uses the library conversion of torch on CPU,
    so that neither the oracle's nor the kernels' own rounding code is involved
    in making inputs."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32 (a shift, no rounding)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
