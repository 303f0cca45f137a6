"""Seeded synthetic weight sets for the five PWLQ workloads.

This module only draws numbers and lists tensor shapes.  It holds none of the
quantizer's arithmetic and imports neither the HIP binding nor the CPU oracle,
so both sides can be fed the same bytes.

The paper evaluates on torchvision's pretrained Inception-v3, ResNet-50 and
MobileNet-v2 (Section 5.1); those weights are not available here, so each
workload takes the *shapes* of the network's conv / FC weights (BN folded, no
biases: Section 5) and bell-shaped or long-tailed *values* of the kind the
paper describes (Section 1, Section 3.1).

Seeding: workload 1 uses ``numpy.random.default_rng(0)``; workloads 2-5 draw
tensor ``t`` from ``default_rng([0, workload, t])`` so any single tensor can
be regenerated on its own.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Sequence, Tuple

import numpy as np

PER_CHANNEL = 0
PER_TENSOR = 1

Shape = Tuple[int, ...]


# --------------------------------------------------------------------------
# shape tables (architecture facts; conv weights are [Cout, Cin/groups, kh, kw])
# --------------------------------------------------------------------------
def resnet50_shapes() -> List[Shape]:
    shapes: List[Shape] = [(64, 3, 7, 7)]
    cin = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(blocks):
            shapes.append((planes, cin, 1, 1))
            shapes.append((planes, planes, 3, 3))
            shapes.append((4 * planes, planes, 1, 1))
            if blk == 0:
                shapes.append((4 * planes, cin, 1, 1))  # projection shortcut
            cin = 4 * planes
    shapes.append((1000, 2048))
    return shapes


def mobilenetv2_shapes() -> List[Shape]:
    shapes: List[Shape] = [(32, 3, 3, 3)]
    cin = 32
    for t, c, n in ((1, 16, 1), (6, 24, 2), (6, 32, 3), (6, 64, 4),
                    (6, 96, 3), (6, 160, 3), (6, 320, 1)):
        for _ in range(n):
            hidden = cin * t
            if t != 1:
                shapes.append((hidden, cin, 1, 1))      # expand
            shapes.append((hidden, 1, 3, 3))            # depthwise
            shapes.append((c, hidden, 1, 1))            # project
            cin = c
    shapes.append((1280, 320, 1, 1))
    shapes.append((1000, 1280))
    return shapes


def inceptionv3_shapes() -> List[Shape]:
    """Main trunk only (the auxiliary classifier is not part of inference)."""
    s: List[Shape] = [(32, 3, 3, 3), (32, 32, 3, 3), (64, 32, 3, 3),
                      (80, 64, 1, 1), (192, 80, 3, 3)]
    for cin, proj in ((192, 32), (256, 64), (288, 64)):          # "A" modules
        s += [(64, cin, 1, 1),
              (48, cin, 1, 1), (64, 48, 5, 5),
              (64, cin, 1, 1), (96, 64, 3, 3), (96, 96, 3, 3),
              (proj, cin, 1, 1)]
    s += [(384, 288, 3, 3),                                       # "B" reduction
          (64, 288, 1, 1), (96, 64, 3, 3), (96, 96, 3, 3)]
    for c7 in (128, 160, 160, 192):                               # "C" modules
        s += [(192, 768, 1, 1),
              (c7, 768, 1, 1), (c7, c7, 1, 7), (192, c7, 7, 1),
              (c7, 768, 1, 1), (c7, c7, 7, 1), (c7, c7, 1, 7),
              (c7, c7, 7, 1), (192, c7, 1, 7),
              (192, 768, 1, 1)]
    s += [(192, 768, 1, 1), (320, 192, 3, 3),                     # "D" reduction
          (192, 768, 1, 1), (192, 192, 1, 7), (192, 192, 7, 1), (192, 192, 3, 3)]
    for cin in (1280, 2048):                                      # "E" modules
        s += [(320, cin, 1, 1),
              (384, cin, 1, 1), (384, 384, 1, 3), (384, 384, 3, 1),
              (448, cin, 1, 1), (384, 448, 3, 3), (384, 384, 1, 3), (384, 384, 3, 1),
              (192, cin, 1, 1)]
    s.append((1000, 2048))
    return s


def transformer_shapes() -> List[Shape]:
    return [(4096, 4096)] * 4 + [(11008, 4096)] * 2


def as_ck(shape: Sequence[int]) -> Tuple[int, int]:
    """[Cout, ...] -> (C, K): one row per output channel."""
    c = int(shape[0])
    k = 1
    for d in shape[1:]:
        k *= int(d)
    return c, k


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    shapes: Tuple[Shape, ...]
    mode: int
    bits: int
    n_cand: int
    dist: str

    @property
    def n_tensors(self) -> int:
        return len(self.shapes)

    def ck(self, t: int) -> Tuple[int, int]:
        return as_ck(self.shapes[t])

    @property
    def n_elements(self) -> int:
        return sum(c * k for c, k in map(as_ck, self.shapes))

    @property
    def n_groups(self) -> int:
        if self.mode == PER_TENSOR:
            return len(self.shapes)
        return sum(as_ck(s)[0] for s in self.shapes)

    @property
    def n_evals(self) -> int:
        return self.n_elements * self.n_cand

    def tensor(self, t: int) -> np.ndarray:
        """fp32 [C, K] array of tensor ``t``, regenerated from its own seed."""
        c, k = self.ck(t)
        return _draw(self, t, c, k)

    def tensors(self) -> Iterator[np.ndarray]:
        for t in range(self.n_tensors):
            yield self.tensor(t)


def _draw(wl: Workload, t: int, c: int, k: int) -> np.ndarray:
    if wl.index == 1:
        rng = np.random.default_rng(0)
        return rng.laplace(0.0, 0.05, size=(c, k)).astype(np.float32)
    rng = np.random.default_rng([0, wl.index, t])
    if wl.dist == "gauss_lognormal":
        sigma = np.exp(rng.normal(-3.0, 0.5, size=(c, 1)))
        return (sigma * rng.standard_normal(size=(c, k))).astype(np.float32)
    if wl.dist == "laplace_lognormal":
        beta = np.exp(rng.normal(-3.0, 0.5, size=(c, 1)))
        return (beta * rng.laplace(0.0, 1.0, size=(c, k))).astype(np.float32)
    if wl.dist == "student_t3":
        return (0.02 * rng.standard_t(3.0, size=(c, k))).astype(np.float32)
    if wl.dist == "laplace_outliers":
        w = rng.laplace(0.0, 0.02, size=(c, k))
        hit = rng.random(size=(c, k)) < 0.001
        w[hit] *= 10.0
        return w.astype(np.float32)
    raise ValueError(wl.dist)


def workload(index: int) -> Workload:
    if index == 1:
        return Workload(1, "conv64x64x3x3_laplace", ((64, 64, 3, 3),),
                        PER_CHANNEL, 4, 100, "laplace")
    if index == 2:
        return Workload(2, "resnet50_shapes_gauss", tuple(resnet50_shapes()),
                        PER_CHANNEL, 4, 1000, "gauss_lognormal")
    if index == 3:
        return Workload(3, "mobilenetv2_shapes_laplace", tuple(mobilenetv2_shapes()),
                        PER_CHANNEL, 4, 1000, "laplace_lognormal")
    if index == 4:
        return Workload(4, "inceptionv3_shapes_student_t", tuple(inceptionv3_shapes()),
                        PER_TENSOR, 3, 2000, "student_t3")
    if index == 5:
        return Workload(5, "transformer_linears_laplace_outliers",
                        tuple(transformer_shapes()), PER_CHANNEL, 4, 1000,
                        "laplace_outliers")
    raise ValueError("workload index must be 1..5")
