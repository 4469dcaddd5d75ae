"""Seeded synthetic workloads: parameter-list shapes and host-side random inputs.

This module holds no arithmetic of the method.  It only (a) lists tensor shapes of the
model families the paper trains (ResNet-50/101, ViT-B/16, PyramidNet; Sec. 6 and the
experiment details in the appendix) so that the per-layer size mix is realistic, and
(b) draws the random numbers (initial point, per-worker spread, per-step gradients) with
numpy's PCG64 generator.  Both the CPU oracle's tests and the GPU path's tests/benchmarks
consume the arrays produced here; neither side's code is used.

Every random array is a flat float32 vector of length d (the tensor list concatenated in
list order) with its own stream, addressed by a spawn key under SeedSequence(seed):
  (0,)        the M log-uniform worker spreads sigma_m (heterogeneous workloads only)
  (1,)        x0 ~ N(0, sigma_x0^2)
  (2, m)      worker m's offset: x_m = x0 + N(0, sigma_m^2)
  (3, k, m)   worker m's gradient at local step k ~ N(0, sigma_grad^2)
A vector is cut into 8 equal segments, each filled from the stream (key..., segment), so the
values do not depend on how many threads do the filling.  Momentum buffers start at zero.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]


def _bn(c: int) -> List[Shape]:
    return [(c,), (c,)]


def resnet_bottleneck_shapes(stage_blocks: Sequence[int]) -> List[Shape]:
    """ImageNet bottleneck ResNet parameter list (ResNet-50: [3,4,6,3]; -101: [3,4,23,3])."""
    shapes: List[Shape] = [(64, 3, 7, 7)] + _bn(64)
    cin = 64
    for nblocks, width in zip(stage_blocks, (64, 128, 256, 512)):
        for b in range(nblocks):
            shapes += [(width, cin, 1, 1)] + _bn(width)
            shapes += [(width, width, 3, 3)] + _bn(width)
            shapes += [(4 * width, width, 1, 1)] + _bn(4 * width)
            if b == 0:  # projection shortcut on the first block of a stage
                shapes += [(4 * width, cin, 1, 1)] + _bn(4 * width)
            cin = 4 * width
    shapes += [(1000, 2048), (1000,)]
    return shapes


def vit_b16_shapes() -> List[Shape]:
    """ViT-B/16 (768 wide, 12 blocks, MLP 3072, 224x224 input, 1000 classes)."""
    shapes: List[Shape] = [(1, 1, 768), (1, 197, 768), (768, 3, 16, 16), (768,)]
    for _ in range(12):
        shapes += [(768,), (768,), (2304, 768), (2304,), (768, 768), (768,)]
        shapes += [(768,), (768,), (3072, 768), (3072,), (768, 3072), (768,)]
    shapes += [(768,), (768,), (1000, 768), (1000,)]
    return shapes


def pyramidnet_like_shapes() -> List[Shape]:
    """A PyramidNet-style CIFAR-100 list: 3 stages x 18 basic blocks whose width grows
    linearly from 16 to 272.  A look-alike with ~26 M parameters in 331 mostly small
    tensors, many with a size that is not a multiple of 4."""
    shapes: List[Shape] = [(16, 3, 3, 3)] + _bn(16)
    width = 16.0
    cin = 16
    for _stage in range(3):
        for _block in range(18):
            width += 256.0 / 54.0
            cout = int(round(width))
            shapes += _bn(cin) + [(cout, cin, 3, 3)] + _bn(cout) + [(cout, cout, 3, 3)]
            cin = cout
    shapes += _bn(cin) + [(100, cin), (100,)]
    return shapes


@dataclass(frozen=True)
class WorkloadSpec:
    """One benchmark/parity configuration (everything except the random numbers)."""
    name: str
    M: int
    shapes: Tuple[Shape, ...]
    seed: int
    sigma_x0: float = 0.02
    sigma_worker: float = 1e-3          # ignored when hetero_spread is True
    hetero_spread: bool = False         # sigma_m = 10**U(-4,-2), one per worker
    sigma_grad: float = 1e-2
    tau: int = 1                        # local steps before the round
    pull: float = 0.1                   # alpha
    push: float = 0.01                  # lambda
    lr: float = 0.1                     # eta
    momentum: float = 0.9
    weight_decay: float = 0.0
    sweep: Tuple[Tuple[float, float], ...] = ()   # extra (pull, push) pairs to run

    @property
    def numel(self) -> Tuple[int, ...]:
        return tuple(int(np.prod(s, dtype=np.int64)) for s in self.shapes)

    @property
    def d(self) -> int:
        return int(sum(self.numel))

    @property
    def T(self) -> int:
        return len(self.shapes)


def _spec_table() -> dict:
    rn50 = tuple(resnet_bottleneck_shapes((3, 4, 6, 3)))
    rn101 = tuple(resnet_bottleneck_shapes((3, 4, 23, 3)))
    vit = tuple(vit_b16_shapes())
    pyr = tuple(pyramidnet_like_shapes())
    specs = [
        WorkloadSpec("flat1m_M2", 2, ((1_000_000,),), seed=0, tau=1),
        WorkloadSpec("resnet50_M4", 4, rn50, seed=1, tau=8),
        WorkloadSpec("resnet101_M4", 4, rn101, seed=2, tau=16,
                     sweep=((0.05, 0.005), (0.05, 0.02), (0.1, 0.005), (0.1, 0.02))),
        WorkloadSpec("vitb16_M4", 4, vit, seed=3, tau=1, sigma_worker=5e-3),
        WorkloadSpec("pyramidnet_M8", 8, pyr, seed=4, tau=4, hetero_spread=True),
    ]
    return {s.name: s for s in specs}


SPECS = _spec_table()
EXPECTED_SIZES = {           # (T, d) of each list; checked by the CPU tests
    "flat1m_M2": (1, 1_000_000),
    "resnet50_M4": (161, 25_557_032),
    "resnet101_M4": (314, 44_549_160),
    "vitb16_M4": (152, 86_567_656),
    "pyramidnet_M8": (331, 25_857_192),
}


def small_spec(name: str = "small_ragged", M: int = 4, seed: int = 7, tau: int = 2,
               shapes: Sequence[Shape] = ((3,), (1,), (4097,), (64, 9), (130, 3, 3), (5,),
                                          (2,), (33000,), (7, 11), (12288,)),
               **kw) -> WorkloadSpec:
    """A small list with ragged sizes (several < 4, several not multiples of 4, a few that
    span multiple tiles) for quick element-by-element parity."""
    return WorkloadSpec(name, M, tuple(tuple(s) for s in shapes), seed=seed, tau=tau, **kw)


_SEGMENTS = 8


def _normal_vector(seed: int, key: Tuple[int, ...], n: int) -> np.ndarray:
    """n standard normals (float32) from the streams (key..., 0..7)."""
    out = np.empty(n, dtype=np.float32)
    bounds = [(n * s) // _SEGMENTS for s in range(_SEGMENTS + 1)]

    def fill(seg: int) -> None:
        a, b = bounds[seg], bounds[seg + 1]
        if b > a:
            ss = np.random.SeedSequence(entropy=seed, spawn_key=tuple(key) + (seg,))
            np.random.Generator(np.random.PCG64(ss)).standard_normal(out=out[a:b], dtype=np.float32)

    if n >= (1 << 20):
        with ThreadPoolExecutor(_SEGMENTS) as pool:
            list(pool.map(fill, range(_SEGMENTS)))
    else:
        for seg in range(_SEGMENTS):
            fill(seg)
    return out


@dataclass
class HostInputs:
    """Host arrays for one workload.  x[m] and v[m] are flat float32 vectors of length d
    (the tensor list concatenated in list order); ``offsets[t]`` is where tensor t starts."""
    spec: WorkloadSpec
    x: List[np.ndarray]
    v: List[np.ndarray]
    offsets: np.ndarray
    sigma_m: np.ndarray

    def grads(self, step: int) -> List[np.ndarray]:
        """The gradients of local step `step` (0-based), one flat vector per worker."""
        spec = self.spec
        out = []
        for m in range(spec.M):
            g = _normal_vector(spec.seed, (3, step, m), spec.d)
            g *= np.float32(spec.sigma_grad)
            out.append(g)
        return out

    def tensor_views(self, flat: np.ndarray) -> List[np.ndarray]:
        o = self.offsets
        return [flat[o[t]:o[t + 1]] for t in range(len(o) - 1)]


def make_inputs(spec: WorkloadSpec) -> HostInputs:
    offsets = np.zeros(spec.T + 1, dtype=np.int64)
    np.cumsum(np.asarray(spec.numel, dtype=np.int64), out=offsets[1:])
    d = spec.d
    if spec.hetero_spread:
        ss = np.random.SeedSequence(entropy=spec.seed, spawn_key=(0,))
        u = np.random.Generator(np.random.PCG64(ss)).uniform(-4.0, -2.0, size=spec.M)
        sigma_m = (10.0 ** u).astype(np.float32)
    else:
        sigma_m = np.full(spec.M, spec.sigma_worker, dtype=np.float32)
    x0 = _normal_vector(spec.seed, (1,), d)
    x0 *= np.float32(spec.sigma_x0)
    xs, vs = [], []
    for m in range(spec.M):
        noise = _normal_vector(spec.seed, (2, m), d)
        noise *= sigma_m[m]
        noise += x0
        xs.append(noise)
        vs.append(np.zeros(d, dtype=np.float32))
    return HostInputs(spec, xs, vs, offsets, sigma_m)
