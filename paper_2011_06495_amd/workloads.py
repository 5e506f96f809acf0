"""Seeded synthetic inputs for the vote step.

This module only draws numbers; it contains none of the method's arithmetic
(no top-K, no votes, no masks) and is the one module that both the CPU oracle's
tests and the HIP path's tests / benchmark may share.

The paper trains ResNet-18 (11,173,962 parameters) on CIFAR-10 with N = 10
workers and sparsity phi in [1e-3, 1e-2] (Sec. 4.1, Sec. 4.2).  Neither the
dataset nor trained weights are available here, so the five workloads below
stand in for the per-iteration model differences: flat vectors with the
per-layer block structure of ResNet-18 / ResNet-50, per-block scales spread
over decades, and a common component shared by all workers so that their
top-K sets overlap as those of real workers do.

Every row is generated from its own PCG64 stream keyed by
(workload, step, worker), so single rows can be regenerated independently.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20110649


# ------------------------------------------------------------------ layouts

def resnet18_cifar_blocks() -> Tuple[int, ...]:
    """Parameter-tensor sizes of a ResNet-18 with a 3x3 stem and 10 classes
    (conv weight, bn weight, bn bias per conv; 1x1 projection at each stage
    change).  Sums to the 11,173,962 parameters of Sec. 4.1."""
    b = [3 * 3 * 3 * 64, 64, 64]
    for _ in range(2):
        b += [9 * 64 * 64, 64, 64, 9 * 64 * 64, 64, 64]
    for w in (128, 256, 512):
        h = w // 2
        b += [9 * h * w, w, w, 9 * w * w, w, w, h * w, w, w]
        b += [9 * w * w, w, w, 9 * w * w, w, w]
    b += [512 * 10, 10]
    return tuple(b)


def resnet50_imagenet_blocks() -> Tuple[int, ...]:
    """Parameter-tensor sizes of a ResNet-50 with a 7x7 stem and 1000 classes."""
    b = [7 * 7 * 3 * 64, 64, 64]
    cin = 64
    for w, nblocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for i in range(nblocks):
            b += [cin * w, w, w, 9 * w * w, w, w, w * 4 * w, 4 * w, 4 * w]
            if i == 0:
                b += [cin * 4 * w, 4 * w, 4 * w]
            cin = 4 * w
    b += [2048 * 1000, 1000]
    return tuple(b)


def _rescale_blocks(blocks: Tuple[int, ...], d: int) -> Tuple[int, ...]:
    """Same layout squeezed into d coordinates (block edges at proportional
    positions; empty blocks dropped)."""
    total = sum(blocks)
    if d == total:
        return blocks
    edges = np.concatenate([[0], np.cumsum(blocks)]).astype(np.float64)
    new_edges = np.floor(edges * (d / total) + 0.5).astype(np.int64)
    new_edges[-1] = d
    sizes = np.diff(new_edges)
    return tuple(int(s) for s in sizes if s > 0)


# ------------------------------------------------------------------ workloads

@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    d: int
    K: int
    steps: int
    grad_dtype: str            # "f32" or "bf16"
    kind: str                  # "lognormal", "blocks_normal", "blocks_t3", "blocks_lattice"
    blocks: Tuple[int, ...]    # contiguous block sizes, sum == d (empty for "lognormal")
    scale_decades: Tuple[float, float]  # block scale = 10**U(lo, hi)
    w_common: float            # weight of the component shared by all workers
    w_own: float               # weight of the worker's own component
    index: int                 # position in the benchmark's configs
    seed: int = BASE_SEED
    # "blocks_lattice" only: magnitudes are l * 2**-lattice_shift, l in 0..255, so
    # sums of lattice values stay exactly representable and ties persist over steps
    lattice_shift: int = 9

    @property
    def phi(self) -> float:
        return self.K / self.d

    def with_size(self, d: int, K: Optional[int] = None, N: Optional[int] = None,
                  steps: Optional[int] = None, lattice_shift: Optional[int] = None) -> "Workload":
        """Same recipe at a reduced size (for parity cases the oracle finishes
        in seconds).  K keeps the sparsity ratio unless given.  A reduced lattice
        workload takes a coarser lattice (smaller shift) to keep its boundary tie
        groups as heavy, relative to K, as at full size."""
        K_new = K if K is not None else max(1, int(round(self.phi * d)))
        return replace(self, d=d, K=K_new, N=N if N is not None else self.N,
                       steps=steps if steps is not None else self.steps,
                       lattice_shift=lattice_shift if lattice_shift is not None else self.lattice_shift,
                       blocks=_rescale_blocks(self.blocks, d) if self.blocks else ())


_R18 = resnet18_cifar_blocks()
_R50 = resnet50_imagenet_blocks()
D_R18 = sum(_R18)
D_R50 = sum(_R50)

C1 = Workload("C1", 4, 1 << 20, 10486, 1, "f32", "lognormal", (), (0.0, 0.0), 0.5, 0.866, 0)
C2 = Workload("C2", 10, D_R18, 11174, 1, "f32", "blocks_normal", _R18, (-3.0, -1.0),
              0.5 ** 0.5, 0.5 ** 0.5, 1)
C3 = Workload("C3", 16, D_R18, 2793, 20, "f32", "blocks_t3", _R18, (-3.0, -1.0), 0.3, 0.95, 2)
C4 = Workload("C4", 16, D_R18, 11174, 5, "f32", "blocks_lattice", _R18, (-3.0, -1.0),
              0.5 ** 0.5, 0.5 ** 0.5, 3)
C5 = Workload("C5", 32, D_R50, 25557, 10, "bf16", "blocks_normal", _R50, (-4.0, -1.0),
              0.5 ** 0.5, 0.5 ** 0.5, 4)

WORKLOADS = {w.name: w for w in (C1, C2, C3, C4, C5)}

LATTICE_LEVELS = 256


def _rng(w: Workload, step: int, stream: int) -> np.random.Generator:
    # stream: -2 = scales, -1 = common component, n >= 0 = worker n, 1000000 = selection clocks
    return np.random.Generator(np.random.PCG64([w.seed, 1000 * w.index + step, stream + 2]))


def coordinate_scale(w: Workload) -> np.ndarray:
    """Per-coordinate scale shared by all workers and all steps (fp32, length d)."""
    rng = _rng(w, 0, -2)
    if w.kind == "lognormal":
        return np.exp(rng.standard_normal(w.d, dtype=np.float32)).astype(np.float32)
    lo, hi = w.scale_decades
    per_block = (10.0 ** rng.uniform(lo, hi, size=len(w.blocks))).astype(np.float32)
    return np.repeat(per_block, np.asarray(w.blocks, dtype=np.int64))


def _draw(w: Workload, rng: np.random.Generator) -> np.ndarray:
    if w.kind == "blocks_t3":
        return rng.standard_t(3.0, size=w.d).astype(np.float32)
    return rng.standard_normal(w.d, dtype=np.float32)


def common_component(w: Workload, step: int) -> np.ndarray:
    return _draw(w, _rng(w, step, -1))


def _to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (inputs are finite)."""
    u = x.view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def gradient_row(w: Workload, step: int, n: int, common: Optional[np.ndarray] = None,
                 scale: Optional[np.ndarray] = None) -> np.ndarray:
    """Row n of the step's gradient matrix: float32, or uint16 bf16 patterns."""
    if common is None:
        common = common_component(w, step)
    if scale is None:
        scale = coordinate_scale(w)
    own = _draw(w, _rng(w, step, n))
    g = (np.float32(w.w_common) * common + np.float32(w.w_own) * own) * scale
    if w.kind == "blocks_lattice":
        q = np.float32(2.0 ** w.lattice_shift)
        level = np.minimum(np.rint(np.abs(g) * q), np.float32(LATTICE_LEVELS - 1))
        g = (np.sign(g) * level / q).astype(np.float32)
    g = np.ascontiguousarray(g, dtype=np.float32)
    if w.grad_dtype == "bf16":
        return _to_bf16_bits(g)
    return g


def gradients(w: Workload, step: int, threads: int = 1) -> np.ndarray:
    """N x d gradient matrix of one step (float32, or uint16 holding bf16).
    threads > 1 draws the rows concurrently (same bytes: every row has its own stream)."""
    common = common_component(w, step)
    scale = coordinate_scale(w)
    out = np.empty((w.N, w.d), np.uint16 if w.grad_dtype == "bf16" else np.float32)

    def one(n: int) -> None:
        out[n] = gradient_row(w, step, n, common, scale)

    if threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(one, range(w.N)))
    else:
        for n in range(w.N):
            one(n)
    return out


def selection_clocks(w: Workload, step: int) -> np.ndarray:
    """The d Exp(1) numbers (fp32) that majority voting with random selection consumes
    in one step: plain random draws from a stream of their own."""
    return _rng(w, step, 1_000_000).standard_exponential(w.d, dtype=np.float32)


def zero_error(w: Workload) -> np.ndarray:
    """The error buffers start at zero (Algorithm 1 carries e from step to step)."""
    return np.zeros((w.N, w.d), np.float32)
