"""Seeded synthetic inputs: layer sets, gradients and weights.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the optimizer's arithmetic: it only describes layer sets and draws
random inputs.

The layer sets follow the Llama sizes of the paper's pre-training experiment
(Sec. 3.1, Table 1: rank / d_model per model size); the paper's training data
is not available, so gradients are synthetic: for every matrix a fixed factor
A (m x k) ~ N(0, 1/k) drawn once, and per step a fresh B (n x k) ~ N(0, 1/k) and
noise E ~ N(0, 1):  G = A B^T + noise * E.  The fixed A gives the slowly moving
low-rank structure GaLore relies on (Sec. 1), the fresh B distinct mini-batch
gradients.  ``collinear=True`` keeps B fixed too (a nearly collinear history:
a stress case for the s x s system).  Weights are N(0, 0.02^2).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class LayerSetConfig:
    name: str
    shapes: Tuple[Tuple[int, int, int], ...]   # (m, n, multiplicity per block)
    blocks: int
    r: int
    s: int
    k: int            # rank of the synthetic low-rank factor
    noise: float
    dtype: str        # "f32" | "bf16" (gradient and weight storage type)
    seed: int
    lam: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    lr: float = 1e-3
    refresh_every: int = 200

    def matrices(self) -> List[Tuple[int, int]]:
        """(m, n) of every matrix, block after block."""
        out = []
        for _ in range(self.blocks):
            for (m, n, mult) in self.shapes:
                out.extend([(m, n)] * mult)
        return out

    def distinct_shapes(self) -> List[Tuple[int, int, int]]:
        """(m, n, total multiplicity) per distinct shape."""
        return [(m, n, mult * self.blocks) for (m, n, mult) in self.shapes]


def _llama(name, d, ff, blocks, r, s, k, seed):
    return LayerSetConfig(
        name=name, shapes=((d, d, 4), (d, ff, 2), (ff, d, 1)), blocks=blocks,
        r=r, s=s, k=k, noise=0.01, dtype="bf16", seed=seed)


CONFIGS = {
    "c1": LayerSetConfig(name="single-256x512-f32", shapes=((256, 512, 1),), blocks=1,
                         r=32, s=4, k=32, noise=0.01, dtype="f32", seed=0),
    "c2": _llama("llama-60m", 512, 1376, 8, 128, 8, 64, 1),
    "c3": _llama("llama-130m", 768, 2048, 12, 256, 8, 64, 2),
    "c4": _llama("llama-350m", 1024, 2736, 24, 256, 16, 64, 3),
    "c5": _llama("llama-1.1b", 2048, 5461, 24, 512, 16, 128, 4),
    # Fine-tuning-shaped sets (paper Sec. 3.2: RoBERTa-Base, ranks 4 and 8, learning rate from its
    # grid): 12 blocks x {4 attention 768x768, 768x3072, 3072x768}.  Ranks far below an MFMA tile:
    # both GEMMs are pure bandwidth here.
    "ft4": LayerSetConfig(name="roberta-base-rank4", shapes=((768, 768, 4), (768, 3072, 1), (3072, 768, 1)),
                          blocks=12, r=4, s=4, k=8, noise=0.01, dtype="bf16", seed=5, lr=2e-5),
    "ft8": LayerSetConfig(name="roberta-base-rank8", shapes=((768, 768, 4), (768, 3072, 1), (3072, 768, 1)),
                          blocks=12, r=8, s=4, k=8, noise=0.01, dtype="bf16", seed=6, lr=2e-5),
}


# --------------------------------------------------------------------------
# numpy generator (host): used for the small fp32 configuration and CPU tests
# --------------------------------------------------------------------------
class NumpyGradientStream:
    """Draw order: A once, then (B, E) per step, from numpy.random.default_rng(seed)."""

    def __init__(self, m: int, n: int, k: int, noise: float, seed: int, collinear: bool = False):
        self.m, self.n, self.k, self.noise = m, n, k, noise
        self.rng = np.random.default_rng(seed)
        self.A = self.rng.normal(0.0, 1.0 / np.sqrt(k), size=(m, k))
        self.collinear = collinear
        self._B = None

    def next(self) -> np.ndarray:
        if self._B is None or not self.collinear:
            self._B = self.rng.normal(0.0, 1.0 / np.sqrt(self.k), size=(self.n, self.k))
        E = self.rng.normal(0.0, 1.0, size=(self.m, self.n))
        return self.A @ self._B.T + self.noise * E


def numpy_weight(m: int, n: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed + 7919).normal(0.0, 0.02, size=(m, n))


# --------------------------------------------------------------------------
# torch generator (host or device): used for the bf16 layer sets
# --------------------------------------------------------------------------
class TorchGradientStream:
    """Per-matrix fixed A, per-call fresh (B, E); one seeded torch generator.

    ``next_set()`` returns one gradient per matrix of the layer set, in the
    storage dtype, on ``device``.  The oracle is fed the very same bytes
    (downloaded), never a re-generation.
    """

    def __init__(self, mats, k: int, noise: float, seed: int, dtype: str, device,
                 collinear: bool = False):
        import torch
        self.torch = torch
        self.mats = list(mats)
        self.k, self.noise = k, noise
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(seed)
        self.dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
        self.collinear = collinear
        sd = 1.0 / float(np.sqrt(k))
        self.A = [self._randn(m, k) * sd for (m, _) in self.mats]
        self._B = None

    def _randn(self, a, b):
        return self.torch.randn(a, b, generator=self.gen, device=self.device,
                                dtype=self.torch.float32)

    def next_set(self):
        sd = 1.0 / float(np.sqrt(self.k))
        if self._B is None or not self.collinear:
            self._B = [self._randn(n, self.k) * sd for (_, n) in self.mats]
        out = []
        for (m, n), A, B in zip(self.mats, self.A, self._B):
            g = A @ B.T
            g.add_(self._randn(m, n), alpha=self.noise)
            out.append(g.to(self.dtype).contiguous())
        return out


def torch_weights(mats, seed: int, dtype: str, device):
    import torch
    gen = torch.Generator(device=torch.device(device))
    gen.manual_seed(seed + 7919)
    dt = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    return [(torch.randn(m, n, generator=gen, device=device, dtype=torch.float32) * 0.02)
            .to(dt).contiguous() for (m, n) in mats]
