"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and shapes them; it holds none of the method's
arithmetic (no quantization, packing or products) and is the single source of inputs for
both the HIP library and the CPU oracle.

The paper evaluates on GPTQ-quantized LLaMA-7B/13B/30B weights; neither those weights nor
calibration data are available here, so the public LLaMA layer shapes with zero-mean
Gaussian weights stand in for them (Section 4, "Goals and setup").  A decoder "layer set"
is the seven linear layers of one block: q, k, v, o (H x H), gate, up (I x H), down (H x I).

Draw order, per matrix i of configuration c (generator = Philox keyed by
SeedSequence([seed_c, i]), so each matrix can be drawn independently of the others):
  1. W = standard_normal((N, K), float32) * std
  2. if outliers: u = random((N, K), float32); W[u < 0.001] *= 20
  3. x = standard_normal((K,), float32)           (GEMV configurations)
     X = standard_normal((M, K), float32)          (small-M GEMM; one draw per M, in order)
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    bits: int
    group: int
    std: float
    outliers: bool
    shapes: Tuple[Tuple[int, int], ...]      # (N, K) per matrix, in draw order
    batch: Tuple[int, ...] = (1,)            # M values; (1,) means GEMV

    @property
    def weights(self) -> int:
        return sum(n * k for n, k in self.shapes)


def _layer_set(h: int, i: int) -> Tuple[Tuple[int, int], ...]:
    return ((h, h),) * 4 + ((i, h),) * 2 + ((h, i),)


CONFIGS = {
    "C1": Config("C1", 0, 4, 64, 0.02, False, ((512, 512),)),
    "C2": Config("C2", 1, 4, 128, 0.02, True, _layer_set(4096, 11008)),
    "C3": Config("C3", 2, 3, 64, 0.02, False, _layer_set(5120, 13824)),
    "C4": Config("C4", 3, 2, 32, 0.015, False, _layer_set(8192, 22016)),
    "C5": Config("C5", 4, 4, 128, 0.02, True,
                 ((4096, 4096), (11008, 4096), (4096, 11008)), batch=(16, 64, 128)),
}


def _rng(seed: int, index: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, index])))


def draw_weights(rng: np.random.Generator, n: int, k: int, std: float, outliers: bool) -> np.ndarray:
    w = rng.standard_normal((n, k), dtype=np.float32)
    w *= np.float32(std)
    if outliers:
        u = rng.random((n, k), dtype=np.float32)
        w[u < np.float32(0.001)] *= np.float32(20.0)
    return w


def matrix(cfg: Config, index: int):
    """Inputs of matrix `index` of a configuration: (W [N,K], [x or X per batch size])."""
    n, k = cfg.shapes[index]
    rng = _rng(cfg.seed, index)
    w = draw_weights(rng, n, k, cfg.std, cfg.outliers)
    acts = []
    for m in cfg.batch:
        if m == 1:
            acts.append(rng.standard_normal((k,), dtype=np.float32))
        else:
            acts.append(rng.standard_normal((m, k), dtype=np.float32))
    return w, acts


def small_case(seed: int, n: int, k: int, std: float = 0.02, outliers: bool = False, m: int = 1):
    """Free-form seeded case for parity tests at odd sizes: (W [n,k], x [k] or X [m,k])."""
    rng = _rng(10_000 + seed, 0)
    w = draw_weights(rng, n, k, std, outliers)
    if m == 1:
        x = rng.standard_normal((k,), dtype=np.float32)
    else:
        x = rng.standard_normal((m, k), dtype=np.float32)
    return w, x
