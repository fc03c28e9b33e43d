"""Seeded synthetic workloads shaped like the paper's LLaVA-1.5-7B runs.

This module holds input generators only -- none of the method's arithmetic --
and is the one module that both the HIP path's callers and the CPU oracle's
tests may use.  The paper evaluates on public benchmark suites with trained
weights (Experiments: calibration and benchmarks); neither is available here,
so seeded random tensors of the same shapes stand in: 576 visual tokens per
image (Table 4), LLaMA-7B / 13B layer shapes, N(0,1) hidden states with a few
large-magnitude outlier channels, N(0, 0.02) weights.
"""
from __future__ import annotations

from dataclasses import dataclass
from fractions import Fraction
import math

import numpy as np


@dataclass(frozen=True)
class Shape:
    name: str
    d: int
    H: int
    F: int
    layers: int
    B: int
    Nv: int
    Nt: int
    n_outlier: int
    vis_begin: int = 0

    @property
    def dh(self) -> int:
        return self.d // self.H

    @property
    def N(self) -> int:
        return self.Nv + self.Nt


# the five workload configurations (index 0 is the small one the oracle
# finishes in seconds; index 1 is one 7B-shaped layer; index 2 the 32-layer
# stack; 3 the batched serving shape; 4 the high-resolution 13B shape)
CONFIGS = [
    Shape("c1_small_layer", d=512, H=8, F=1376, layers=1, B=1, Nv=64, Nt=16, n_outlier=4),
    Shape("c2_7b_layer", d=4096, H=32, F=11008, layers=1, B=1, Nv=576, Nt=64, n_outlier=41),
    Shape("c3_7b_stack", d=4096, H=32, F=11008, layers=32, B=1, Nv=576, Nt=64, n_outlier=41),
    Shape("c4_7b_batch16", d=4096, H=32, F=11008, layers=32, B=16, Nv=576, Nt=128, n_outlier=41),
    Shape("c5_13b_hires", d=5120, H=40, F=13824, layers=40, B=4, Nv=2880, Nt=64, n_outlier=51),
]


def rng(seed: int, *stream) -> np.random.Generator:
    """Independent stream per (seed, tensor tag...)."""
    tag = [int(seed)] + [int.from_bytes(str(s).encode(), "little") % (2 ** 31) for s in stream]
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(tag)))


def hidden_state(shape: Shape, seed: int = 0) -> np.ndarray:
    """fp16 [B*N, d] ~ N(0,1); n_outlier seeded channels multiplied by 20."""
    g = rng(seed, "x0")
    x = g.standard_normal((shape.B * shape.N, shape.d), dtype=np.float32)
    ch = rng(seed, "outlier").permutation(shape.d)[: shape.n_outlier]
    x[:, ch] *= 20.0
    return x.astype(np.float16)


def positions(shape: Shape) -> np.ndarray:
    """int32 [B*N]: original position ids 0..N-1 for every sequence."""
    return np.tile(np.arange(shape.N, dtype=np.int32), shape.B)


def fp_weights(shape: Shape, seed: int = 0, layer: int = 0) -> dict:
    """fp32 N(0, 0.02) projection matrices of one layer, [N_out, K] row-major."""
    d, F = shape.d, shape.F
    out = {}
    for name, (n, k) in dict(qkv=(3 * d, d), o=(d, d), gu=(2 * F, d), down=(d, F)).items():
        g = rng(seed + layer, "w", name)
        out[name] = g.standard_normal((n, k), dtype=np.float32) * np.float32(0.02)
    return out


def rope_tables(dh: int, max_pos: int, theta: float = 1.0e4):
    """cos/sin fp32 [max_pos, dh/2], angles computed in fp64."""
    inv = theta ** (-np.arange(0, dh, 2, dtype=np.float64) / dh)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def keep_schedule(layers: int, V0: int, avg: Fraction, last: Fraction, full_layers: int = 2):
    """Per-layer integer budgets K_l: keep everything in the first
    ``full_layers`` layers, then a linear ramp that ends at ``last`` and makes
    the mean keep ratio over all layers equal ``avg``; K_l = ceil(r_l * V0)."""
    n = layers - full_layers
    # full_layers * 1 + n * (r_first + last) / 2 = avg * layers
    r_first = (avg * layers - full_layers) * 2 / n - last
    ks = []
    for l in range(layers):
        if l < full_layers:
            r = Fraction(1)
        else:
            r = r_first + (last - r_first) * Fraction(l - full_layers, n - 1)
        ks.append(int(math.ceil(r * V0)))
    return ks


def schedule_for(shape: Shape):
    """Budgets used by the benchmark configurations."""
    if shape.layers == 1:
        # single-layer cases: 30 % of the visual tokens (19 of 64 as the small
        # configuration states it; ceil(0.3 * 576) = 173 for the 7B layer)
        return [19] if shape.Nv == 64 else [int(math.ceil(Fraction(3, 10) * shape.Nv))]
    if shape.name.startswith("c5"):
        return keep_schedule(shape.layers, shape.Nv, Fraction(1, 5), Fraction(1, 20))
    return keep_schedule(shape.layers, shape.Nv, Fraction(3, 10), Fraction(1, 10))


def fp_weights_device(shape: Shape, seed: int = 0, layer: int = 0, device: str = "cuda") -> dict:
    """The same four fp32 N(0, 0.02) matrices drawn by torch's seeded DEVICE generator: what the
    benchmark and the full-depth tests use, where 32-40 layers of 200-300 M weights each are too slow
    to draw on the host.  Returns torch tensors on ``device``; ``.cpu().numpy()`` gives the oracle the
    same values."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + layer)
    d, F = shape.d, shape.F
    out = {}
    for name, (n, k) in dict(qkv=(3 * d, d), o=(d, d), gu=(2 * F, d), down=(d, F)).items():
        out[name] = torch.randn((n, k), generator=g, device=device, dtype=torch.float32) * 0.02
    return out
