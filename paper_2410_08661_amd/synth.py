"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only random draws with the shapes and value
distributions of the workloads (Llama-2 7B / 13B / 70B linear-layer shapes of the
paper's Tab. 2 models; activations with k outlier channels, which is what makes
a column "weak", Sec. 2.4 / Sec. 3.2).  Host-side numpy only.
"""
from __future__ import annotations

import numpy as np

# (out_features, in_features) of the linear layers of one decoder block.
LLAMA_7B = [(4096, 4096), (11008, 4096), (4096, 11008)]
LLAMA_13B = [(5120, 5120), (13824, 5120), (5120, 13824)]
LLAMA_70B = [(8192, 8192), (1024, 8192), (28672, 8192), (8192, 28672)]
# One 7B decoder block as seven launches: q, k, v, o, gate, up, down.
LLAMA_7B_BLOCK = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]

CONFIGS = {
    1: dict(shapes=[(512, 512)], bits=[4], group_size=128, n_weak=8, M=[1, 16]),
    2: dict(shapes=LLAMA_7B, bits=[4], group_size=128, n_weak=128, M=[1, 8]),
    3: dict(shapes=LLAMA_13B, bits=[3, 4], group_size=128, n_weak=128, M=list(range(1, 17))),
    4: dict(shapes=LLAMA_7B, bits=[4], group_size=128, n_weak=128, M=[4096]),
    5: dict(shapes=LLAMA_70B, bits=[4], group_size=128, n_weak=256, M=[1, 2048]),
}


def seed_for(config: int, shape_index: int) -> int:
    return 1000 * int(config) + int(shape_index)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def make_weight(out_features: int, in_features: int, seed: int, std: float = 0.02) -> np.ndarray:
    """W ~ N(0, std) as float16 [OC][IC]."""
    r = _rng(seed)
    return (r.standard_normal((out_features, in_features), dtype=np.float32) * np.float32(std)).astype(np.float16)


def make_activations(m: int, in_features: int, n_weak: int, seed: int, outlier: float = 20.0) -> np.ndarray:
    """X ~ N(0, 1) float16 [M][IC] with the last n_weak channels scaled by `outlier`."""
    r = _rng(seed + 500_000)
    x = r.standard_normal((m, in_features), dtype=np.float32)
    if n_weak:
        x[:, in_features - n_weak:] *= np.float32(outlier)
    return x.astype(np.float16)


def make_grad_output(m: int, out_features: int, seed: int, std: float = 0.01) -> np.ndarray:
    """dY ~ N(0, std) float16 [M][OC]."""
    r = _rng(seed + 900_000)
    return (r.standard_normal((m, out_features), dtype=np.float32) * np.float32(std)).astype(np.float16)


def make_codes(out_features: int, kq: int, n_groups: int, bits: int, seed: int):
    """Random stored components without running a quantizer: uniform codes,
    scales ~ 0.008 * U(0.5, 1.5), integer zero-points in [0, qmax]."""
    r = _rng(seed + 700_000)
    qmax = (1 << bits) - 1
    codes = r.integers(0, qmax + 1, size=(out_features, kq), dtype=np.uint8)
    scales = (0.008 * r.uniform(0.5, 1.5, size=(out_features, n_groups))).astype(np.float16)
    zeros = r.integers(0, qmax + 1, size=(out_features, n_groups)).astype(np.float16)
    return codes, scales, zeros
