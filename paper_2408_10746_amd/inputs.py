"""Seeded synthetic inputs for the cached Parallel-Adapter step.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmark.  It holds none of the method's arithmetic: it only
draws numbers (hidden states, labels, lengths, initial parameters, epoch
orders) with the shapes and statistics of the paper's workloads
(transformer hidden states of GLUE-style classification inputs, paper Sec. 6.1).
It needs numpy only.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_DATA = 1234
SEED_PARAMS = 1235
SEED_PERM = 1236


@dataclass(frozen=True)
class Workload:
    """Shape of one configuration (r is the adapter width, not a reduction factor)."""
    name: str
    L: int
    d: int
    n_max: int
    B: int
    r: int
    C: int
    N: int
    cache_dtype: str = "bf16"        # "bf16" or "f32"
    outlier_frac: float = 0.0        # fraction of channels scaled by outlier_scale
    outlier_scale: float = 20.0
    len_lo: int = 0                  # 0: every sample has n_max tokens
    epochs: int = 1

    @property
    def layer_block(self) -> int:
        return 2 * self.d * self.r + self.r + self.d + 1

    @property
    def P(self) -> int:
        return self.L * self.layer_block + self.d * self.C + self.C


WORKLOADS = {
    "tiny": Workload("tiny", L=4, d=256, n_max=64, B=8, r=32, C=2, N=64, cache_dtype="f32", epochs=3),
    "t5base": Workload("t5base", L=12, d=768, n_max=128, B=32, r=96, C=3, N=4096),
    "large": Workload("large", L=24, d=1024, n_max=128, B=32, r=128, C=2, N=8192),
    "llama7b": Workload("llama7b", L=32, d=4096, n_max=256, B=16, r=256, C=4, N=2048,
                        outlier_frac=0.01),
    "longseq": Workload("longseq", L=32, d=4096, n_max=1024, B=8, r=512, C=2, N=1024, len_lo=256),
}


def outlier_channels(seed: int, d: int, frac: float) -> np.ndarray:
    """The fixed channel set that carries large-magnitude values (same for all layers/tokens)."""
    k = int(np.floor(frac * d))
    if k == 0:
        return np.zeros(0, dtype=np.int64)
    rng = np.random.default_rng([seed, 0x0c11a])
    return np.sort(rng.choice(d, size=k, replace=False))


def sample_acts(seed: int, sample_id: int, L: int, n: int, d: int,
                outlier_frac: float = 0.0, outlier_scale: float = 20.0) -> np.ndarray:
    """Hidden states of one sample: [L][n][d] float32.

    N(0,1) draws, then every token row is normalised over d (zero mean, unit
    variance, eps 1e-5, no affine) like the output of a transformer's layer
    norm; optional outlier channels are scaled afterwards."""
    rng = np.random.default_rng([seed, int(sample_id)])
    u = rng.standard_normal(size=(L, n, d), dtype=np.float32)
    mu = u.mean(axis=-1, keepdims=True, dtype=np.float32)
    var = ((u - mu) ** 2).mean(axis=-1, keepdims=True, dtype=np.float32)
    a = ((u - mu) / np.sqrt(var + np.float32(1e-5))).astype(np.float32)
    if outlier_frac > 0.0:
        ch = outlier_channels(seed, d, outlier_frac)
        a[..., ch] *= np.float32(outlier_scale)
    return a


def batch_acts(w: Workload, sample_ids, seed: int = SEED_DATA) -> np.ndarray:
    """[count][L][n_max][d] float32 for the given sample ids."""
    return np.stack([sample_acts(seed, int(s), w.L, w.n_max, w.d, w.outlier_frac, w.outlier_scale)
                     for s in sample_ids])


def labels(w: Workload, seed: int = SEED_DATA) -> np.ndarray:
    rng = np.random.default_rng([seed, 0x1abe1])
    return rng.integers(0, w.C, size=w.N, dtype=np.int32)


def lengths(w: Workload, seed: int = SEED_DATA) -> np.ndarray:
    """Valid token count per sample: n_max, or uniform in [len_lo, n_max]."""
    if w.len_lo <= 0:
        return np.full(w.N, w.n_max, dtype=np.int32)
    rng = np.random.default_rng([seed, 0x1e45])
    return rng.integers(w.len_lo, w.n_max + 1, size=w.N, dtype=np.int32)


def init_params(w: Workload, seed: int = SEED_PARAMS) -> np.ndarray:
    """Initial flat parameter vector (float32).

    Down-projections and the classifier are N(0, 1/d); biases and every
    up-projection are zero (the side network starts as a no-op, paper Sec. 4.3);
    every gate starts at 0.5 (paper Sec. 4.1)."""
    rng = np.random.default_rng([seed, 1])
    p = np.zeros(w.P, dtype=np.float32)
    PL, d, r, C = w.layer_block, w.d, w.r, w.C
    s = np.float32(1.0 / np.sqrt(d))
    for l in range(w.L):
        o = l * PL
        p[o:o + d * r] = rng.standard_normal(d * r, dtype=np.float32) * s
        p[o + PL - 1] = 0.5
    o = w.L * PL
    p[o:o + d * C] = rng.standard_normal(d * C, dtype=np.float32) * s
    return p


def random_params(w: Workload, seed: int = SEED_PARAMS, scale: float = 1.0, up_scale: float = 1.0) -> np.ndarray:
    """A generic (non-initial) state: every entry non-zero, gates spread around 0.5.

    up_scale shrinks the up-projections (a partly trained network: they start at zero)."""
    rng = np.random.default_rng([seed, 2])
    p = np.zeros(w.P, dtype=np.float32)
    PL, d, r, C = w.layer_block, w.d, w.r, w.C
    for l in range(w.L):
        o = l * PL
        p[o:o + d * r] = rng.standard_normal(d * r, dtype=np.float32) * np.float32(scale / np.sqrt(d))
        o += d * r
        p[o:o + r] = rng.standard_normal(r, dtype=np.float32) * np.float32(0.1 * scale)
        o += r
        p[o:o + r * d] = rng.standard_normal(r * d, dtype=np.float32) * np.float32(scale * up_scale / np.sqrt(r))
        o += r * d
        p[o:o + d] = rng.standard_normal(d, dtype=np.float32) * np.float32(0.1 * scale)
        o += d
        p[o] = np.float32(0.5 + 0.3 * rng.standard_normal())
    o = w.L * PL
    p[o:o + d * C] = rng.standard_normal(d * C, dtype=np.float32) * np.float32(scale / np.sqrt(d))
    o += d * C
    p[o:o + C] = rng.standard_normal(C, dtype=np.float32) * np.float32(0.1 * scale)
    return p


def epoch_order(w: Workload, epoch: int, seed: int = SEED_PERM) -> np.ndarray:
    """Sample order of an epoch (0-based): identity first, seeded shuffles afterwards."""
    if epoch == 0:
        return np.arange(w.N, dtype=np.int64)
    rng = np.random.default_rng([seed, epoch])
    return rng.permutation(w.N).astype(np.int64)
