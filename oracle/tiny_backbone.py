"""A tiny frozen transformer encoder in numpy (float64).

TEST INFRASTRUCTURE ONLY.  It exists for one check: training the adapters from
activations cached once gives the same losses as re-running the frozen backbone
every epoch (paper Sec. 4.2: with the backbone frozen and independent of the
adapters, its activations for a given input never change).  It stands in for the
pretrained backbone, whose weights are not available; only its per-layer outputs
b_1..b_L (each [n][d]) matter.
"""
from __future__ import annotations

import numpy as np


def _layer_norm(x):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + 1e-5)


class TinyBackbone:
    """L post-norm encoder layers, single attention head, ReLU feed-forward."""

    def __init__(self, L: int, d: int, vocab: int, n_max: int, seed: int):
        rng = np.random.default_rng([seed, 0xbb])
        s = 1.0 / np.sqrt(d)
        self.L, self.d = L, d
        self.emb = rng.standard_normal((vocab, d))
        self.pos = 0.1 * rng.standard_normal((n_max, d))
        self.layers = []
        for _ in range(L):
            self.layers.append({
                "Wq": rng.standard_normal((d, d)) * s, "Wk": rng.standard_normal((d, d)) * s,
                "Wv": rng.standard_normal((d, d)) * s, "Wo": rng.standard_normal((d, d)) * s,
                "W1": rng.standard_normal((d, 2 * d)) * s, "W2": rng.standard_normal((2 * d, d)) * s / np.sqrt(2.0),
            })
        self.calls = 0

    def forward(self, tokens: np.ndarray) -> np.ndarray:
        """tokens int[n] -> per-layer hidden states [L][n][d] (the embedding b_0 is not returned)."""
        self.calls += 1
        n = tokens.shape[0]
        x = _layer_norm(self.emb[tokens] + self.pos[:n])
        outs = []
        for w in self.layers:
            q, k, v = x @ w["Wq"], x @ w["Wk"], x @ w["Wv"]
            a = q @ k.T / np.sqrt(self.d)
            a = np.exp(a - a.max(axis=-1, keepdims=True))
            a /= a.sum(axis=-1, keepdims=True)
            x = _layer_norm(x + (a @ v) @ w["Wo"])
            x = _layer_norm(x + np.maximum(x @ w["W1"], 0.0) @ w["W2"])
            outs.append(x)
        return np.stack(outs)
