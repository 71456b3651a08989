"""CPU oracle of the paper's default Parallel-Adapter architecture (Sec. 4.1, Fig. "pa-detail"; Sec. 6.1): the
r-wide ladder whose adapter is a reduced transformer layer.

TEST INFRASTRUCTURE ONLY (imported by tests/ alone).  Plain PyTorch CPU operations in float64, written the slow
obvious way, one sample at a time; gradients come from reverse-mode differentiation of exactly these lines (a
library primitive), and are pinned independently by finite differences (tests/test_ladder_oracle.py).

With w = d / reduction factor the adapter width, cached backbone outputs b_1..b_L (n x d) and a_0 = 0:

    u_l = b_l W_down^l + c_down^l                      (downsample the backbone activation, Sec. 4.1)
    x_l = lambda_l u_l + (1 - lambda_l) a_{l-1}        (gate, initial value 0.5, applied AFTER the down-projection)
    a_l = Block_l(x_l)                                 (a transformer layer at width w: "a lightweight version of
                                                         the backbone", all dimensions 1/reduction factor)
    y   = b_L + a_L W_up + c_up                        (one up-projection at the end; side output summed with the
                                                         backbone's)
    p = mean over valid tokens of y ;  z = p W_cls + c_cls ;  loss = mean over the batch of cross-entropy(z, label)

Block (readings, the paper names no layer internals): pre-norm encoder layer,
    xn = LayerNorm(x; g1, h1) ;  q, k, v = split(xn W_qkv + b_qkv) ;  per head  P = softmax(q k^T / sqrt(dh)) over the
    sample's valid tokens,  o = P v ;  t = x + concat(o) W_o + b_o ;
    tn = LayerNorm(t; g2, h2) ;  a = t + GELU_erf(tn W_1 + b_1) W_2 + b_2 ,   LayerNorm eps 1e-5, FFN width 4 w.

Flat parameter vector (the layout the library uses too; interfaces have to agree):
  per layer [ W_down d x w | c_down w | ln1_g w | ln1_b w | W_qkv w x 3w | b_qkv 3w | W_o w x w | b_o w | ln2_g w |
              ln2_b w | W_1 w x 4w | b_1 4w | W_2 4w x w | b_2 w | lambda, 3 unused zeros ]
  then      [ W_up w x d | c_up d | W_cls d x C | c_cls C ]
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class LadderDims:
    L: int
    d: int
    w: int
    heads: int
    C: int

    @property
    def f(self):
        return 4 * self.w

    def layer_fields(self):
        d, w, f = self.d, self.w, self.f
        return [("W_down", d * w), ("c_down", w), ("ln1_g", w), ("ln1_b", w), ("W_qkv", w * 3 * w), ("b_qkv", 3 * w),
                ("W_o", w * w), ("b_o", w), ("ln2_g", w), ("ln2_b", w), ("W_1", w * f), ("b_1", f), ("W_2", f * w),
                ("b_2", w), ("lambda", 4)]

    @property
    def layer_block(self):
        return sum(n for _, n in self.layer_fields())

    @property
    def P(self):
        return self.L * self.layer_block + self.w * self.d + self.d + self.d * self.C + self.C


def param_slices(dims: LadderDims):
    out = {}
    o = 0
    for l in range(dims.L):
        for name, n in dims.layer_fields():
            out[f"{name}{l}"] = slice(o, o + (1 if name == "lambda" else n))
            o += n
    for name, n in (("W_up", dims.w * dims.d), ("c_up", dims.d), ("W_cls", dims.d * dims.C), ("c_cls", dims.C)):
        out[name] = slice(o, o + n)
        o += n
    assert o == dims.P
    return out


def decayed_mask(dims: LadderDims) -> np.ndarray:
    """AdamW decays the matrices only (projections and the classifier), not biases, norms or gates."""
    m = np.zeros(dims.P, dtype=bool)
    for name, sl in param_slices(dims).items():
        if name.startswith("W_"):
            m[sl] = True
    return m


def _layer_norm(x, g, h):
    mu = x.mean(dim=-1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=-1, keepdim=True)
    return (x - mu) / torch.sqrt(var + 1e-5) * g + h


def _gelu(u):
    return 0.5 * u * (1.0 + torch.erf(u / math.sqrt(2.0)))


def forward(dims: LadderDims, acts, lens, labels, p: torch.Tensor, return_attention: bool = False):
    """acts [B][L][n_max][d] (float64 values of the cache), p flat float64 tensor.  Returns (loss, logits[B][C], extra)."""
    sl = param_slices(dims)
    d, w, f, nh, C = dims.d, dims.w, dims.f, dims.heads, dims.C
    dh = w // nh
    losses, logits, att = [], [], []
    for s in range(len(labels)):
        n = int(lens[s])
        b = torch.as_tensor(acts[s, :, :n, :], dtype=torch.float64)
        a = torch.zeros(n, w, dtype=torch.float64)
        for l in range(dims.L):
            g = lambda name: p[sl[f"{name}{l}"]]
            lam = g("lambda")
            u = b[l] @ g("W_down").reshape(d, w) + g("c_down")
            x = lam * u + (1.0 - lam) * a
            xn = _layer_norm(x, g("ln1_g"), g("ln1_b"))
            qkv = xn @ g("W_qkv").reshape(w, 3 * w) + g("b_qkv")
            q, k, v = qkv[:, :w], qkv[:, w:2 * w], qkv[:, 2 * w:]
            heads = []
            for h in range(nh):
                cs = slice(h * dh, (h + 1) * dh)
                P = torch.softmax(q[:, cs] @ k[:, cs].T / math.sqrt(dh), dim=-1)
                if return_attention:
                    att.append(P.detach().numpy())
                heads.append(P @ v[:, cs])
            t = x + torch.cat(heads, dim=1) @ g("W_o").reshape(w, w) + g("b_o")
            tn = _layer_norm(t, g("ln2_g"), g("ln2_b"))
            a = t + _gelu(tn @ g("W_1").reshape(w, f) + g("b_1")) @ g("W_2").reshape(f, w) + g("b_2")
        y = b[dims.L - 1] + a @ p[sl["W_up"]].reshape(w, d) + p[sl["c_up"]]
        z = y.mean(dim=0) @ p[sl["W_cls"]].reshape(d, C) + p[sl["c_cls"]]
        logits.append(z)
        losses.append(torch.logsumexp(z, 0) - z[int(labels[s])])
    return torch.stack(losses).mean(), torch.stack(logits), att


def loss_grad(dims: LadderDims, acts, lens, labels, params: np.ndarray, want_grads: bool = True):
    p = torch.tensor(np.asarray(params, dtype=np.float64), requires_grad=want_grads)
    loss, logits, _ = forward(dims, acts, lens, labels, p)
    grads = None
    if want_grads:
        loss.backward()
        grads = p.grad.numpy().copy()
    return {"loss": float(loss.item()), "logits": logits.detach().numpy(), "grads": grads}


def adamw(dims: LadderDims, p, m, v, t_new, g, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """In place on float64 arrays: decoupled decay on the matrices, bias-corrected moments, eps added to the root."""
    dec = decayed_mask(dims)
    m *= beta1
    m += (1 - beta1) * g
    v *= beta2
    v += (1 - beta2) * g * g
    mhat = m / (1 - beta1 ** t_new)
    vhat = v / (1 - beta2 ** t_new)
    p[dec] -= lr * weight_decay * p[dec]
    p -= lr * mhat / (np.sqrt(vhat) + eps)


def init_params(dims: LadderDims, seed: int, trained: bool = False) -> np.ndarray:
    """Initial state: Gaussian N(0, 1/fan_in) matrices (the paper's pruning-based initialisation needs backbone weights;
    Gaussian is one of its ablation arms), unit norm gains, zero biases, gates 0.5, and a ZERO up-projection (Sec. 4.3:
    the side network starts as a no-op).  trained=True: a generic state with every entry non-zero."""
    rng = np.random.default_rng([seed, 7])
    p = np.zeros(dims.P, dtype=np.float32)
    sl = param_slices(dims)
    fan = {"W_down": dims.d, "W_qkv": dims.w, "W_o": dims.w, "W_1": dims.w, "W_2": dims.f, "W_up": dims.w, "W_cls": dims.d}
    for name, s in sl.items():
        base = name.rstrip("0123456789")
        n = s.stop - s.start
        if base in fan:
            if base == "W_up" and not trained:
                continue
            p[s] = rng.standard_normal(n).astype(np.float32) / np.float32(math.sqrt(fan[base]))
        elif base in ("ln1_g", "ln2_g"):
            p[s] = 1.0 + (0.1 * rng.standard_normal(n).astype(np.float32) if trained else 0.0)
        elif base == "lambda":
            p[s] = 0.5 + (0.2 * rng.standard_normal() if trained else 0.0)
        elif trained:
            p[s] = 0.1 * rng.standard_normal(n).astype(np.float32)
    return p
