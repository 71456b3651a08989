"""CPU-only pins of the ladder oracle (paper Sec. 4.1 default architecture) against things other than itself."""
import math

import numpy as np
import pytest
import torch

from oracle import ladder_oracle as lo
from paper_2408_10746_amd import inputs


def problem(seed=0, L=2, d=8, n=5, w=4, heads=2, C=3, B=3, lens=None, trained=True):
    dims = lo.LadderDims(L, d, w, heads, C)
    wl = inputs.Workload("t", L=L, d=d, n_max=n, B=B, r=w, C=C, N=B, cache_dtype="f32")
    acts = inputs.batch_acts(wl, range(B), seed=seed + 31).astype(np.float64)
    rng = np.random.default_rng(seed)
    labels = rng.integers(0, C, size=B).astype(np.int32)
    lens = np.full(B, n, dtype=np.int32) if lens is None else np.asarray(lens, dtype=np.int32)
    return dims, acts, lens, labels, lo.init_params(dims, seed, trained=trained).astype(np.float64)


def test_layout_counts_and_mask():
    dims = lo.LadderDims(2, 8, 4, 2, 3)
    w, d, f = 4, 8, 16
    per_layer = d * w + w + 2 * w + 3 * w * w + 3 * w + w * w + w + 2 * w + w * f + f + f * w + w + 4
    assert dims.layer_block == per_layer and dims.P == 2 * per_layer + w * d + d + d * 3 + 3
    sl = lo.param_slices(dims)
    assert sl["lambda1"].stop - sl["lambda1"].start == 1 and sl["W_up"].start == 2 * per_layer
    assert all(s.start % 4 == 0 for name, s in sl.items() if name != "c_cls")     # 16-byte aligned rows for the library
    dec = lo.decayed_mask(dims)
    assert dec[sl["W_qkv0"]].all() and not dec[sl["b_qkv0"]].any() and not dec[sl["ln1_g1"]].any() and not dec[sl["lambda0"]].any()


def test_zero_up_projection_is_the_identity_closed_form():
    """Sec. 4.3: with W_up = 0 and c_up = 0 the side network is a no-op, y = b_L: softmax regression on mean(b_L)."""
    dims, acts, lens, labels, p = problem(seed=1, lens=[5, 2, 4], trained=False)
    out = lo.loss_grad(dims, acts, lens, labels, p)
    sl = lo.param_slices(dims)
    pooled = np.stack([acts[s, -1, :lens[s]].mean(axis=0) for s in range(3)])
    z = pooled @ p[sl["W_cls"]].reshape(dims.d, dims.C) + p[sl["c_cls"]]
    ref = np.mean([math.log(np.exp(zz).sum()) - zz[y] for zz, y in zip(z, labels)])
    assert abs(out["loss"] - ref) < 1e-13
    np.testing.assert_allclose(out["logits"], z, atol=1e-13)
    g = out["grads"]
    assert np.all(g[: dims.L * dims.layer_block] == 0.0)             # nothing reaches the adapters ...
    assert np.any(g[sl["W_up"]] != 0.0)                              # ... except through the up-projection itself


def test_gradients_finite_differences_every_parameter():
    dims, acts, lens, labels, p = problem(seed=2, lens=[5, 3, 1])
    g = lo.loss_grad(dims, acts, lens, labels, p)["grads"]
    eps = 1e-6
    for name, sl in lo.param_slices(dims).items():
        idx = np.arange(sl.start, sl.stop)
        for i in idx[:: max(1, len(idx) // 6)]:                         # a spread of entries of every tensor
            q = p.copy(); q[i] += eps
            lp = lo.loss_grad(dims, acts, lens, labels, q, want_grads=False)["loss"]
            q[i] -= 2 * eps
            lm = lo.loss_grad(dims, acts, lens, labels, q, want_grads=False)["loss"]
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - g[i]) <= 2e-6 * abs(fd) + 2e-9, (name, i, fd, g[i])
        assert np.linalg.norm(g[sl]) > 0, name
    # the padding slots after each gate take no gradient
    for l in range(dims.L):
        s = lo.param_slices(dims)[f"lambda{l}"]
        assert np.all(g[s.stop: s.stop + 3] == 0.0)


def test_attention_rows_sum_to_one_and_see_only_valid_tokens():
    dims, acts, lens, labels, p = problem(seed=3, lens=[5, 2, 4])
    _, _, att = lo.forward(dims, acts, lens, labels, torch.tensor(p), return_attention=True)
    assert len(att) == 3 * dims.L * dims.heads
    for P in att:
        np.testing.assert_allclose(P.sum(axis=1), 1.0, atol=1e-14)
        assert np.all(P > 0)
    assert att[0].shape == (5, 5) and att[dims.L * dims.heads].shape == (2, 2)
    # padding is ignored: garbage beyond a sample's length changes nothing
    acts2 = acts.copy()
    acts2[1, :, 2:, :] = 1e3
    a = lo.loss_grad(dims, acts, lens, labels, p)
    b = lo.loss_grad(dims, acts2, lens, labels, p)
    assert a["loss"] == b["loss"] and np.array_equal(a["grads"], b["grads"])


def test_token_permutation_and_batch_invariances():
    """Attention is equivariant under a permutation of a sample's tokens and the pooled mean invariant, so loss and
    gradients do not change; the batch mean is linear in the samples."""
    dims, acts, lens, labels, p = problem(seed=4, n=6, lens=[6, 6, 6])
    base = lo.loss_grad(dims, acts, lens, labels, p)
    perm = np.random.default_rng(0).permutation(6)
    acts_p = acts.copy()
    acts_p[0] = acts[0][:, perm, :]
    out = lo.loss_grad(dims, acts_p, lens, labels, p)
    assert abs(out["loss"] - base["loss"]) < 1e-13
    np.testing.assert_allclose(out["grads"], base["grads"], rtol=1e-10, atol=1e-14)
    halves = [lo.loss_grad(dims, acts[i], lens[i], labels[i], p) for i in (slice(0, 1), slice(1, 3))]
    np.testing.assert_allclose(base["grads"], (halves[0]["grads"] + 2 * halves[1]["grads"]) / 3, rtol=1e-10, atol=1e-14)


def test_single_token_sample_attention_is_trivial():
    """One token: softmax over one key is 1, the head output is v itself (closed form of the whole block)."""
    dims, acts, lens, labels, p = problem(seed=5, L=1, n=1, B=1, heads=2)
    sl = lo.param_slices(dims)
    d, w, f = dims.d, dims.w, dims.f
    g = lambda name: p[sl[name + "0"]]
    ln = lambda x, gg, hh: (x - x.mean()) / math.sqrt(((x - x.mean()) ** 2).mean() + 1e-5) * gg + hh
    b = acts[0, 0, 0]
    x = g("lambda")[0] * (b @ g("W_down").reshape(d, w) + g("c_down"))
    v = (ln(x, g("ln1_g"), g("ln1_b")) @ g("W_qkv").reshape(w, 3 * w) + g("b_qkv"))[2 * w:]
    t = x + v @ g("W_o").reshape(w, w) + g("b_o")
    u = ln(t, g("ln2_g"), g("ln2_b")) @ g("W_1").reshape(w, f) + g("b_1")
    a = t + (0.5 * u * (1 + np.vectorize(math.erf)(u / math.sqrt(2)))) @ g("W_2").reshape(f, w) + g("b_2")
    y = b + a @ p[sl["W_up"]].reshape(w, d) + p[sl["c_up"]]
    z = y @ p[sl["W_cls"]].reshape(d, dims.C) + p[sl["c_cls"]]
    np.testing.assert_allclose(lo.loss_grad(dims, acts, lens, labels, p, want_grads=False)["logits"][0], z, atol=1e-13)


def test_adamw_first_step_and_mask():
    dims, acts, lens, labels, p = problem(seed=6)
    g = lo.loss_grad(dims, acts, lens, labels, p)["grads"]
    p1, m, v = p.copy(), np.zeros_like(p), np.zeros_like(p)
    lo.adamw(dims, p1, m, v, 1, g)
    dec = lo.decayed_mask(dims)
    # first step: mhat = g, vhat = g^2 -> step lr * g / (|g| + eps), after the decoupled decay of the matrices
    expect = np.where(dec, p * (1 - 1e-3 * 0.01), p) - 1e-3 * g / (np.abs(g) + 1e-8)
    np.testing.assert_allclose(p1, expect, rtol=1e-12, atol=1e-15)
    ref = torch.tensor(p.copy(), requires_grad=True)
    opt = torch.optim.AdamW([{"params": [ref], "weight_decay": 0.0}], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    ref.grad = torch.tensor(g)
    opt.step()
    np.testing.assert_allclose(p1[~dec], ref.detach().numpy()[~dec], rtol=1e-12, atol=1e-15)   # a library optimizer, no decay
