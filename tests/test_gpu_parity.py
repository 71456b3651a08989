"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances (relative L2 error per tensor, |a-b|_2 / |b|_2, and relative error of the loss):
  fp32 mode  1e-5      bf16 cache + bf16 MFMA operands with fp32 accumulation  2e-2
Tensors the oracle says are exactly zero must be exactly zero.
Integer/byte work (the cache contents) is bit-exact.
Gate gradients: each one is a sum of tokens x d signed terms that may cancel, so besides the L-vector of all
gates (relative L2, as any tensor) every single gate is held to |error| <= tolerance x the sum of the absolute
values of its own terms, which the oracle reports (its cancellation scale).
"""
import os
import sys
import time

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2408_10746_amd import inputs
from paper_2408_10746_amd.inputs import Workload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def note(msg):
    """Progress line (long tests must not look hung): to stderr, and appended to the file PAC_TEST_NOTES names,
    which pytest's capture does not hold back."""
    line = f"[{time.strftime('%H:%M:%S')}] {msg}\n"
    sys.__stderr__.write(line)
    sys.__stderr__.flush()
    path = os.environ.get("PAC_TEST_NOTES")
    if path:
        with open(path, "a") as f:
            f.write(line)


def rel_err(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    if nb == 0.0:
        return 0.0 if np.max(np.abs(a), initial=0.0) <= 1e-30 else np.inf
    return float(np.linalg.norm(a - b) / nb)


def tensors(dims):
    """Parameter tensors compared one by one.  The L gate scalars are compared as one L-vector:
    a single gate gradient is a sum of tokens x d signed terms that can cancel to (nearly)
    nothing, and then no finite-precision path has a meaningful relative error on it alone."""
    out = {}
    lam = []
    for name, sl in orc.param_slices(dims).items():
        if name.startswith("lambda"):
            lam.append(sl.start)
        else:
            out[name] = sl
    out["lambda[0:L]"] = np.array(lam)
    return out


def check_gates(dims, grads, ref, tol, what=""):
    """Every gate gradient against the oracle's, |error| <= tol x that gate's cancellation scale; a gate whose
    terms are all zero (zero-initialised up-projections) must be exactly zero.  Returns the worst ratio."""
    sl = orc.param_slices(dims)
    worst = 0.0
    for l in range(dims.L):
        i = sl[f"lambda{l}"].start
        scale = float(ref["glam_abs"][l])
        err = abs(float(grads[i]) - float(ref["grads"][i]))
        if scale == 0.0:
            assert grads[i] == 0.0, (what, f"lambda{l}", float(grads[i]))
            continue
        assert err <= tol * scale, (what, f"lambda{l}", err, scale, err / scale)
        worst = max(worst, err / scale)
    return worst


def oracle_batch(w: Workload, acts, lens, labels, params, want_grads=True):
    cache, off, lens_a = orc.cache_fill(acts, lens=lens, as_bf16=(w.cache_dtype == "bf16"))
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    return dims, orc.loss_grad(dims, orc.widen(cache), off, lens_a, labels, params.astype(np.float64),
                               want_grads=want_grads)


def check_against_oracle(w, sess, ids, acts, lens, labels, params, tol, what=""):
    note(f"{what}: oracle on {len(ids)} samples")
    dims, ref = oracle_batch(w, acts, lens, labels, params)
    note(f"{what}: HIP path")
    lab_dev = torch.from_numpy(labels).to(sess.dev)
    sess.set_params(params)
    sess.loss_grad(ids, lab_dev)
    torch.cuda.synchronize()
    loss = float(sess.loss.item())
    B = len(ids)
    logits = sess.logits.cpu().numpy()[: B * w.C].reshape(B, w.C)
    grads = sess.grads.cpu().numpy()
    assert np.isfinite(loss), what
    assert abs(loss - ref["loss"]) <= tol * max(abs(ref["loss"]), 1e-3), (what, loss, ref["loss"])
    assert rel_err(logits, ref["logits"]) <= tol, (what, "logits", rel_err(logits, ref["logits"]))
    worst = {}
    for name, sl in tensors(dims).items():
        e = rel_err(grads[sl], ref["grads"][sl])
        worst[name] = e
        assert e <= tol, (what, name, e)
    worst["gate/scale"] = check_gates(dims, grads, ref, tol, what)
    note(f"{what}: loss {loss:.6f} vs {ref['loss']:.6f}; worst grad rel err {max(worst.values()):.2e} "
         f"({max(worst, key=worst.get)})")
    return ref, loss, grads, worst


def make_session(w, lens=None, flags=0):
    from paper_2408_10746_amd.runtime import Session
    return Session(w, lens=lens, flags=flags)


# ---------------------------------------------------------------------------
# a0: cache fill (bit-exact)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_cache_fill_bits_ragged_and_specials(dtype):
    w = Workload("cf", L=3, d=96, n_max=21, B=4, r=32, C=2, N=9, cache_dtype=dtype)
    rng = np.random.default_rng(3)
    lens = rng.integers(1, w.n_max + 1, size=w.N).astype(np.int32)
    lens[0] = w.n_max
    lens[1] = 1
    acts = inputs.batch_acts(w, range(w.N))
    acts[2, 0, 0, :8] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.0e38]
    acts[3, 1, 0, :4] = [1e-40, -1e-45, 65504.0, np.finfo(np.float32).max]
    sess = make_session(w, lens=lens)
    order = np.array([4, 0, 7, 2, 1, 8, 3, 6, 5])       # fill order != id order, two calls
    sess.cache_fill(order[:5], acts[order[:5]], lens[order[:5]])
    sess.cache_fill(order[5:], acts[order[5:]], lens[order[5:]])
    torch.cuda.synchronize()
    ref, off, _ = orc.cache_fill(acts[order], lens=lens[order], as_bf16=(dtype == "bf16"))
    from paper_2408_10746_amd import binding as pb
    for k, sid in enumerate(order):
        o, ln = pb.pac_cache_lookup(sess.ctx, int(sid))
        assert o == off[k] and ln == lens[sid]
        got = sess.cache_block(int(sid))
        exp = ref[off[k]: off[k] + w.L * ln * w.d].reshape(w.L, ln, w.d)
        if dtype == "bf16":
            np.testing.assert_array_equal(got, exp)
        else:
            np.testing.assert_array_equal(got.view(np.uint32), exp.view(np.uint32))
    # refill in place with new values keeps the layout
    acts2 = acts[[7]] * np.float32(0.5)
    sess.cache_fill([7], acts2, lens[[7]])
    torch.cuda.synchronize()
    ref2, _, _ = orc.cache_fill(acts2, lens=lens[[7]], as_bf16=(dtype == "bf16"))
    np.testing.assert_array_equal(sess.cache_block(7).ravel(), ref2)
    # bf16 input activations
    a16 = torch.from_numpy(acts[[5]]).to(torch.bfloat16).cuda()
    sess.cache_fill([5], a16, lens[[5]])
    torch.cuda.synchronize()
    exp16, _, _ = orc.cache_fill(a16.float().cpu().numpy(), lens=lens[[5]], as_bf16=(dtype == "bf16"))
    np.testing.assert_array_equal(sess.cache_block(5).ravel().view(np.uint16 if dtype == "bf16" else np.uint32),
                                  exp16.view(np.uint16 if dtype == "bf16" else np.uint32))


# ---------------------------------------------------------------------------
# a1-a4: forward, head, loss, reverse pass
# ---------------------------------------------------------------------------
SMALL = [
    # several 64-row tiles with a ragged tail, r and d spanning more than one 64-column tile
    Workload("s1", L=3, d=160, n_max=37, B=5, r=96, C=3, N=5, cache_dtype="f32", len_lo=9),
    Workload("s2", L=2, d=64, n_max=70, B=3, r=32, C=2, N=3, cache_dtype="f32"),
    Workload("s3", L=3, d=160, n_max=37, B=5, r=96, C=3, N=5, cache_dtype="bf16", len_lo=9),
    Workload("s4", L=4, d=256, n_max=64, B=8, r=32, C=4, N=8, cache_dtype="bf16"),
    Workload("s5", L=1, d=32, n_max=1, B=1, r=32, C=1, N=1, cache_dtype="f32"),      # degenerate: one token
]


@pytest.mark.parametrize("w", SMALL, ids=[w.name for w in SMALL])
@pytest.mark.parametrize("state", ["init", "random"])
def test_loss_grad_small(w, state):
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    params = inputs.init_params(w) if state == "init" else inputs.random_params(w)
    sess = make_session(w, lens=lens)
    sess.cache_fill(ids, acts, lens)
    ref, loss, grads, worst = check_against_oracle(w, sess, ids, acts, lens, labels, params, TOL[w.cache_dtype],
                                                   what=f"{w.name}/{state}")
    if state == "init":
        dims = orc.Dims(w.L, w.d, w.r, w.C)
        sl = orc.param_slices(dims)
        for l in range(w.L):
            for nm in (f"W_down{l}", f"c_down{l}", f"lambda{l}"):
                assert np.all(ref["grads"][sl[nm]] == 0.0)
                assert np.all(grads[sl[nm]] == 0.0), nm


# The bf16 configurations above run on the Gram-matrix formulation where it applies; the shapes
# below exercise its tile variants (adapter width 32..128, one layer, ragged 32-token tiles,
# hidden sizes that are not multiples of 64), and the per-layer kernels are forced for the same inputs.
GRAM = [
    Workload("g1", L=1, d=96, n_max=45, B=3, r=32, C=2, N=3, cache_dtype="bf16", len_lo=1),
    Workload("g2", L=5, d=128, n_max=70, B=4, r=64, C=3, N=4, cache_dtype="bf16", len_lo=20),
    Workload("g3", L=3, d=224, n_max=33, B=6, r=128, C=5, N=6, cache_dtype="bf16", len_lo=30),
    Workload("g4", L=6, d=192, n_max=64, B=2, r=96, C=16, N=2, cache_dtype="bf16"),
    # as many layers and as wide an adapter as the Large-shaped configuration: the chain kernels' LDS near its limit
    Workload("g5", L=24, d=128, n_max=40, B=3, r=128, C=2, N=3, cache_dtype="bf16", len_lo=17),
]


# Adapter widths above 128: the Gram-matrix formulation with one chain launch per layer and 128 x 128
# workgroup tiles (widths that are and are not multiples of 64, several column tiles, ragged rows).
WIDE = [
    Workload("w1", L=3, d=160, n_max=37, B=5, r=160, C=3, N=5, cache_dtype="bf16", len_lo=9),
    Workload("w2", L=5, d=256, n_max=70, B=4, r=256, C=4, N=4, cache_dtype="bf16", len_lo=20),
    Workload("w3", L=9, d=192, n_max=150, B=3, r=192, C=2, N=3, cache_dtype="bf16", len_lo=100),
    Workload("w4", L=6, d=96, n_max=50, B=3, r=224, C=16, N=3, cache_dtype="bf16", len_lo=3),
]


@pytest.mark.parametrize("w", GRAM + WIDE, ids=[w.name for w in GRAM + WIDE])
@pytest.mark.parametrize("flags", [0, 1, 4], ids=["gram", "per_layer", "layer_chain"])
def test_bf16_paths(w, flags):
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    sess = make_session(w, lens=lens, flags=flags)
    sess.cache_fill(ids, acts, lens)
    check_against_oracle(w, sess, ids, acts, lens, labels, inputs.random_params(w, up_scale=0.5), TOL["bf16"],
                         what=f"{w.name}/flags{flags}")
    ref, loss, grads, _ = check_against_oracle(w, sess, ids, acts, lens, labels, inputs.init_params(w), TOL["bf16"],
                                               what=f"{w.name}/flags{flags}/init")
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    sl = orc.param_slices(dims)
    for l in range(w.L):
        for nm in (f"W_down{l}", f"c_down{l}", f"lambda{l}"):
            assert np.all(grads[sl[nm]] == 0.0), nm


# Adapter widths above 256 (the long-sequence configuration's r = 512): the Gram-matrix formulation in multiples of
# 64 up to 512 (two column tiles of the 256-wide workgroup tiles, groups of two or three layers), per-layer
# kernels otherwise.
XWIDE = [
    (Workload("x1", L=3, d=160, n_max=70, B=4, r=512, C=2, N=4, cache_dtype="bf16", len_lo=20), 2),
    (Workload("x2", L=4, d=96, n_max=37, B=3, r=288, C=3, N=3, cache_dtype="bf16", len_lo=9), 0),
    (Workload("x3", L=7, d=192, n_max=150, B=3, r=320, C=3, N=3, cache_dtype="bf16", len_lo=100), 2),
    (Workload("x4", L=5, d=256, n_max=50, B=5, r=448, C=16, N=5, cache_dtype="bf16", len_lo=3), 2),
    (Workload("x5", L=9, d=128, n_max=90, B=24, r=384, C=4, N=24, cache_dtype="bf16", len_lo=1), 2),
]


@pytest.mark.parametrize("w,path", XWIDE, ids=[w.name for w, _ in XWIDE])
@pytest.mark.parametrize("flags", [0, 1], ids=["default", "per_layer"])
def test_bf16_widths_above_256(w, path, flags):
    from paper_2408_10746_amd import binding as pb
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    sess = make_session(w, lens=lens, flags=flags)
    assert pb.pac_step_path(sess.ctx) == (0 if flags else path)
    sess.cache_fill(ids, acts, lens)
    check_against_oracle(w, sess, ids, acts, lens, labels, inputs.random_params(w, up_scale=0.5), TOL["bf16"],
                         what=f"{w.name}/flags{flags}")
    ref, loss, grads, _ = check_against_oracle(w, sess, ids, acts, lens, labels, inputs.init_params(w), TOL["bf16"],
                                               what=f"{w.name}/flags{flags}/init")
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    sl = orc.param_slices(dims)
    for l in range(w.L):
        for nm in (f"W_down{l}", f"c_down{l}", f"lambda{l}"):
            assert np.all(grads[sl[nm]] == 0.0), nm


@pytest.mark.parametrize("wname", ["g2", "w2", "x1"])
@pytest.mark.parametrize("flags", [0, 1, 4], ids=["gram", "per_layer", "layer_chain"])
def test_forward_only_call(flags, wname):
    """loss and logits without gradients (no backward launches; the gradient buffer stays untouched)."""
    w = {x.name: x for x in GRAM + WIDE + [x for x, _ in XWIDE]}[wname]
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    params = inputs.random_params(w, up_scale=0.5)
    dims, ref = oracle_batch(w, acts, lens, labels, params, want_grads=False)
    sess = make_session(w, lens=lens, flags=flags)
    sess.cache_fill(ids, acts, lens)
    sess.set_params(params)
    sess.grads.fill_(123.0)
    sess.loss_grad(ids, torch.from_numpy(labels).to(sess.dev), want_grads=False)
    torch.cuda.synchronize()
    loss = float(sess.loss.item())
    logits = sess.logits.cpu().numpy()[: w.B * w.C].reshape(w.B, w.C)
    assert abs(loss - ref["loss"]) <= TOL["bf16"] * abs(ref["loss"]), (loss, ref["loss"])
    assert rel_err(logits, ref["logits"]) <= TOL["bf16"]
    assert torch.all(sess.grads == 123.0)


def test_maximum_batch_many_ragged_tiles():
    """64 samples (the largest batch the kernel argument block describes), lengths from 1 to 100:
    more than 200 token tiles, most of them ragged, several samples of a single token."""
    w = Workload("gmax", L=4, d=128, n_max=100, B=64, r=64, C=3, N=64, cache_dtype="bf16", len_lo=1)
    lens = inputs.lengths(w)
    lens[:3] = 1
    lens[3] = 100
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    sess = make_session(w, lens=lens)
    sess.cache_fill(ids, acts, lens)
    check_against_oracle(w, sess, ids, acts, lens, labels, inputs.random_params(w, up_scale=0.5), TOL["bf16"],
                         what="gmax")


@pytest.mark.parametrize("w", [GRAM[1], GRAM[3], WIDE[1], WIDE[2], XWIDE[2][0]], ids=["g2", "g4", "w2", "w3", "x3"])
def test_training_step_loss_and_gate_gradients(w):
    """In a training step the optimizer launch does the last two ordered sums (loss, gate gradients):
    both must equal what the gradient call reports, bit for bit, and match the oracle."""
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    params = inputs.random_params(w, up_scale=0.5)
    sess = make_session(w, lens=lens)
    sess.cache_fill(ids, acts, lens)
    ref, loss_lg, grads_lg, _ = check_against_oracle(w, sess, ids, acts, lens, labels, params, TOL["bf16"],
                                                     what=f"{w.name}/loss_grad")
    sess.set_params(params)
    sess.grads.zero_()
    sess.step(ids, torch.from_numpy(labels).to(sess.dev), keep_grads=True)
    torch.cuda.synchronize()
    assert float(sess.loss.item()) == loss_lg
    assert np.array_equal(sess.grads.cpu().numpy(), grads_lg)
    # and the parameters moved as AdamW says they should from those gradients
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    p, m, v = params.astype(np.float64), np.zeros(dims.P), np.zeros(dims.P)
    hp = sess.hp
    orc.adamw(dims, p, m, v, 1, grads_lg.astype(np.float64),
              orc.AdamW(lr=hp.lr, beta1=hp.beta1, beta2=hp.beta2, eps=hp.eps, weight_decay=hp.weight_decay))
    assert np.max(np.abs(sess.params.cpu().numpy() - p)) <= 1e-6


def test_wide_adapter_many_ragged_tiles_and_groups():
    """r = 256 with more layers than two chain groups of four, 40 samples of 1..90 tokens (row tiles of the
    128-row contractions end inside samples, the last one is short), a single-token sample first and last."""
    w = Workload("wmax", L=10, d=128, n_max=90, B=40, r=256, C=3, N=40, cache_dtype="bf16", len_lo=1)
    lens = inputs.lengths(w)
    lens[0] = lens[-1] = 1
    lens[1] = 90
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    sess = make_session(w, lens=lens)
    sess.cache_fill(ids, acts, lens)
    check_against_oracle(w, sess, ids, acts, lens, labels, inputs.random_params(w, up_scale=0.5), TOL["bf16"],
                         what="wmax")


def test_outlier_channels_bf16():
    w = Workload("out", L=3, d=512, n_max=40, B=4, r=64, C=4, N=4, cache_dtype="bf16", outlier_frac=0.01)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    assert np.abs(acts).max() > 20.0
    labels = inputs.labels(w)[ids]
    sess = make_session(w)
    sess.cache_fill(ids, acts)
    check_against_oracle(w, sess, ids, acts, None, labels, inputs.random_params(w, up_scale=0.25), TOL["bf16"], "outliers")


def test_subset_and_order_of_cached_samples():
    """A step may address any filled samples in any order (batch gather)."""
    w = Workload("gather", L=2, d=64, n_max=19, B=4, r=32, C=3, N=10, cache_dtype="f32", len_lo=5)
    lens = inputs.lengths(w)
    acts = inputs.batch_acts(w, range(w.N))
    sess = make_session(w, lens=lens)
    sess.cache_fill(np.arange(w.N), acts, lens)
    ids = np.array([7, 2, 9, 0])
    labels = inputs.labels(w)[ids]
    check_against_oracle(w, sess, ids, acts[ids], lens[ids], labels, inputs.random_params(w), TOL["f32"], "gather")
    # a smaller batch than B_max
    ids = np.array([3, 8])
    labels = inputs.labels(w)[ids]
    check_against_oracle(w, sess, ids, acts[ids], lens[ids], labels, inputs.random_params(w), TOL["f32"], "gather2")


@pytest.mark.parametrize("w", [SMALL[2], WIDE[2], XWIDE[3][0]], ids=["s3", "w3", "x4"])
def test_bitwise_reproducible(w):
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    sess = make_session(w, lens=lens)
    sess.cache_fill(ids, inputs.batch_acts(w, ids), lens)
    sess.set_params(inputs.random_params(w))
    lab = torch.from_numpy(inputs.labels(w)[ids]).cuda()
    sess.loss_grad(ids, lab)
    g1, l1 = sess.grads.clone(), sess.loss.clone()
    sess.grads.zero_()
    sess.loss_grad(ids, lab)
    torch.cuda.synchronize()
    assert torch.equal(g1, sess.grads) and torch.equal(l1, sess.loss)


# ---------------------------------------------------------------------------
# a5 + whole step: the Tiny configuration end to end (fp32 mode)
# ---------------------------------------------------------------------------
def test_tiny_config_three_epochs():
    w = inputs.WORKLOADS["tiny"]
    tol = TOL["f32"]
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    acts = inputs.batch_acts(w, range(w.N))
    labels = inputs.labels(w)
    cache, off, lens = orc.cache_fill(acts, as_bf16=False)
    p = inputs.init_params(w).astype(np.float64)
    m, v, t = np.zeros(dims.P), np.zeros(dims.P), 0
    hp = orc.AdamW()
    sess = make_session(w)
    sess.cache_fill(np.arange(w.N), acts)
    sess.set_params(inputs.init_params(w))
    lab_all = torch.from_numpy(labels).cuda()
    k = 0
    worst_same_state = 0.0
    for e in range(w.epochs):
        order = inputs.epoch_order(w, e)
        for b in range(w.N // w.B):
            ids = order[b * w.B:(b + 1) * w.B]
            k += 1
            check = k in (1, 2, 9, 24)
            # the state this step's gradient is taken at, as the device holds it
            p_dev = sess.params.cpu().numpy().astype(np.float64) if check else None
            loss_ref, g_ref, t = orc.step(dims, cache, off[ids], lens[ids], labels[ids], p, m, v, t, hp)
            sess.step(ids, lab_all[torch.from_numpy(ids).cuda()].contiguous())
            loss = float(sess.loss.item())
            # the loss along the two trajectories (fp32 on the device, fp64 in the oracle)
            assert abs(loss - loss_ref) <= tol * abs(loss_ref), (k, loss, loss_ref)
            if check:
                # Loss and gradients at the SAME state: the oracle evaluated at the device's own parameters, so
                # that the drift between an fp32 and an fp64 AdamW trajectory plays no part and the stated
                # tolerance applies as it stands.
                same = orc.loss_grad(dims, cache, off[ids], lens[ids], labels[ids], p_dev)
                assert abs(loss - same["loss"]) <= tol * abs(same["loss"]), (k, loss, same["loss"])
                g = sess.grads.cpu().numpy()
                for name, sl in tensors(dims).items():
                    err = rel_err(g[sl], same["grads"][sl])
                    worst_same_state = max(worst_same_state, err)
                    assert err <= tol, (k, name, err)
                check_gates(dims, g, same, tol, f"tiny step {k}")
    assert k == 24 and sess.step_count == 24
    note(f"tiny: worst same-state gradient error {worst_same_state:.2e}")
    # Final parameters of the two trajectories.  An update moves an entry by lr * u, u = mhat / (sqrt(vhat) + eps),
    # and a relative gradient error delta changes u by about 2 delta |u| where the entry's gradients keep their
    # scale (numerator and denominator move together), by up to delta |g| / sqrt(vhat) <= delta / sqrt(1 - beta2)
    # where they do not: with delta <= 1e-5, K = 24 steps and entries that moved by about K lr, the difference
    # stays below K lr delta / sqrt(1 - beta2) = 7.6e-6 absolute per entry, i.e. below 10 x the tolerance relative
    # to tensors whose entries moved by K lr / 3 or more (all of them here: zero-initialised tensors have moved
    # that far, the others are larger).  Measured: about 2e-6.
    pg = sess.params.cpu().numpy()
    worst_drift = 0.0
    for name, sl in tensors(dims).items():
        worst_drift = max(worst_drift, rel_err(pg[sl], p[sl]))
        assert rel_err(pg[sl], p[sl]) <= 10 * tol, (name, rel_err(pg[sl], p[sl]))
    note(f"tiny: worst final-parameter difference between the trajectories {worst_drift:.2e}")


def test_adamw_single_step_and_resume():
    """One update from the same state matches the oracle; saving and restoring (params, m, v, step)
    continues bit-identically."""
    w = SMALL[0]
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    labels = inputs.labels(w)[ids]
    lab = torch.from_numpy(labels).cuda()
    sess = make_session(w, lens=lens)
    sess.cache_fill(ids, acts, lens)
    p0 = inputs.random_params(w)
    cache, off, lens_a = orc.cache_fill(acts, lens=lens, as_bf16=False)
    p, m, v = p0.astype(np.float64), np.zeros(dims.P), np.zeros(dims.P)
    t = 0
    sess.set_params(p0)
    for _ in range(3):
        _, _, t = orc.step(dims, cache, off, lens_a, labels, p, m, v, t, orc.AdamW())
        sess.step(ids, lab)
    pg, mg, vg = sess.params.cpu().numpy(), sess.m.cpu().numpy(), sess.v.cpu().numpy()
    for name, sl in tensors(dims).items():
        assert rel_err(pg[sl], p[sl]) <= 1e-5, name
        assert rel_err(mg[sl], m[sl]) <= 1e-4, name
        assert rel_err(vg[sl], v[sl]) <= 1e-4, name
    saved = (sess.params.clone(), sess.m.clone(), sess.v.clone(), sess.step_count)
    sess.step(ids, lab)
    after = sess.params.clone()
    sess.params.copy_(saved[0]); sess.m.copy_(saved[1]); sess.v.copy_(saved[2]); sess.step_count = saved[3]
    sess.step(ids, lab)
    torch.cuda.synchronize()
    assert torch.equal(after, sess.params)


# ---------------------------------------------------------------------------
# full-size configurations
# ---------------------------------------------------------------------------
def _full_size(name, n_fill, B_check=None, steps_before=0):
    w = inputs.WORKLOADS[name]
    lens_all = inputs.lengths(w)
    ids_fill = np.arange(n_fill)
    from paper_2408_10746_amd.runtime import Session
    sess = Session(w, cache_samples=n_fill, lens=lens_all[:n_fill] if w.len_lo else None)
    note(f"{name}: filling {n_fill} samples")
    for s in ids_fill:                                     # one sample at a time keeps host memory small
        sess.cache_fill([int(s)], inputs.batch_acts(w, [s]), lens_all[[s]] if w.len_lo else None)
    labels = inputs.labels(w)
    lab_all = torch.from_numpy(labels).cuda()
    sess.set_params(inputs.init_params(w))
    for k in range(steps_before):                          # move away from the zero-initialised state
        ids = np.roll(ids_fill, -k * w.B)[:w.B]
        sess.step(ids, lab_all[torch.from_numpy(ids).cuda()].contiguous(), keep_grads=False)
    torch.cuda.synchronize()
    params = sess.params.cpu().numpy().copy()
    ids = ids_fill[:w.B] if B_check is None else ids_fill[:B_check]
    return w, sess, ids, lens_all, labels, params


@pytest.mark.parametrize("steps_before", [0, 12])
def test_t5base_full_batch(steps_before):
    """The benchmark's configuration and launch shape (B=32 x 128 tokens, d=768, r=96, L=12)."""
    w, sess, ids, lens_all, labels, params = _full_size("t5base", 64, steps_before=steps_before)
    acts = inputs.batch_acts(w, ids)
    if steps_before:
        dims = orc.Dims(w.L, w.d, w.r, w.C)
        sl = orc.param_slices(dims)
        assert np.abs(params[sl["W_up0"]]).max() > 0
    check_against_oracle(w, sess, ids, acts, None, labels[ids], params, TOL["bf16"], f"t5base/{steps_before}")


@pytest.mark.parametrize("steps_before", [0, 12])
def test_large_full_batch(steps_before):
    """The BART/T5-Large-shaped configuration at its own launch shape (B=32 x 128 tokens, d=1024, r=128, L=24:
    the single-launch chains with a 16-token tile's history of all 24 layers in LDS), whole batch against the oracle."""
    from paper_2408_10746_amd import binding as pb
    w, sess, ids, lens_all, labels, params = _full_size("large", 32, steps_before=steps_before)
    assert pb.pac_step_path(sess.ctx) == 1
    acts = inputs.batch_acts(w, ids)
    if steps_before:
        dims = orc.Dims(w.L, w.d, w.r, w.C)
        assert np.abs(params[orc.param_slices(dims)["W_up0"]]).max() > 0
    check_against_oracle(w, sess, ids, acts, None, labels[ids], params, TOL["bf16"], f"large/{steps_before}")


def test_t5base_batch_behind_four_giga_elements():
    """Cache blocks at high offsets: the 32 checked samples sit behind more than 2^32 cache elements of filler
    (3700 samples written from one reused device buffer), so every row offset of the step exceeds 32 bits."""
    from paper_2408_10746_amd import binding as pb
    from paper_2408_10746_amd.runtime import Session
    w = inputs.WORKLOADS["t5base"]
    n_fill, chunk = 3700, 50
    sess = Session(w, cache_samples=n_fill + w.B)
    note(f"high offsets: {n_fill} filler samples + {w.B} checked ones, {sess.cache_bytes / 1e9:.2f} GB")
    filler = torch.from_numpy(inputs.batch_acts(w, range(1000, 1000 + chunk))).cuda()
    for s0 in range(0, n_fill, chunk):
        sess.cache_fill(np.arange(s0, s0 + chunk), filler)
    ids = np.arange(n_fill, n_fill + w.B)
    acts = inputs.batch_acts(w, ids)
    sess.cache_fill(ids, acts)
    torch.cuda.synchronize()
    off0, _ = pb.pac_cache_lookup(sess.ctx, int(ids[0]))
    assert off0 >= 1 << 32
    exp, _, _ = orc.cache_fill(acts[:1], as_bf16=True)
    np.testing.assert_array_equal(sess.cache_block(int(ids[0])).ravel(), exp)   # the fill itself, bit for bit
    labels = inputs.labels(w)
    check_against_oracle(w, sess, ids, acts, None, labels[ids], inputs.random_params(w, up_scale=0.5), TOL["bf16"],
                         "t5base/high offsets")


@pytest.mark.parametrize("wname", ["g2", "g5", "w2", "x3"])
def test_split_launches_match_fused_launches_bitwise(wname):
    """PAC_FLAG_SPLIT_LAUNCH (the form the per-part profiles are taken in) only changes how the parts of the fused
    launches are dispatched: loss, logits and gradients must equal the default form's bit for bit."""
    w = {x.name: x for x in GRAM + WIDE + [x for x, _ in XWIDE]}[wname]
    lens = inputs.lengths(w)
    ids = np.arange(w.B)
    acts = inputs.batch_acts(w, ids)
    lab = torch.from_numpy(inputs.labels(w)[ids]).cuda()
    params = inputs.random_params(w, up_scale=0.5)
    got = []
    for flags in (0, 2):
        sess = make_session(w, lens=lens, flags=flags)
        sess.cache_fill(ids, acts, lens)
        sess.set_params(params)
        sess.loss_grad(ids, lab)
        torch.cuda.synchronize()
        got.append((sess.loss.clone(), sess.logits.clone(), sess.grads.clone()))
    for a, b in zip(got[0], got[1]):
        assert torch.equal(a, b)


@pytest.mark.timeout(1500)
def test_llama7b_shape_full_batch():
    """d=4096, r=256, L=32, 256-token samples with outlier channels: the whole 16-sample batch (the launch shape
    the benchmark times: 4096 token rows) against the oracle (1.65 TFLOP in plain loops: a minute or so)."""
    w, sess, ids, lens_all, labels, params = _full_size("llama7b", 16, steps_before=2)
    acts = inputs.batch_acts(w, ids)
    check_against_oracle(w, sess, ids, acts, None, labels[ids], params, TOL["bf16"], "llama7b/full batch")
    del acts

    # The launch configuration bench.py times is the full batch (16 samples, 4096 token rows: 256 chain tiles,
    # 32 row tiles of the wide contractions), which the oracle would take minutes for.  A property that holds at
    # any size instead: loss and gradients are batch means, so the full batch must equal the mean of its two
    # halves, whose launch shapes differ from the full one's (and from the oracle-checked two-sample one's).
    def run(sel):
        sess.set_params(params)
        sess.grads.zero_()
        sess.loss_grad(np.asarray(sel), torch.from_numpy(labels[sel]).to(sess.dev))
        torch.cuda.synchronize()
        return float(sess.loss.item()), sess.grads.cpu().numpy().astype(np.float64)

    full = np.arange(16)
    l_full, g_full = run(full)
    l_a, g_a = run(full[:8])
    l_b, g_b = run(full[8:])
    assert abs(l_full - 0.5 * (l_a + l_b)) <= 1e-4 * abs(l_full)
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    sl = orc.param_slices(dims)
    g_half = 0.5 * (g_a + g_b)
    for l in (0, 15, 31):
        for nm in (f"W_down{l}", f"c_down{l}", f"W_up{l}", f"c_up{l}"):
            e = rel_err(g_full[sl[nm]], g_half[sl[nm]])
            note(f"llama7b full vs halves {nm}: {e:.2e}")
            assert e <= 5e-3, (nm, e)
    assert rel_err(g_full[sl["W_cls"]], g_half[sl["W_cls"]]) <= 5e-3


@pytest.mark.timeout(1800)
def test_longseq_shape_ragged_full_batch():
    """d=4096, r=512, L=32, samples of 256..1024 tokens packed without padding: the widest adapter the Gram-matrix
    formulation takes, at its largest shape.  The whole ragged eight-sample batch (the launch shape the benchmark
    times) against the oracle, then the batch-mean property as an extra."""
    from paper_2408_10746_amd import binding as pb
    w, sess, ids8, lens_all, labels, trained = _full_size("longseq", 8, steps_before=2)
    assert pb.pac_step_path(sess.ctx) == 2
    # Two updates of a 4096-wide classifier on eight samples already separate them (loss about 1e-9: softmax minus
    # one-hot is then below fp32 resolution and a relative comparison of gradients says nothing), so the trained
    # state only shows that the update ran at this size; the comparison uses random parameters of ordinary scale.
    assert np.all(np.isfinite(trained)) and np.any(trained != inputs.init_params(w))
    params = inputs.random_params(w, up_scale=0.5)
    lens8 = lens_all[:8]
    assert lens8.min() < lens8.max() and lens8.max() <= w.n_max
    acts = inputs.batch_acts(w, ids8)
    check_against_oracle(w, sess, ids8, acts, lens_all[ids8], labels[ids8], params, TOL["bf16"], "longseq/full batch")
    del acts

    def run(sel):
        sess.set_params(params)
        sess.grads.zero_()
        sess.loss_grad(np.asarray(sel), torch.from_numpy(labels[sel]).to(sess.dev))
        torch.cuda.synchronize()
        return float(sess.loss.item()), sess.grads.cpu().numpy()

    dims = orc.Dims(w.L, w.d, w.r, w.C)
    sl = orc.param_slices(dims)
    names = [f"{nm}{l}" for l in (0, 16, 31) for nm in ("W_down", "c_down", "W_up", "c_up")] + ["W_cls"]
    l_full, g = run(ids8)
    g_full = {nm: g[sl[nm]].astype(np.float64) for nm in names}
    l_a, g = run(ids8[:4])
    g_half = {nm: 0.5 * g[sl[nm]].astype(np.float64) for nm in names}
    l_b, g = run(ids8[4:])
    for nm in names:
        g_half[nm] += 0.5 * g[sl[nm]]
    del g
    assert abs(l_full - 0.5 * (l_a + l_b)) <= 1e-4 * abs(l_full)
    for nm in names:
        e = rel_err(g_full[nm], g_half[nm])
        note(f"longseq full vs halves {nm}: {e:.2e}")
        assert e <= 5e-3, (nm, e)
