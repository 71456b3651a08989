#!/usr/bin/env python3
"""Benchmark of the cached Parallel-Adapter training step on one MI355X.

A "step" is one pass of the whole hot path (batch gather, adapter forward, pooled head +
cross-entropy, reverse pass, AdamW) over one batch read from an HBM-resident activation cache.
Prints ONE JSON line.  The headline (`value`, `roofline`, `cpu_baseline`) is the T5-Base-shaped
configuration; `configs` carries the other configurations of the same path (Large-, LLaMA-7B- and
long-sequence-shaped), each with its own step time and roofline fractions, so that both halves of the
metric (HBM rate on the cache stream, MFMA rate on the adapter contractions) are in the one line.
Kernel durations come from HIP events the library records around each launch on the stream it
launches on; `measured_peak` from the library's two probes (a plain read of the resident cache, a
register-only loop of matrix instructions) timed the same way.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
CACHE_PASS_CLASSES = ("g_proj", "g_tokred", "fwd_down", "bwd_wgrad")


def kernel_models(w, M):
    """Algorithmic work of one step's launches of each kernel class: (HBM bytes, flops).
    (The per-layer classes launch once per layer; the layer-by-layer chains of the wide-adapter
    path launch several kernels per layer; every other class is one launch per step.)

    Bytes are what the method must move for that piece of the step (cache slab of the layer,
    saved pre-activations, parameters/gradients), not what a particular kernel happens to
    re-read; flops are those of the dense contractions."""
    d, r, L, B, C = w.d, w.r, w.L, w.B, w.C
    slab = M * d * 2                       # one layer of the batch's cache slice, bf16
    pre = M * r * 4
    PL = 2 * d * r + r + d + 1
    pairs = L * (L - 1) // 2
    return {
        "fwd_down": (L * (slab + pre), 2.0 * M * d * r * L),
        "fwd_up": (0, 2.0 * M * d * r * L),
        "bwd_dpre": (L * pre, 2.0 * M * d * r * L),
        "bwd_wgrad": (L * (slab + PL * 4), 4.0 * M * d * r * L),
        "bwd_dx": (L * slab, 2.0 * M * d * r * L),
        "adamw": (w.P * 28, 12.0 * w.P),
        "reduce": (L * PL * 4, 0.0),
        "shadows": (w.P * 4, 0.0),
        "pool": (slab, 0.0),
        "head": (B * d * 4, 2.0 * B * d * C),
        "head_bwd": (0, 2.0 * B * d * C),
        "setup": (0, 0.0),
        # Gram-matrix path: the two cache passes are g_proj (U = b W_down, all layers) and
        # g_tokred (E = b^T dpre, all layers, plus the h^T dpre Gram matrix)
        "g_prep": (w.P * 4, 0.0),
        "g_proj": (L * (slab + pre), 2.0 * M * d * r * L + 2.0 * r * r * d * pairs),
        "g_chain_fwd": (2 * L * pre + L * M * r * 2, 2.0 * M * r * r * pairs),
        "g_head": (B * d * 4, 2.0 * B * (d + L * r) * C),
        "g_chain_bwd": (L * pre + L * M * r * 2, 2.0 * M * r * r * pairs),
        "g_tokred": (L * slab + 2 * L * M * r * 2, 2.0 * M * d * r * L + 2.0 * M * r * r * pairs),
        "g_ggsum": (0, 0.0),
        "g_post": (w.P * 4, 4.0 * d * r * r * pairs),
        "g_finish": (0, 0.0),
        # fused streaming path (adapter widths up to 128): forward cache pass with the projection and the
        # forward chain in one launch; backward chain; second cache pass with the token reductions
        "g_fwd": (L * slab + L * M * r * 4, 2.0 * M * d * r * L + 2.0 * M * r * r * pairs),
        "g_bwd": (L * slab + 2 * L * M * r * 2, 2.0 * M * d * r * L + 2.0 * M * r * r * pairs),
    }


def roofline_of(cls, ms_total, launches, prof_steps, models, measured):
    """Roofline entry of one kernel class from its event-timed launches."""
    abytes, aflops = models[cls]
    step_s = ms_total * 1e-3 / prof_steps   # all of the class's launches of one step
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    if aflops and (abytes == 0 or aflops / abytes > ridge):
        r = {"bound": "mfma", "achieved": aflops / step_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
        mp = measured.get("mfma_bf16_TFLOPs") if measured else None
    else:
        r = {"bound": "hbm", "achieved": abytes / step_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        mp = measured.get("hbm_read_GBs") if measured else None
    r["frac"] = r["achieved"] / r["peak"]
    r["frac_of_measured_peak"] = (r["achieved"] / mp) if mp else None
    r["kernel"] = cls
    r["avg_launch_us"] = ms_total * 1e3 / launches
    r["launches_per_step"] = launches / prof_steps
    return r


def measure_peaks(torch, pb, sess, slice_bytes):
    """What the chip sustains, measured with the library's probes on the stream the step runs on:
    a plain read of 2 GiB of the resident cache (far more than any on-chip cache holds), a plain read of
    one step's worth of cache (a fresh region each repetition), and a register-only bf16 MFMA loop."""
    sink = torch.zeros(256, dtype=torch.float32, device=sess.dev)
    st = int(torch.cuda.current_stream().cuda_stream)
    out = {}

    def timed(fn, reps):
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i + 1)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    base = sess.cache.data_ptr()
    big = min(sess.cache_bytes // 2, 2 << 30) & ~255
    if big >= (64 << 20):
        nreg = max(1, sess.cache_bytes // big)
        t = timed(lambda i: pb.pac_probe_hbm_read(base + (i % nreg) * big, big, sink.data_ptr(), st), 6)
        out["hbm_read_GBs"] = big / t / 1e9
        out["hbm_read_bytes"] = big
    sl = int(slice_bytes) & ~255
    nsl = max(1, sess.cache_bytes // sl)
    if nsl >= 8:
        t = timed(lambda i: pb.pac_probe_hbm_read(base + ((i * 37) % nsl) * sl, sl, sink.data_ptr(), st), 24)
        out["slice_read_GBs"] = sl / t / 1e9
        out["slice_read_bytes"] = sl
    # the optimizer's access mix (four arrays read, three written back) on arrays of the LLaMA-7B-shaped parameter count,
    # far larger than any on-chip cache
    n = 67264548 & ~3
    arr = [torch.zeros(n, dtype=torch.float32, device=sess.dev) for _ in range(4)]
    t = timed(lambda i: pb.pac_probe_hbm_update(arr[0].data_ptr(), arr[1].data_ptr(), arr[2].data_ptr(), arr[3].data_ptr(), n, st), 6)
    out["update_stream_GBs"] = 28.0 * n / t / 1e9
    out["update_stream_bytes"] = 28 * n
    del arr
    iters = 20000
    t = timed(lambda i: pb.pac_probe_mfma_bf16(iters, sink.data_ptr(), st), 3)
    out["mfma_bf16_TFLOPs"] = pb.pac_probe_mfma_flops(iters) / t / 1e12
    return out


def run_workload(name, N, steps, warmup, flags, keep_cpu_samples=0, want_peaks=False):
    """Fill a cache of N samples on the device, time `steps` training steps, profile per kernel class."""
    import numpy as np
    import torch
    from paper_2408_10746_amd import binding as pb
    from paper_2408_10746_amd import inputs
    from paper_2408_10746_amd.runtime import Session

    w = inputs.WORKLOADS[name]
    N = N or w.N
    assert N % w.B == 0
    dev = torch.device("cuda:0")
    lens_all = inputs.lengths(w)[:N]
    sess = Session(w, cache_samples=N, lens=lens_all if w.len_lo else None, flags=flags)

    # ---- fill the cache on the device: N(0,1), per-token layer norm, optional outlier channels
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_DATA)
    chunk = max(1, min(64, (1 << 29) // (w.L * w.n_max * w.d * 4)))
    out_ch = torch.from_numpy(inputs.outlier_channels(inputs.SEED_DATA, w.d, w.outlier_frac)).to(dev)
    t_fill0 = time.perf_counter()
    keep_host = {}
    for s0 in range(0, N, chunk):
        ids = np.arange(s0, min(N, s0 + chunk))
        a = torch.randn((len(ids), w.L, w.n_max, w.d), generator=gen, device=dev, dtype=torch.float32)
        a = torch.nn.functional.layer_norm(a, (w.d,), eps=1e-5)
        if out_ch.numel():
            a[..., out_ch] *= w.outlier_scale
        a = a.contiguous()
        sess.cache_fill(ids, a, lens_all[ids] if w.len_lo else None)
        for s in range(keep_cpu_samples):
            if s0 <= s < s0 + len(ids):
                keep_host[s] = a[s - s0].cpu().numpy()
        del a
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t_fill0

    labels = inputs.labels(w)
    lab_dev = torch.from_numpy(labels).to(dev)
    sess.set_params(inputs.init_params(w))
    steps_per_epoch = N // w.B

    def batch_ids(k):
        e, b = divmod(k, steps_per_epoch)
        order = inputs.epoch_order(w, e)[:N] if N == w.N else np.arange(N)
        return order[b * w.B:(b + 1) * w.B]

    plan = [batch_ids(k) for k in range(warmup + steps)]
    labs = [lab_dev[torch.from_numpy(ids).to(dev)].contiguous() for ids in plan]

    for k in range(warmup):
        sess.step(plan[k], labs[k], keep_grads=False)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for k in range(warmup, warmup + steps):
        sess.step(plan[k], labs[k], keep_grads=False)
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps
    final_loss = float(sess.loss.item())
    assert np.isfinite(final_loss), "training diverged"

    # ---- per-kernel durations: the library records HIP events around each launch on its stream
    prof_steps = min(steps, 32)
    pb.pac_profile_begin(sess.ctx)
    for k in range(warmup, warmup + prof_steps):
        sess.step(plan[k], labs[k], keep_grads=False)
    prof = pb.pac_profile_end(sess.ctx)
    M = float(np.mean([lens_all[ids].sum() for ids in plan[warmup:warmup + prof_steps]]))
    models = kernel_models(w, M)
    slice_bytes = w.L * M * w.d * (2 if w.cache_dtype == "bf16" else 4)
    measured = measure_peaks(torch, pb, sess, slice_bytes) if want_peaks else None

    dom = max((c for c in prof if c in models), key=lambda c: prof[c][0])
    roof = roofline_of(dom, prof[dom][0], prof[dom][1], prof_steps, models, measured)
    passes = {c: roofline_of(c, prof[c][0], prof[c][1], prof_steps, models, measured)
              for c in CACHE_PASS_CLASSES if c in prof}
    step_bytes = 2 * slice_bytes + w.P * 32 + 2 * w.L * M * w.r * 4
    step_flops = 12.0 * M * w.d * w.r * w.L
    whole = {"hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "mfma_frac": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
             "algorithmic_MB": step_bytes / 1e6, "algorithmic_GFLOP": step_flops / 1e9,
             "kernel_ms_per_step": {c: prof[c][0] / prof_steps for c in prof}}
    res = {
        "workload": f"{w.name}: L={w.L} d={w.d} seq={w.n_max} B={w.B} r={w.r} C={w.C} "
                    f"N={N} resident ({sess.cache_bytes / 1e9:.2f} GB {w.cache_dtype} cache)",
        "N_resident": N, "N_config": w.N, "tokens_per_step": M, "cache_fill_s": t_fill,
        "formulation": ["per-layer kernels", "gram, single-launch chains", "gram, layer-by-layer chains",
                        "gram, fused streaming passes"][pb.pac_step_path(sess.ctx)],
        "steps": steps, "ms_per_step": ms_per_step, "samples_per_s": steps * w.B / elapsed,
        "gpu_event_ms_per_step": ev0.elapsed_time(ev1) / steps, "final_loss": final_loss,
        "roofline": roof, "cache_passes": passes, "whole_step": whole, "measured_peak": measured,
    }
    sess.close()
    return res, keep_host, lens_all, labels


def cpu_baseline(w, keep_host, lens_all, labels, cpu_ids, seconds, one_core=True):
    """The CPU oracle as it stands on a bounded sample of the workload: whole training steps on the same few
    samples, once on all host cores and once on one core."""
    import numpy as np
    from paper_2408_10746_amd import inputs
    from oracle import oracle as orc
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    acts = np.stack([keep_host[s] for s in cpu_ids])
    ln = lens_all[cpu_ids] if w.len_lo else None
    cache, off, lens_a = orc.cache_fill(acts, lens=ln, as_bf16=(w.cache_dtype == "bf16"))
    cache = orc.widen(cache)
    hp = orc.AdamW()
    all_cores = orc.num_threads()

    def leg(threads, budget):
        orc.set_num_threads(threads)
        p = inputs.init_params(w).astype(np.float64)
        m, v = np.zeros(dims.P), np.zeros(dims.P)
        c1 = time.perf_counter()
        n = 0
        while True:
            orc.step(dims, cache, off, lens_a, labels[cpu_ids], p, m, v, n, hp)
            n += 1
            c2 = time.perf_counter()
            if c2 - c1 >= budget or n >= 1000:
                break
        return {"value": n * len(cpu_ids) / (c2 - c1), "unit": "samples/s", "cores": threads, "kind": "oracle",
                "sample": f"{n} training steps (forward, loss, backward, AdamW) on {len(cpu_ids)} samples "
                          f"of the {w.name} workload, cache already in host memory; {c2 - c1:.1f} s"}

    out = leg(all_cores, seconds)
    if one_core:
        out["single_core"] = leg(1, seconds)
    orc.set_num_threads(all_cores)
    return out


def cpu_baseline_tiny():
    """The oracle on the whole Tiny run (3 epochs x 8 steps on 64 samples, fp32 cache), all cores and one core."""
    import numpy as np
    from paper_2408_10746_amd import inputs
    from oracle import oracle as orc
    w = inputs.WORKLOADS["tiny"]
    dims = orc.Dims(w.L, w.d, w.r, w.C)
    acts = inputs.batch_acts(w, range(w.N))
    labels = inputs.labels(w)
    cache, off, lens = orc.cache_fill(acts, as_bf16=False)
    hp = orc.AdamW()
    all_cores = orc.num_threads()
    out = {}
    for name, threads in (("all_cores", all_cores), ("single_core", 1)):
        orc.set_num_threads(threads)
        p = inputs.init_params(w).astype(np.float64)
        m, v, t = np.zeros(dims.P), np.zeros(dims.P), 0
        c1 = time.perf_counter()
        for e in range(w.epochs):
            order = inputs.epoch_order(w, e)
            for b in range(w.N // w.B):
                ids = order[b * w.B:(b + 1) * w.B]
                _, _, t = orc.step(dims, cache, off[ids], lens[ids], labels[ids], p, m, v, t, hp)
        el = time.perf_counter() - c1
        out[name] = {"value": t * w.B / el, "unit": "samples/s", "cores": threads, "kind": "oracle",
                     "sample": f"the whole Tiny run: {t} training steps of {w.B} samples; {el:.2f} s"}
    orc.set_num_threads(all_cores)
    return out


def bench_first_epoch_storage(torch, pb):
    """The first epoch's storage side on one backbone-sized projection (4096 x 4096, the LLaMA-7B shape's hidden size):
    block-wise quantisation (HBM-bound: 4 bytes read + 1 written per weight) and the mixed-precision linear layer on
    4096 token rows (matrix-bound: 2 M K N flops), each timed with events on the stream it runs on."""
    dev = torch.device("cuda:0")
    st = int(torch.cuda.current_stream().cuda_stream)
    N = K = M = 4096
    block = 64
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    W = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) / 64.0
    x = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    y = torch.empty((M, N), dtype=torch.float32, device=dev)
    consts = torch.empty(N * K // block, dtype=torch.float32, device=dev)
    out = {}

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    for bits in (8, 4):
        codes = torch.empty(N * K * bits // 8, dtype=torch.int8, device=dev)
        tq = timed(lambda: pb.pac_quant_blockwise(W.data_ptr(), N * K, block, bits, codes.data_ptr(), consts.data_ptr(), st), 20)
        tl = timed(lambda: pb.pac_dequant_linear(x.data_ptr(), M, K, codes.data_ptr(), consts.data_ptr(), N, block, bits,
                                                 y.data_ptr(), st), 10)
        qbytes = N * K * (4 + bits / 8) + consts.numel() * 4
        out[f"int{bits}"] = {
            "quantise": {"us": tq * 1e6, "bound": "hbm", "achieved": qbytes / tq / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": qbytes / tq / 1e9 / HBM_PEAK_GBS},
            "linear": {"us": tl * 1e6, "bound": "mfma", "achieved": 2.0 * M * K * N / tl / 1e12,
                       "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": 2.0 * M * K * N / tl / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        }
    out["shape"] = f"W {N}x{K} fp32 in blocks of {block}; linear layer on {M} bf16 token rows"
    return out


def bench_host_tier(torch, steps=48, warmup=8, N=512):
    """The T5-Base-shaped step with the cache in pinned host memory: batch k + 1 is reloaded into a device window on a
    copy stream while batch k trains (paper Sec. 5.2: the cache is reloaded per micro-batch from the larger tier).  Bound
    by the host link, not by HBM: the figure to read is the reload rate."""
    import numpy as np
    from paper_2408_10746_amd import inputs
    from paper_2408_10746_amd.runtime import TieredSession
    w = inputs.WORKLOADS["t5base"]
    dev = torch.device("cuda:0")
    sess = TieredSession(w, cache_samples=N)
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_DATA)
    for s0 in range(0, N, w.B):
        a = torch.randn((w.B, w.L, w.n_max, w.d), generator=gen, device=dev, dtype=torch.float32)
        a = torch.nn.functional.layer_norm(a, (w.d,), eps=1e-5).contiguous()
        sess.cache_fill(np.arange(s0, s0 + w.B), a)
    torch.cuda.synchronize()
    labels = torch.from_numpy(inputs.labels(w)).to(dev)
    sess.set_params(inputs.init_params(w))
    plan = [np.arange(w.B) + w.B * (k % (N // w.B)) for k in range(warmup + steps + 1)]
    labs = [labels[torch.from_numpy(ids).to(dev)].contiguous() for ids in plan]
    sess.prefetch(0, plan[0])
    t0 = None
    for k in range(warmup + steps):
        if k == warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        sess.prefetch(k + 1, plan[k + 1])
        sess.step_staged(k, plan[k], labs[k], keep_grads=False)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    slice_bytes = w.L * w.B * w.n_max * w.d * 2
    return {"workload": f"t5base, {N} samples in pinned host memory ({sess.cache_bytes / 1e9:.2f} GB), two device windows",
            "ms_per_step": el * 1e3 / steps, "samples_per_s": steps * w.B / el,
            "reload_GBs": slice_bytes * steps / el / 1e9, "reload_MB_per_step": slice_bytes / 1e6,
            "final_loss": float(sess.loss.item())}


def bench_ladder(torch, pb, steps=48, warmup=8, N=1024, heads=12):
    """The paper's default architecture (the w-wide ladder with a reduced transformer layer per adapter, Sec. 4.1) on the
    T5-Base-shaped cache: whole training steps, per-kernel-class durations, and the roofline of its two passes over the
    cache slice (fp32 matrix instructions: 157.3 TFLOP/s peak; the cache stream itself against 8 TB/s)."""
    import numpy as np
    from paper_2408_10746_amd import inputs
    from paper_2408_10746_amd.runtime import LadderSession
    from oracle import ladder_oracle as lo
    w = inputs.WORKLOADS["t5base"]
    dev = torch.device("cuda:0")
    sess = LadderSession(w, heads, cache_samples=N)
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_DATA)
    for s0 in range(0, N, w.B):
        a = torch.randn((w.B, w.L, w.n_max, w.d), generator=gen, device=dev, dtype=torch.float32)
        a = torch.nn.functional.layer_norm(a, (w.d,), eps=1e-5).contiguous()
        sess.cache_fill(np.arange(s0, s0 + w.B), a)
    torch.cuda.synchronize()
    labels = torch.from_numpy(inputs.labels(w)).to(dev)
    sess.set_params(lo.init_params(lo.LadderDims(w.L, w.d, w.r, heads, w.C), inputs.SEED_PARAMS))
    plan = [np.arange(w.B) + w.B * (k % (N // w.B)) for k in range(warmup + steps)]
    labs = [labels[torch.from_numpy(ids).to(dev)].contiguous() for ids in plan]
    for k in range(warmup):
        sess.step(plan[k], labs[k], keep_grads=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(warmup, warmup + steps):
        sess.step(plan[k], labs[k], keep_grads=False)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    final_loss = float(sess.loss.item())
    prof_steps = min(steps, 16)
    pb.pac_profile_begin(sess.ctx)
    for k in range(warmup, warmup + prof_steps):
        sess.step(plan[k], labs[k], keep_grads=False)
    prof = pb.pac_profile_end(sess.ctx)
    M, wd = w.B * w.n_max, w.r
    slab = w.L * M * w.d * 2
    # per token and layer: down-projection 2 d w, qkv 6 w^2, attention 4 n w, output projection 2 w^2, FFN 16 w^2;
    # the reverse pass costs twice the forward
    fwd_flops = w.L * M * (2.0 * w.d * wd + 24.0 * wd * wd + 4.0 * w.n_max * wd)
    act_bytes = w.L * M * wd * 4
    passes = {}
    for cls, abytes, aflops in (("l_down", slab + act_bytes, 2.0 * M * w.d * wd * w.L),
                                ("l_wgrad", slab + 13 * act_bytes, 2.0 * M * w.L * (w.d * wd + 12.0 * wd * wd))):
        if cls in prof:
            t = prof[cls][0] * 1e-3 / prof_steps
            passes[cls] = {"us": t * 1e6, "hbm_GBs": abytes / t / 1e9, "hbm_frac": abytes / t / 1e9 / HBM_PEAK_GBS}
            if cls == "l_down":
                # the bf16 cache times the projection written as three bf16 terms: 3 x the flops, on the bf16 matrix units
                passes[cls].update({"arithmetic": "bf16 x (bf16 hi + mid + lo), fp32 accumulation",
                                    "bf16_mfma_TFLOPs": 3.0 * aflops / t / 1e12,
                                    "bf16_mfma_frac": 3.0 * aflops / t / 1e12 / MFMA_BF16_PEAK_TFLOPS})
            else:
                passes[cls].update({"fp32_mfma_TFLOPs": aflops / t / 1e12, "fp32_mfma_frac": aflops / t / 1e12 / 157.3})
    sess.close()
    return {"workload": f"ladder on t5base: L={w.L} d={w.d} seq={w.n_max} B={w.B} w={wd} heads={heads} C={w.C}, "
                        f"{N} samples resident ({sess.cache_bytes / 1e9:.2f} GB bf16 cache), fp32 arithmetic "
                        f"(down-projection: exact bf16 products of the cache with a three-term bf16 split of the weights)",
            "ms_per_step": el * 1e3 / steps, "samples_per_s": steps * w.B / el, "final_loss": final_loss,
            "algorithmic_GFLOP": 3.0 * fwd_flops / 1e9, "cache_passes": passes,
            "kernel_ms_per_step": {c: prof[c][0] / prof_steps for c in prof},
            "launches_per_step": {c: prof[c][1] / prof_steps for c in prof}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="t5base")
    ap.add_argument("--samples", type=int, default=0, help="resident samples (0 = the workload's N)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations (headline workload only)")
    ap.add_argument("--only", default="", help="run one of the extra legs alone and print its JSON (ladder)")
    ap.add_argument("--flags", type=int, default=0, help="pac_config flags (1 per-layer kernels, 2 split launches)")
    ap.add_argument("--cpu-samples", type=int, default=4, help="samples per oracle step")
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="CPU time per leg of the oracle baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2408_10746_amd import inputs
    torch.cuda.set_device(0)
    if args.only == "ladder":
        from paper_2408_10746_amd import binding as pb
        print(json.dumps(bench_ladder(torch, pb)))
        return

    w = inputs.WORKLOADS[args.workload]
    ncpu = 0 if args.no_cpu_baseline else min(args.cpu_samples, w.B)
    head, keep_host, lens_all, labels = run_workload(args.workload, args.samples, args.steps, args.warmup, args.flags,
                                                     keep_cpu_samples=ncpu, want_peaks=True)
    roof = head["roofline"]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(roof["kernel"])
        except Exception:
            traffic = None
    roof["traffic"] = traffic
    roof["traffic_source"] = ("static: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary kept in profiles/traffic.json, "
                              "not measured in this run") if traffic else None
    roof["measured_peak"] = head["measured_peak"]
    roof["cache_passes"] = head["cache_passes"]

    cpu = None
    if ncpu:
        cpu = cpu_baseline(w, keep_host, lens_all, labels, list(range(ncpu)), args.cpu_seconds)
        if args.workload == "t5base" and not args.no_configs:
            cpu["tiny"] = cpu_baseline_tiny()
    del keep_host

    configs = {}
    if not args.no_configs and args.workload == "t5base" and not args.samples and not args.flags:
        for name, steps, warmup in (("large", 64, 8), ("llama7b", 24, 4), ("longseq", 12, 3)):
            gc.collect()
            torch.cuda.empty_cache()
            try:
                wl = inputs.WORKLOADS[name]
                ncpu_cfg = wl.B if (name == "llama7b" and not args.no_cpu_baseline) else 0
                res, kh, la, lb = run_workload(name, 0, steps, warmup, 0, keep_cpu_samples=ncpu_cfg)
                configs[name] = {k: res[k] for k in ("workload", "N_resident", "N_config", "tokens_per_step", "formulation",
                                                     "steps", "ms_per_step", "samples_per_s", "cache_fill_s",
                                                     "roofline", "cache_passes", "whole_step")}
                if ncpu_cfg:
                    # one whole step of this configuration in the oracle on all host cores (1.65 TFLOP: tens of seconds;
                    # the one-core leg would take minutes and is left out)
                    configs[name]["cpu_baseline"] = cpu_baseline(wl, kh, la, lb, list(range(ncpu_cfg)), 0.5, one_core=False)
                del kh
            except Exception as ex:  # the headline stays valid if another configuration cannot run on this machine
                configs[name] = {"error": f"{type(ex).__name__}: {ex}"}

    extras = {}
    if not args.no_configs:
        gc.collect()
        torch.cuda.empty_cache()
        try:
            from paper_2408_10746_amd import binding as pb
            extras["first_epoch_storage"] = bench_first_epoch_storage(torch, pb)
        except Exception as ex:
            extras["first_epoch_storage"] = {"error": f"{type(ex).__name__}: {ex}"}
        gc.collect()
        torch.cuda.empty_cache()
        try:
            extras["ladder"] = bench_ladder(torch, pb)
        except Exception as ex:
            extras["ladder"] = {"error": f"{type(ex).__name__}: {ex}"}
        gc.collect()
        torch.cuda.empty_cache()
        try:
            extras["host_tier"] = bench_host_tier(torch)
        except Exception as ex:
            extras["host_tier"] = {"error": f"{type(ex).__name__}: {ex}"}

    out = {
        "metric": "adapter-train samples/sec from activation cache",
        "value": head["samples_per_s"],
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.cache_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": head["workload"], "tokens_per_step": head["tokens_per_step"],
                   "cache_fill_s": head["cache_fill_s"], "formulation": head["formulation"],
                   "gpu_event_ms_per_step": head["gpu_event_ms_per_step"], "final_loss": head["final_loss"]},
        "roofline": roof,
        "whole_step": head["whole_step"],
        "cpu_baseline": cpu,
        "configs": configs,
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
