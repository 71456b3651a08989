#!/usr/bin/env python3
"""Benchmark of the cached Parallel-Adapter training step on one MI355X.

A "step" is one pass of the whole hot path (batch gather, adapter forward, pooled head +
cross-entropy, reverse pass, AdamW) over one batch read from an HBM-resident activation cache.
Prints ONE JSON line: whole-job samples/s, the roofline of the dominant kernel (measured with
HIP events recorded by the library on the stream it launches on) and the CPU oracle timed on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0


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
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="t5base")
    ap.add_argument("--samples", type=int, default=0, help="resident samples (0 = the workload's N)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--flags", type=int, default=0, help="pac_config flags (1 per-layer kernels, 2 split launches)")
    ap.add_argument("--cpu-samples", type=int, default=0, help="samples per oracle step (0 = one batch)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time to spend on the oracle baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2408_10746_amd import binding as pb
    from paper_2408_10746_amd import inputs
    from paper_2408_10746_amd.runtime import Session

    w = inputs.WORKLOADS[args.workload]
    N = args.samples or w.N
    assert N % w.B == 0
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lens_all = inputs.lengths(w)[:N]
    sess = Session(w, cache_samples=N, lens=lens_all if w.len_lo else None, flags=args.flags)

    # ---- fill the cache on the device: N(0,1), per-token layer norm, optional outlier channels
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_DATA)
    chunk = max(1, min(64, (1 << 29) // (w.L * w.n_max * w.d * 4)))
    out_ch = torch.from_numpy(inputs.outlier_channels(inputs.SEED_DATA, w.d, w.outlier_frac)).to(dev)
    t_fill0 = time.perf_counter()
    keep_host = {}
    cpu_ids = list(range(min(args.cpu_samples or w.B, w.B)))
    for s0 in range(0, N, chunk):
        ids = np.arange(s0, min(N, s0 + chunk))
        a = torch.randn((len(ids), w.L, w.n_max, w.d), generator=gen, device=dev, dtype=torch.float32)
        a = torch.nn.functional.layer_norm(a, (w.d,), eps=1e-5)
        if out_ch.numel():
            a[..., out_ch] *= w.outlier_scale
        a = a.contiguous()
        sess.cache_fill(ids, a, lens_all[ids] if w.len_lo else None)
        for s in cpu_ids:
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

    plan = [batch_ids(k) for k in range(args.warmup + args.steps)]
    labs = [lab_dev[torch.from_numpy(ids).to(dev)].contiguous() for ids in plan]

    for k in range(args.warmup):
        sess.step(plan[k], labs[k], keep_grads=False)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for k in range(args.warmup, args.warmup + args.steps):
        sess.step(plan[k], labs[k], keep_grads=False)
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    final_loss = float(sess.loss.item())
    assert np.isfinite(final_loss), "training diverged"

    # ---- per-kernel durations: the library records HIP events around each launch on its stream
    prof_steps = min(args.steps, 32)
    pb.pac_profile_begin(sess.ctx)
    for k in range(args.warmup, args.warmup + prof_steps):
        sess.step(plan[k], labs[k], keep_grads=False)
    prof = pb.pac_profile_end(sess.ctx)
    M = int(lens_all[plan[0]].sum())
    models = kernel_models(w, M)
    dom = max((c for c in prof if c in models), key=lambda c: prof[c][0])
    dom_ms, dom_n = prof[dom]
    avg_s = dom_ms * 1e-3 / dom_n
    step_s = dom_ms * 1e-3 / prof_steps   # all of the class's launches of one step
    abytes, aflops = models[dom]
    if aflops and (abytes == 0 or aflops / abytes > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)):
        roof = {"bound": "mfma", "achieved": aflops / step_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": abytes / step_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = dom
    roof["avg_launch_us"] = avg_s * 1e6
    roof["launches_per_step"] = dom_n / prof_steps
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(dom)
        except Exception:
            traffic = None
    roof["traffic"] = traffic
    step_bytes = 2 * w.L * M * d_bytes(w) + w.P * 32 + 2 * w.L * M * w.r * 4
    step_flops = 12.0 * M * w.d * w.r * w.L
    whole = {"hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "mfma_frac": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
             "kernel_ms_per_step": {c: prof[c][0] / prof_steps for c in prof}}

    # ---- the CPU oracle on a bounded sample of the same workload (one step on a few samples)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        dims = orc.Dims(w.L, w.d, w.r, w.C)
        acts = np.stack([keep_host[s] for s in cpu_ids])
        ln = lens_all[cpu_ids] if w.len_lo else None
        p = inputs.init_params(w).astype(np.float64)
        m, v = np.zeros(dims.P), np.zeros(dims.P)
        cache, off, lens_a = orc.cache_fill(acts, lens=ln, as_bf16=(w.cache_dtype == "bf16"))
        cache = orc.widen(cache)
        hp = orc.AdamW()
        c1 = time.perf_counter()
        nsteps_cpu = 0
        while True:  # whole training steps on the same samples until the time budget is used
            orc.step(dims, cache, off, lens_a, labels[cpu_ids], p, m, v, nsteps_cpu, hp)
            nsteps_cpu += 1
            c2 = time.perf_counter()
            if c2 - c1 >= args.cpu_seconds or nsteps_cpu >= 1000:
                break
        cpu = {"value": nsteps_cpu * len(cpu_ids) / (c2 - c1), "unit": "samples/s", "cores": orc.num_threads(),
               "kind": "oracle",
               "sample": f"{nsteps_cpu} training steps (forward, loss, backward, AdamW) on {len(cpu_ids)} samples "
                         f"of the {w.name} workload, cache already in host memory; {c2 - c1:.1f} s"}

    out = {
        "metric": "adapter-train samples/sec from activation cache",
        "value": args.steps * w.B / elapsed,
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.cache_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: L={w.L} d={w.d} seq={w.n_max} B={w.B} r={w.r} C={w.C} "
                               f"N={N} resident ({sess.cache_bytes / 1e9:.2f} GB {w.cache_dtype} cache)",
                   "tokens_per_step": M, "cache_fill_s": t_fill,
                   "formulation": ["per-layer kernels", "gram, single-launch chains",
                                   "gram, layer-by-layer chains"][pb.pac_step_path(sess.ctx)],
                   "gpu_event_ms_per_step": ev0.elapsed_time(ev1) / args.steps,
                   "final_loss": final_loss},
        "roofline": roof,
        "whole_step": whole,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def d_bytes(w):
    return w.d * (2 if w.cache_dtype == "bf16" else 4)


if __name__ == "__main__":
    main()
