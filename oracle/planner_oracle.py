"""Brute-force oracle of the hybrid-parallelism planner (paper Sec. 5.1).

TEST INFRASTRUCTURE ONLY (imported by tests/ alone).  It shares no code with the library's planner and uses no
dynamic programming: every way of cutting the layers into consecutive stages, every way of cutting the ordered
device list into consecutive groups, and every way of dealing a micro-batch's samples over a group's devices is
enumerated, and the definitions are evaluated on each:

  stage time         T(x->y, G) = min over dispatches of max over the group's devices of
                     sum_{l=x..y} [t_f(d, l, i_d) + t_b(d, l, i_d)]        (what Eq. "dp2" computes), with a
                     device whose footprint sum_l (mem_fixed[l] + i_d mem_act[l]) exceeds its budget at +inf
  balanced pipeline  W_s = min over (layer cuts, device cuts) of the slowest stage   (what Eq. "dp-main" computes)
  latency of W_s     L_b + L_e + L_n as in Eq. "Lb" / "Ln" (parenthesis of "Ln" closed after the inner sum),
                     e_f / e_b the slowest device of each stage under its dispatch, c_f / c_b = B * bytes / bandwidth,
                     AR = ring all-reduce 2 (g-1)/g * trainable bytes / bandwidth
  sigma              argmin_s of that latency (Eq. "sigma"), smallest s on ties

Only practical for tiny inputs (a handful of layers, devices and samples).

Pins (tests/test_planner.py): a single device (closed form), identical devices with linear times (even split),
a hand-evaluated two-device example kept under tests/golden/, monotonicity in the device set, memory limits that
force a pipeline.  The paper prints no worked planning example: against its own numbers "parity unpinned".
"""
from __future__ import annotations

import itertools
import math
from dataclasses import dataclass

import numpy as np


@dataclass
class Problem:
    t_f: np.ndarray          # [n_dev][L][B+1]
    t_b: np.ndarray
    mem_fixed: np.ndarray    # [L]
    mem_act: np.ndarray      # [L]
    mem_budget: np.ndarray   # [n_dev]
    act_bytes: np.ndarray    # [L]
    grad_bytes: np.ndarray   # [L]
    train_bytes: np.ndarray  # [L]
    bandwidth: float
    M: int

    @property
    def L(self):
        return self.t_f.shape[1]

    @property
    def n_dev(self):
        return self.t_f.shape[0]

    @property
    def B(self):
        return self.t_f.shape[2] - 1


def _device(p: Problem, d, x, y, i):
    mem = sum(p.mem_fixed[l] + i * p.mem_act[l] for l in range(x, y + 1))
    if mem > p.mem_budget[d]:
        return math.inf, math.inf
    return (sum(p.t_f[d, l, i] for l in range(x, y + 1)), sum(p.t_b[d, l, i] for l in range(x, y + 1)))


def _dispatches(b, n):
    """All ways of writing b as an ordered sum of n non-negative integers."""
    if n == 1:
        yield (b,)
        return
    for i in range(b + 1):
        for rest in _dispatches(b - i, n - 1):
            yield (i,) + rest


def stage_time_all(p: Problem, x, y, d0, n):
    """(T, every dispatch that attains it) by trying every dispatch."""
    vals = []
    for alloc in _dispatches(p.B, n):
        worst = 0.0
        for k, i in enumerate(alloc):
            f, b = _device(p, d0 + k, x, y, i)
            worst = max(worst, f + b)
        vals.append((worst, alloc))
    best = min(v for v, _ in vals)
    if best == math.inf:
        return best, []
    return best, [a for v, a in vals if abs(v - best) <= 1e-12 * max(1.0, abs(best))]


def stage_time(p: Problem, x, y, d0, n):
    """(T, one dispatch that attains it)."""
    best, args = stage_time_all(p, x, y, d0, n)
    return best, (args[0] if args else None)


def _compositions(total, parts):
    """Ordered ways of writing total as a sum of `parts` positive integers."""
    for cuts in itertools.combinations(range(1, total), parts - 1):
        edges = (0,) + cuts + (total,)
        yield [edges[k + 1] - edges[k] for k in range(parts)]


def latency(p: Problem, layers, groups, allocs):
    """L_b, L_e, L_n of one configuration (lists of per-stage layer counts, device counts, dispatches)."""
    s = len(layers)
    ef, eb, cf, cb, ar = [], [], [], [], []
    x = d0 = 0
    for i in range(s):
        y = x + layers[i] - 1
        fs, bs = zip(*[_device(p, d0 + k, x, y, allocs[i][k]) for k in range(groups[i])])
        ef.append(max(fs))
        eb.append(max(bs))
        cf.append(p.B * p.act_bytes[y] / p.bandwidth)
        cb.append(p.B * p.grad_bytes[y] / p.bandwidth)
        g = groups[i]
        ar.append(2.0 * (g - 1) / g * sum(p.train_bytes[x:y + 1]) / p.bandwidth if g > 1 else 0.0)
        x, d0 = y + 1, d0 + g
    Lb = sum(ef[i] + cf[i] for i in range(s - 1))
    Le = p.M * (ef[s - 1] + eb[s - 1])
    Ln = max(ar[i] + sum(eb[j] + cb[j] for j in range(i, s - 1)) for i in range(s))
    return Lb, Le, Ln


def plan(p: Problem):
    """{s: (W_s, latencies of all configurations that attain W_s with every stage at its own optimum)}."""
    per_s = {}
    for s in range(1, min(p.L, p.n_dev) + 1):
        best, lats = math.inf, []
        for layers in _compositions(p.L, s):
            for groups in _compositions(p.n_dev, s):
                x = d0 = 0
                times, choices = [], []
                for i in range(s):
                    t, a = stage_time_all(p, x, x + layers[i] - 1, d0, groups[i])
                    times.append(t)
                    choices.append(a)
                    x += layers[i]
                    d0 += groups[i]
                w = max(times)
                if w == math.inf:
                    continue
                if w < best - 1e-12 * max(1.0, abs(best) if best < math.inf else 1.0):
                    best, lats = w, []
                if abs(w - best) <= 1e-12 * max(1.0, abs(best)):
                    # every stage at its own optimum (what Eq. "dp2" records), all tied dispatches
                    for allocs in itertools.product(*choices):
                        lats.append(sum(latency(p, layers, groups, list(allocs))))
        per_s[s] = (best, lats)
    return per_s
