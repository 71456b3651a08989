"""The hybrid-parallelism planner (paper Sec. 5.1): pins of the brute-force oracle, then the library's dynamic
programs (through the C ABI) against that oracle on seeded random instances.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import planner_oracle as po
from paper_2408_10746_amd import binding as pb

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_problem(rng, L, n_dev, B, M, mem_tight=False, kind="random"):
    """Profiles with the structure of the paper's setting: per-device speed factors (heterogeneous boards),
    per-layer costs, time growing with the number of samples (not necessarily linearly)."""
    speed = rng.uniform(0.5, 3.0, size=n_dev) if kind != "identical" else np.ones(n_dev)
    layer = rng.uniform(0.5, 2.0, size=L) if kind != "identical" else np.ones(L)
    beta = np.arange(B + 1, dtype=np.float64)
    curve = beta if kind != "random" else beta + 0.3 * np.sqrt(beta) * rng.uniform(0.0, 1.0)
    t_f = speed[:, None, None] * layer[None, :, None] * curve[None, None, :]
    t_b = 2.0 * t_f * (rng.uniform(0.8, 1.2, size=(n_dev, L, 1)) if kind == "random" else 1.0)
    mem_fixed = rng.uniform(1.0, 3.0, size=L)
    mem_act = rng.uniform(0.5, 1.5, size=L)
    if mem_tight:
        mem_budget = rng.uniform(0.35, 0.8, size=n_dev) * (mem_fixed.sum() + B * mem_act.sum())
    else:
        mem_budget = np.full(n_dev, 1e9)
    return po.Problem(t_f, t_b, mem_fixed, mem_act, mem_budget, rng.uniform(1, 4, size=L), rng.uniform(1, 4, size=L),
                      rng.uniform(1, 8, size=L), float(rng.uniform(2.0, 20.0)), M)


def lib_plan(p):
    return pb.pac_plan_hybrid(p.t_f, p.t_b, p.mem_fixed, p.mem_act, p.mem_budget, p.act_bytes, p.grad_bytes,
                              p.train_bytes, p.bandwidth, p.M)


# ---------------------------------------------------------------------------
# pins of the oracle
# ---------------------------------------------------------------------------
def golden():
    out = {}
    for line in open(os.path.join(GOLDEN, "planner_two_device_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def two_device_example():
    a = np.array([1.0, 2.0])
    beta = np.arange(3, dtype=np.float64)
    t_f = a[:, None, None] * np.ones((1, 2, 1)) * beta[None, None, :]
    return po.Problem(t_f, 2.0 * t_f, np.zeros(2), np.zeros(2), np.full(2, 1e9), np.full(2, 4.0), np.full(2, 4.0),
                      np.full(2, 6.0), 8.0, 3)


def test_oracle_hand_evaluated_example():
    g = golden()
    res = po.plan(two_device_example())
    assert res[1][0] == g["W_1"] and res[2][0] == g["W_2"]
    assert all(abs(x - g["latency_1"]) < 1e-12 for x in res[1][1]) and len(res[1][1]) == 2   # two dispatches tie
    assert res[2][1] == [g["latency_2"]]
    best = min(res, key=lambda s: (min(res[s][1]), s))
    assert best == int(g["sigma"])


def test_oracle_single_device_closed_form():
    rng = np.random.default_rng(5)
    p = make_problem(rng, L=4, n_dev=1, B=3, M=5)
    res = po.plan(p)
    assert list(res) == [1]
    f, b = p.t_f[0, :, 3].sum(), p.t_b[0, :, 3].sum()
    assert abs(res[1][0] - (f + b)) < 1e-12
    assert abs(res[1][1][0] - 5 * (f + b)) < 1e-12      # L_b = 0, L_n = AR of one device = 0


def test_oracle_identical_devices_even_split():
    """Identical devices, times linear in the samples: the slowest device of a group of n with b samples carries
    ceil(b / n) of them."""
    rng = np.random.default_rng(6)
    p = make_problem(rng, L=3, n_dev=3, B=4, M=2, kind="identical")
    for n in (1, 2, 3):
        t, alloc = po.stage_time(p, 0, 2, 0, n)
        per_sample = p.t_f[0, :, 1].sum() + p.t_b[0, :, 1].sum()
        assert abs(t - math.ceil(4 / n) * per_sample) < 1e-12 and sum(alloc) == 4


def test_oracle_memory_limits_force_a_pipeline():
    """No device can hold both layers: one stage is infeasible, two stages are not."""
    p = two_device_example()
    p.mem_fixed = np.array([3.0, 3.0])
    p.mem_budget = np.array([4.0, 4.0])
    res = po.plan(p)
    assert res[1][0] == math.inf and res[2][0] == 12.0


def test_oracle_more_devices_never_slower():
    rng = np.random.default_rng(7)
    p = make_problem(rng, L=3, n_dev=3, B=3, M=2)
    t1, _ = po.stage_time(p, 0, 2, 0, 1)
    t2, _ = po.stage_time(p, 0, 2, 0, 2)
    t3, _ = po.stage_time(p, 0, 2, 0, 3)
    assert t3 <= t2 <= t1


# ---------------------------------------------------------------------------
# the library against the oracle
# ---------------------------------------------------------------------------
def check_configuration(p, out):
    """What the library returns must be a valid configuration that attains the values it reports."""
    s = out["sigma"]
    assert out["stage_first_layer"][0] == 0 and out["stage_last_layer"][-1] == p.L - 1
    assert out["stage_first_dev"][0] == 0 and out["stage_first_dev"][-1] + out["stage_n_dev"][-1] == p.n_dev
    layers, groups, allocs = [], [], []
    for i in range(s):
        if i:
            assert out["stage_first_layer"][i] == out["stage_last_layer"][i - 1] + 1
            assert out["stage_first_dev"][i] == out["stage_first_dev"][i - 1] + out["stage_n_dev"][i - 1]
        layers.append(out["stage_last_layer"][i] - out["stage_first_layer"][i] + 1)
        groups.append(out["stage_n_dev"][i])
        a = out["samples"][out["stage_first_dev"][i]: out["stage_first_dev"][i] + groups[i]]
        assert sum(a) == p.B and min(a) >= 0
        allocs.append(a)
    Lb, Le, Ln = po.latency(p, layers, groups, allocs)
    assert abs(Lb - out["L_b"]) <= 1e-12 * max(1, Lb) and abs(Le - out["L_e"]) <= 1e-12 * Le
    assert abs(Ln - out["L_n"]) <= 1e-12 * max(1, Ln)
    return Lb + Le + Ln


def test_library_on_the_hand_evaluated_example():
    g = golden()
    out = lib_plan(two_device_example())
    assert out["sigma"] == int(g["sigma"])
    assert out["slowest_by_stage_count"][1] == g["W_1"] and out["slowest_by_stage_count"][2] == g["W_2"]
    assert abs(out["latency_by_stage_count"][1] - g["latency_1"]) < 1e-12
    assert abs(out["latency_by_stage_count"][2] - g["latency_2"]) < 1e-12
    assert out["samples"] == [2, 0] and out["stage_n_dev"] == [2]


@pytest.mark.parametrize("seed,L,n_dev,B,M,tight,kind", [
    (1, 3, 2, 3, 4, False, "random"), (2, 4, 3, 3, 2, False, "random"), (3, 4, 3, 4, 6, True, "random"),
    (4, 5, 3, 2, 3, True, "random"), (5, 3, 4, 3, 2, False, "linear"), (6, 5, 4, 2, 8, True, "random"),
    (7, 2, 4, 4, 3, False, "identical"), (8, 6, 2, 3, 5, True, "linear"), (9, 4, 4, 3, 1, True, "random"),
])
def test_library_matches_brute_force(seed, L, n_dev, B, M, tight, kind):
    rng = np.random.default_rng(seed)
    p = make_problem(rng, L, n_dev, B, M, mem_tight=tight, kind=kind)
    ref = po.plan(p)
    out = lib_plan(p)
    feasible = {s: v for s, v in ref.items() if v[0] < math.inf}
    for s, (w, lats) in ref.items():
        got = out["slowest_by_stage_count"][s]
        if w == math.inf:
            assert got == math.inf and out["latency_by_stage_count"][s] == math.inf
        else:
            assert abs(got - w) <= 1e-12 * w, (s, got, w)
            # the latency the library reports for W_s belongs to a configuration that attains W_s
            assert any(abs(out["latency_by_stage_count"][s] - x) <= 1e-9 * x for x in lats), (s, lats)
    if not feasible:
        assert out["sigma"] == 0
        return
    s = out["sigma"]
    assert s in feasible
    total = check_configuration(p, out)
    assert abs(total - out["latency_by_stage_count"][s]) <= 1e-12 * total
    assert all(total <= out["latency_by_stage_count"][q] + 1e-12 for q in feasible)   # argmin over s
    # every stage of the chosen configuration is as fast as its group can be (Eq. "dp2"), and the slowest is W_sigma
    worst = 0.0
    for i in range(s):
        t, _ = po.stage_time(p, out["stage_first_layer"][i], out["stage_last_layer"][i], out["stage_first_dev"][i],
                             out["stage_n_dev"][i])
        worst = max(worst, t)
    assert abs(worst - feasible[s][0]) <= 1e-12 * worst


def test_stage_time_entry_point_and_argument_errors():
    rng = np.random.default_rng(11)
    p = make_problem(rng, 4, 3, 4, 2, mem_tight=True)
    for (x, y, d0, n) in [(0, 3, 0, 3), (1, 2, 1, 2), (2, 2, 2, 1), (0, 0, 0, 2)]:
        t, alloc = pb.pac_plan_stage_time(p.t_f, p.t_b, p.mem_fixed, p.mem_act, p.mem_budget, x, y, d0, n)
        ref, _ = po.stage_time(p, x, y, d0, n)
        assert (t == ref == math.inf) or abs(t - ref) <= 1e-12 * ref
        if t < math.inf:
            assert sum(alloc[:n]) == p.B
    t, _ = pb.pac_plan_stage_time(p.t_f, p.t_b, p.mem_fixed, p.mem_act, p.mem_budget, 2, 1, 0, 1)
    assert math.isnan(t)
    assert pb.lib().pac_plan_hybrid(None, None) == pb.PAC_ERR_NULL
    bad = make_problem(rng, 2, 2, 2, 1)
    bad.t_f[0, 0, 1] = -1.0
    with pytest.raises(pb.PacError) as e:
        lib_plan(bad)
    assert e.value.status == pb.PAC_ERR_RANGE
