"""Destination choice between the slow tier and a budgeted host-memory tier (Section 3.2, "Decide offloading
destination"; the paper's best variant uses both).  Oracle pins: a hand-worked example (tests/golden/
plan_example_d.txt), reduction to the single-tier plan when the host tier cannot be used, the budget as an
invariant on random traces, and the performance model's numbers for the worked example."""
import numpy as np
import pytest

from oracle import plan as op
from oracle import replay as orp
from oracle import trace as ot
from synth import CONFIGS
from planlib import load_golden_two_tier, random_trace


def test_hand_worked_example():
    g = load_golden_two_tier("plan_example_d.txt")
    tr = g["trace"]
    life = op.analyze_lifetimes(tr)
    pl = op.build_plan(tr, life, g["cap"], g["bw"], host_bw=g["host_bw"], host_budget=g["host_budget"])
    assert pl["entries"] == g["entries"] and pl["Mp"] == g["Mp"] and pl["tier"] == g["tier"]
    assert (pl["n_greedy"], pl["n_forced"], pl["host_peak"]) == (2, 0, 1000)
    st = orp.check_plan(tr, life, pl, g["cap"], host_budget=g["host_budget"])
    assert st["host_pairs"] == 1 and st["host_bytes_per_direction"] == 1000
    assert orp.simulate(tr, pl, g["bw"], host_bw=g["host_bw"])["per_iteration"] == [1000, 1000, 1000]
    # one byte less of budget: the same entries, everything on the slow tier, and the shared channel costs 200 ns
    p1 = op.build_plan(tr, life, g["cap"], g["bw"], host_bw=g["host_bw"], host_budget=999)
    assert p1["entries"] == g["entries"] and p1["tier"] == [0, 0] and p1["host_peak"] == 0
    assert orp.simulate(tr, p1, g["bw"], host_bw=g["host_bw"])["per_iteration"] == [1200, 1200, 1200]
    assert p1 == dict(op.build_plan(tr, life, g["cap"], g["bw"]))


@pytest.mark.parametrize("name", ["tiny_gpt_fp32", "tiny_llama_fp32"])
def test_unusable_host_tier_gives_the_single_tier_plan(name):
    tr = ot.build_trace(CONFIGS[name])
    life = op.analyze_lifetimes(tr)
    cap = max(life["M"]) // 2
    base = op.build_plan(tr, life, cap, 10**9)
    smallest = min(s for _, s, _, _ in life["periods"])
    for kw in (dict(host_bw=0, host_budget=10**9), dict(host_bw=10**10, host_budget=0),
               dict(host_bw=10**10, host_budget=smallest - 1)):
        assert op.build_plan(tr, life, cap, 10**9, **kw) == base


@pytest.mark.parametrize("name", ["tiny_gpt_fp32", "tiny_llama_fp32"])
def test_host_tier_is_used_when_the_slow_tier_is_saturated_and_helps(name):
    """Slow tier so slow that its channels are congested: with a host tier the plan stays valid, respects the
    budget, moves part of the bytes through the host, and the model predicts a faster step; a larger budget
    never makes the prediction worse on these traces."""
    tr = ot.build_trace(CONFIGS[name])
    life = op.analyze_lifetimes(tr)
    cap = max(life["M"]) // 2
    bw, hbw = 2 * 10**9, 20 * 10**9
    base = op.build_plan(tr, life, cap, bw)
    t_base = orp.simulate(tr, base, bw)["step_ns"]
    prev = t_base
    for budget in (max(life["M"]) // 8, max(life["M"]) // 2, 2 * max(life["M"])):
        pl = op.build_plan(tr, life, cap, bw, host_bw=hbw, host_budget=budget)
        st = orp.check_plan(tr, life, pl, cap, host_budget=budget)
        assert st["host_pairs"] > 0 and 0 < pl["host_peak"] <= budget
        t = orp.simulate(tr, pl, bw, host_bw=hbw)["step_ns"]
        assert t <= prev
        prev = t
    assert prev < t_base


@pytest.mark.parametrize("duplex", [True, False])
def test_random_traces_respect_the_host_budget(duplex):
    rng = np.random.default_rng(11)
    used = 0
    for _ in range(150):
        tr = random_trace(rng, int(rng.integers(6, 20)), int(rng.integers(1, 4)), int(rng.integers(3, 12)))
        life = op.analyze_lifetimes(tr)
        peak = max(life["M"])
        cap = int(peak * rng.uniform(0.5, 0.95))
        bw = int(rng.integers(1, 20)) * 10**8
        budget = int(peak * rng.uniform(0.05, 0.6))
        try:
            pl = op.build_plan(tr, life, cap, bw, duplex=duplex, host_bw=4 * bw, host_budget=budget)
        except ValueError:
            continue
        st = orp.check_plan(tr, life, pl, cap, host_budget=budget)
        used += st["host_pairs"] > 0
        sim = orp.simulate(tr, pl, bw, duplex=duplex, host_bw=4 * bw)
        assert sim["step_ns"] >= sim["compute_ns"]
    assert used > 10
