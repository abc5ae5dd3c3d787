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


# ------------------------------------------------------------------ library against the oracle
import paper_2506_06472_amd as tio  # noqa: E402
from test_plan_parity import lib_trace_from_oracle  # noqa: E402


def _same(tr, lt, ll, cap, bw, hbw, budget, duplex=True, arena=None):
    pl = tio.tio_build_plan(lt, ll, cap, bw, duplex=duplex, host_bw=hbw, host_budget=budget, arena_bytes=arena or 0)
    pe = pl.export()
    life = op.analyze_lifetimes(tr)
    ref = op.build_plan(tr, life, pe["planning_cap"], bw, duplex=duplex, host_bw=hbw, host_budget=budget)
    assert pe["entries"] == ref["entries"] and pe["Mp"] == ref["Mp"] and pe["tier"] == ref["tier"]
    assert (pe["n_greedy"], pe["n_forced"], pe["host_peak"]) == (ref["n_greedy"], ref["n_forced"], ref["host_peak"])
    st = orp.check_plan(tr, life, ref, pe["planning_cap"], host_budget=budget if hbw and budget else None)
    # the host pool the library asks for holds every host-tier pair without overlap in time
    assert pe["host_tier_needed"] >= pe["host_peak"]
    for it in (1, 3):
        want = orp.simulate(tr, ref, bw, duplex=duplex, iterations=it, host_bw=hbw)
        assert tio.tio_plan_simulate(lt, pl, bw, duplex=duplex, iterations=it) == (want["step_ns"], want["compute_ns"])
    return pe, st


def test_library_golden_two_tier():
    g = load_golden_two_tier("plan_example_d.txt")
    lt = lib_trace_from_oracle(g["trace"])
    ll = tio.tio_analyze_lifetimes(lt)
    pl = tio.tio_build_plan(lt, ll, g["cap"], g["bw"], host_bw=g["host_bw"], host_budget=g["host_budget"], arena_bytes=1 << 20)
    pe = pl.export()
    assert pe["planning_cap"] == g["cap"] and pe["entries"] == g["entries"] and pe["tier"] == g["tier"] and pe["Mp"] == g["Mp"]
    assert pe["host_peak"] == 1000 and pe["host_tier_needed"] == 1000
    assert tio.tio_plan_simulate(lt, pl, g["bw"]) == (1000, 800)


@pytest.mark.parametrize("name", ["tiny_gpt_fp32", "tiny_llama_fp32"])
def test_library_model_plans_bit_exact_with_a_host_tier(name):
    cfg = CONFIGS[name]
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    peak = int(ll.export()["M"].max())
    used = 0
    for frac, bw, hbw, bfrac, duplex in ((0.5, 2 * 10**9, 2 * 10**10, 0.25, True), (0.4, 10**9, 4 * 10**9, 1.0, True),
                                         (0.5, 5 * 10**9, 10**10, 0.1, False), (0.6, 25 * 10**9, 50 * 10**9, 0.5, True)):
        pe, st = _same(tr, lt, ll, int(peak * frac) // 256 * 256, bw, hbw, int(peak * bfrac), duplex)
        used += st["host_pairs"] > 0
    assert used >= 2


def test_library_random_traces_bit_exact_with_a_host_tier():
    rng = np.random.default_rng(23)
    n = 0
    for _ in range(120):
        tr = random_trace(rng, int(rng.integers(6, 20)), int(rng.integers(1, 4)), int(rng.integers(3, 12)))
        life = op.analyze_lifetimes(tr)
        peak = max(life["M"])
        cap = int(peak * rng.uniform(0.5, 0.95))
        bw = int(rng.integers(1, 20)) * 10**8
        budget = int(peak * rng.uniform(0.05, 0.6))
        lt = lib_trace_from_oracle(tr)
        ll = tio.tio_analyze_lifetimes(lt)
        try:
            op.build_plan(tr, life, cap, bw, host_bw=4 * bw, host_budget=budget)
        except ValueError:
            continue
        _same(tr, lt, ll, cap, bw, 4 * bw, budget, duplex=bool(rng.integers(0, 2)), arena=1 << 20)
        n += 1
    assert n > 60


def test_library_gpt2_small_bit_exact_with_a_host_tier():
    cfg = dict(CONFIGS["gpt2_small_bf16"], L=4)
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    peak = int(ll.export()["M"].max())
    pe, st = _same(tr, lt, ll, int(peak * 0.5) // 256 * 256, 16 * 10**9, 48 * 10**9, peak // 4)
    assert st["host_pairs"] > 0
