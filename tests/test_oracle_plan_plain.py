"""oracle/plan.py (organised for speed) against oracle/plan_plain.py (the same reading of Algorithm 1 and of the
urgent pass written out directly: unsorted transfer lists scanned in full, C and the benefit by loops over k).
The two were written separately and share no code; equality here is what lets the fast one stand in for the
plain one on the traces of the large models."""
import numpy as np
import pytest

from oracle import plan as op
from oracle import plan_plain as pp
from oracle import trace as ot
from synth import CONFIGS
from planlib import golden_options, load_golden, mini_trace, random_trace


def _same(tr, cap, bw, **kw):
    life = op.analyze_lifetimes(tr)
    periods, M = pp.inactive_periods(tr)
    assert sorted(periods) == sorted(life["periods"]) and M == life["M"]
    try:
        fast = op.build_plan(tr, life, cap, bw, **kw)
    except ValueError:
        with pytest.raises(ValueError):
            pp.build_plan(tr, cap, bw, **kw)
        return None
    plain = pp.build_plan(tr, cap, bw, **kw)
    assert plain["entries"] == fast["entries"]
    assert plain["Mp"] == fast["Mp"]
    assert (plain["n_greedy"], plain["n_forced"]) == (fast["n_greedy"], fast["n_forced"])
    return plain


@pytest.mark.parametrize("name", ["plan_example_a.txt", "plan_example_b.txt", "plan_example_c.txt", "plan_example_e.txt",
                                  "plan_example_f.txt"])
def test_plain_planner_on_the_hand_worked_examples(name):
    tr, cap, bw, entries, Mp, err = load_golden(name)
    kw = golden_options(name)
    if err:
        with pytest.raises(ValueError):
            pp.build_plan(tr, cap, bw, **kw)
        return
    pl = pp.build_plan(tr, cap, bw, **kw)
    assert pl["entries"] == entries and pl["Mp"] == Mp


def test_slot_search_by_definition():
    # transfers at [100,200) and [900,1050) on a cycle of 1000 (the second one reappears at [-100,50))
    tr, P = [(100, 200), (900, 1050)], 1000
    assert pp.earliest_slot(tr, P, 0, 1000, 50) == 50
    assert pp.earliest_slot(tr, P, 0, 1000, 60) == 200
    assert pp.earliest_slot(tr, P, 150, 290, 100) is None
    assert pp.latest_slot(tr, P, 0, 1000, 100) == 800
    assert pp.latest_slot(tr, P, 0, 150, 50) == 50
    assert pp.latest_slot(tr, P, 0, 150, 51) is None
    assert pp.earliest_slot(tr, P, 950, 1300, 60) == 1200
    assert pp.latest_slot(tr, P, 950, 2100, 60) == 1840
    # brute force over every integer start
    rng = np.random.default_rng(0)
    for _ in range(200):
        P = int(rng.integers(50, 120))
        placed = []
        for _ in range(int(rng.integers(0, 5))):
            b = int(rng.integers(0, 2 * P)); ln = int(rng.integers(1, 15))
            if all(not any(x - j * P < b + ln and b < y - j * P for j in range(-3, 4)) for (x, y) in placed) and ln < P:
                placed.append((b, b + ln))
        lo = int(rng.integers(0, P)); hi = lo + int(rng.integers(1, 2 * P)); d = int(rng.integers(1, 20))
        ok = [t for t in range(lo, hi - d + 1)
              if all(not (x + j * P < t + d and t < y + j * P) for (x, y) in placed for j in range(-4, 5))]
        assert pp.earliest_slot(placed, P, lo, hi, d) == (ok[0] if ok else None)
        assert pp.latest_slot(placed, P, lo, hi, d) == (ok[-1] if ok else None)


@pytest.mark.parametrize("duplex", [True, False])
def test_fast_planner_equals_plain_planner_on_random_traces_at_finite_bandwidth(duplex):
    rng = np.random.default_rng(7 + duplex)
    n_plans = n_greedy = n_forced = 0
    for trial in range(160):
        N = int(rng.integers(5, 28))
        tr = random_trace(rng, N=N, n_pers=int(rng.integers(1, 5)), n_trans=int(rng.integers(3, 22)))
        life = op.analyze_lifetimes(tr)
        cap = int(max(life["M"]) * rng.uniform(0.3, 0.95))
        # transfer times from a fraction of a kernel to several kernels: slots collide and get displaced
        bw = int(10 ** rng.uniform(8.3, 10.5))
        min_bytes = int(rng.choice([0, 0, 200]))
        pl = _same(tr, cap, bw, duplex=duplex, min_bytes=min_bytes)
        if pl is not None:
            n_plans += 1
            n_greedy += pl["n_greedy"]
            n_forced += pl["n_forced"]
    print(n_plans, n_greedy, n_forced)
    assert n_plans > 60 and n_greedy > 100 and n_forced > 40       # both halves of the planner are exercised


@pytest.mark.parametrize("name,frac,bw", [("tiny_gpt_fp32", 0.5, 25 * 10**9), ("tiny_gpt_fp32", 0.35, 2 * 10**9),
                                          ("tiny_llama_fp32", 0.5, 25 * 10**9), ("tiny_llama_fp32", 0.6, 10**8)])
def test_fast_planner_equals_plain_planner_on_the_small_model_traces(name, frac, bw):
    tr = ot.build_trace(CONFIGS[name])
    cap = int(max(op.analyze_lifetimes(tr)["M"]) * frac)
    for min_bytes in (0, 65536):
        assert _same(tr, cap, bw, min_bytes=min_bytes) is not None


@pytest.mark.slow
def test_fast_planner_equals_plain_planner_at_the_gpt2_small_shape():
    """The GPT-2-small-shaped workload (436 launches, 1162 inactive periods) at its own cap fraction and bandwidth."""
    cfg = CONFIGS["gpt2_small_bf16"]
    tr = ot.build_trace(cfg)
    cap = int(max(op.analyze_lifetimes(tr)["M"]) * cfg["cap_frac"])
    pl = _same(tr, cap, 25 * 10**9, min_bytes=1 << 20)
    assert pl is not None and pl["n_greedy"] > 50 and pl["n_forced"] > 100
