"""CPU oracle: re-timed planning.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

This is an extension of this repository, not a passage of the paper: the paper plans once, on the kernel
times of an iteration that runs without stalls (Section 3.1 profiles them, Algorithm 1 of Section 3.2 places
migrations on that timeline).  Where the bytes that must move take longer than the compute, the iteration
stalls, and the timeline Algorithm 1 plans on is several times shorter than the iteration that will run.
Re-timing repeats the paper's planner, unchanged, on the timeline of the iteration as the performance model
of Section 2.2 (oracle/replay.py simulate) predicts it under the previous plan: kernel k takes tau[k] plus the
stall in front of it.  Every pass's plan is simulated on the true kernel times; the pass with the shortest
predicted iteration is kept, the first pass (the paper's plan) included, so the result is by construction
never predicted slower than the paper's plan.  A plan's validity does not depend on kernel times (residency
is counted per kernel index), so every pass yields a valid plan for the same trace.

Being a definition of this build, it has no pin in the paper; tests/test_retime.py pins what the definition
implies (pass 0 is oracle/plan.py build_plan; the prediction never gets worse with more passes; every result
passes oracle/replay.py check_plan) and one example worked by hand.
"""
from __future__ import annotations

from . import plan as op
from . import replay as orp


def build_plan_retimed(trace, life, cap, bw, passes, duplex=True, min_bytes=0, host_bw=0, host_budget=0,
                       clamp_benefit=False):
    """Result of oracle/plan.py build_plan plus retime_pass (which pass won) and predicted_step_ns."""
    kw = dict(duplex=duplex, min_bytes=min_bytes, host_bw=host_bw, host_budget=host_budget, clamp_benefit=clamp_benefit)
    best = op.build_plan(trace, life, cap, bw, **kw)
    best["retime_pass"] = 0
    if passes <= 0 or bw == 0:
        return best
    sim = orp.simulate(trace, best, bw, duplex=duplex, host_bw=host_bw)
    best["predicted_step_ns"] = sim["step_ns"]
    stretched = sim["stretched"]
    for p in range(1, passes + 1):
        cand = op.build_plan(dict(trace, tau=list(stretched)), life, cap, bw, **kw)
        sim = orp.simulate(trace, cand, bw, duplex=duplex, host_bw=host_bw)
        stretched = sim["stretched"]
        if sim["step_ns"] < best["predicted_step_ns"]:
            best = cand
            best["retime_pass"] = p
            best["predicted_step_ns"] = sim["step_ns"]
    return best
