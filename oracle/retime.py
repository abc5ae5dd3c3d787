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


def retimed_candidates(trace, life, cap, bw, passes, duplex=True, min_bytes=0, host_bw=0, host_budget=0,
                       clamp_benefit=False):
    """Every pass's plan, in pass order: results of oracle/plan.py build_plan plus retime_pass and predicted_step_ns
    (the iteration the performance model predicts on the true kernel times).  Pass 0 is the paper's plan; passes
    1..passes are chain A (planned on the fully stretched timeline of the pass before), passes+1..2*passes chain B
    (only the kernels from the first kernel of largest memory demand M on are stretched: before it memory grows and
    the stalls wait for offloads; stretching there invites the planner to offload there again)."""
    kw = dict(duplex=duplex, min_bytes=min_bytes, host_bw=host_bw, host_budget=host_budget, clamp_benefit=clamp_benefit)
    first = op.build_plan(trace, life, cap, bw, **kw)
    first["retime_pass"] = 0
    out = [first]
    if passes <= 0 or bw == 0:
        return out
    sim = orp.simulate(trace, first, bw, duplex=duplex, host_bw=host_bw)
    first["predicted_step_ns"] = sim["step_ns"]
    tau = trace["tau"]
    kpeak = life["M"].index(max(life["M"]))
    for chain in (0, 1):
        stretched = sim["stretched"]
        for p in range(1, passes + 1):
            planned_on = [tau[k] if (chain == 1 and k < kpeak) else stretched[k] for k in range(len(tau))]
            cand = op.build_plan(dict(trace, tau=planned_on), life, cap, bw, **kw)
            s2 = orp.simulate(trace, cand, bw, duplex=duplex, host_bw=host_bw)
            stretched = s2["stretched"]
            cand["retime_pass"] = chain * passes + p
            cand["predicted_step_ns"] = s2["step_ns"]
            out.append(cand)
    return out


def build_plan_retimed(trace, life, cap, bw, passes, **kw):
    """The candidate with the shortest predicted iteration, the earliest pass among equals.  (The library keeps the
    best candidate whose address layout fits its arena: with an ample arena that is this one.)"""
    cands = retimed_candidates(trace, life, cap, bw, passes, **kw)
    if len(cands) == 1:
        return cands[0]
    return min(cands, key=lambda c: (c["predicted_step_ns"], c["retime_pass"]))
