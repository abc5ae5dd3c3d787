"""Performance model of the migration engine with ready queues, chunked transfers and urgent-first service
(Section 3.2, "Minimize kernel stalls"; Section 3.3): the oracle's model against hand-worked timelines, and the
library's (tio_plan_simulate_engine) against the oracle's, bit for bit."""
import numpy as np
import pytest

import paper_2506_06472_amd as tio
from oracle import plan as op
from oracle import replay as orp
from oracle import trace as ot
from synth import CONFIGS
from planlib import load_golden, mini_trace, random_trace

OFF, PRE = 0, 1


def _overtaking_case():
    """4 kernels of 100 ns, 1 B/ns.  L (1000 B) is prefetched, not urgent, issued before kernel 0 and due at kernel 3;
    U (100 B) is prefetched, urgent, issued when kernel 0 completes and due at kernel 1.  Their offloads are issued before
    kernel 3 (after kernel 2) and are due at kernel 0 of the next iteration, so every iteration is the same."""
    tr = mini_trace([100] * 4, [("L", 1000, False, [0, 3]), ("U", 100, False, [0, 1]), ("Z", 8, False, [0, 1, 2, 3])])
    L, U = tr["ids"]["L"], tr["ids"]["U"]
    # (tensor, kind, trigger, deadline, urgent, pair); issue order as the planner sorts it
    entries = [(L, PRE, 0, 3, 0, 0), (U, PRE, 1, 1, 1, 1), (L, OFF, 3, 4, 0, 0), (U, OFF, 3, 4, 0, 1)]
    return tr, dict(entries=entries)


def test_urgent_request_overtakes_at_a_chunk_boundary_by_hand():
    tr, plan = _overtaking_case()
    bw = 10**9                                            # 1 B/ns
    # First iteration by hand, chunks of 250 B, urgent first:
    #   t=0    L's prefetch is issued and takes the channel: chunks [0,250) [250,500) ...; kernel 0 runs [0,100)
    #   t=100  kernel 0 ends; U's prefetch is issued, urgent, due at kernel 1: kernel 1 must wait for it
    #   t=250  chunk boundary: U is ready and urgent -> [250,350); kernel 1 runs [350,450), kernel 2 [450,550)
    #   L continues [350,600) [600,850) [850,1100); kernel 3 (needs L) runs [1100,1200)
    #   t=550  kernel 2 ends: both offloads are issued (trigger 3) on the other channel: L [550,800) ... done 1550?  No:
    #          the offload channel is free: L's offload moves [550,1550) in four chunks, U's (issue order, none urgent)
    #          follows [1550,1650).  They are due at kernel 0 of the next iteration, which therefore starts at 1650,
    #          and the prefetches issued there wait for "every offload whose deadline has been reached": ready at 1650.
    #   iteration 1 ends at 1200 (kernel 3); iteration 2: kernel 0 [1650,1750) ... the same pattern shifted: it ends at
    #          1650 + 1200 = 2850; length 2850 - 1200 = 1650: the offloads (1100 ns of traffic after kernel 2) are exposed.
    got = orp.simulate_engine(tr, plan, bw, chunk_bytes=250, urgent_first=True, iterations=3)
    assert got["per_iteration"] == [1200, 1650, 1650]
    # without priority U waits for all of L: kernel 1 starts at 1100: iteration 1 = 1400; from then on 1100 + 450 + 100 + ...
    #   kernel 1 [1100,1200) kernel 2 [1200,1300) kernel 3 [1300,1400); offloads issued at 1300: L [1300,2300) U [2300,2400)
    #   iteration 2: kernel 0 at 2400 -> [2400,2500); L prefetch [2400,3400), U [3400,3500): kernel 1 at 3500 ... ends 3800
    fifo = orp.simulate_engine(tr, plan, bw, chunk_bytes=250, urgent_first=False, iterations=3)
    assert fifo["per_iteration"] == [1400, 2400, 2400]
    # whole-tensor transfers leave nothing to overtake at: same as without priority
    assert orp.simulate_engine(tr, plan, bw, chunk_bytes=0, urgent_first=True, iterations=3)["per_iteration"] == [1400, 2400, 2400]
    # and the plain first-come-first-served model agrees with that
    assert orp.simulate(tr, plan, bw, iterations=3)["per_iteration"] == [1400, 2400, 2400]


def test_ready_queue_does_not_wait_behind_a_blocked_request_by_hand():
    """Two prefetches on one channel: the first one issued waits for its own offload, which is still running; the second is
    ready.  First come first served holds the channel for the blocked one, the ready queue serves the other meanwhile."""
    tr = mini_trace([100] * 4, [("A", 400, False, [0, 2]), ("B", 100, False, [0, 1]), ("Z", 8, False, [0, 1, 2, 3])])
    A, B = tr["ids"]["A"], tr["ids"]["B"]
    # A: offload issued before kernel 1 (400 ns), prefetch issued before kernel 1 too (legal: it waits for the offload);
    # B: prefetch issued before kernel 1 after A's, due at kernel 1; B's offload before kernel 3, due at kernel 0
    entries = [(A, OFF, 1, 2, 0, 0), (A, PRE, 1, 2, 0, 0), (B, PRE, 1, 1, 0, 1), (B, OFF, 3, 4, 0, 1)]
    plan = dict(entries=entries)
    bw = 10**9
    # ready queue: t=100 A's offload [100,500); B's prefetch is ready -> [100,200): kernel 1 [200,300);
    #   A's prefetch ready at 500 -> [500,900): kernel 2 (due) waits for the offload (deadline 2) and the prefetch: [900,1000)
    #   kernel 3 [1000,1100); B's offload issued at 1000 -> [1000,1100), due at kernel 0: next iteration starts at 1100
    eng = orp.simulate_engine(tr, plan, bw, chunk_bytes=0, urgent_first=False, iterations=2)
    assert eng["per_iteration"] == [1100, 1100]
    # first come first served: B's prefetch starts when A's has finished (900): kernel 1 at 1000 ... iteration 1300
    assert orp.simulate(tr, plan, bw, iterations=2)["per_iteration"] == [1300, 1300]


@pytest.mark.parametrize("name,frac", [("tiny_gpt_fp32", 0.5), ("tiny_llama_fp32", 0.4), ("gpt2_small_bf16", 0.4)])
def test_engine_model_bit_exact(name, frac):
    cfg = CONFIGS[name] if name != "gpt2_small_bf16" else dict(CONFIGS[name], L=3)
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    life = op.analyze_lifetimes(tr)
    cap = int(max(life["M"]) * frac) // 256 * 256
    biggest = max(t[0] for t in tr["tensors"])
    for bw in (10**9, 25 * 10**9, 0):
        for duplex in (True, False):
            pl = tio.tio_build_plan(lt, ll, cap, bw, duplex=duplex)
            ref = op.build_plan(tr, life, pl.export()["planning_cap"], bw, duplex=duplex)
            assert pl.export()["entries"] == ref["entries"]
            for sim_bw in (bw, 5 * 10**9):
                for chunk in (0, biggest // 7 + 1, biggest // 40 + 1):
                    for uf in (True, False):
                        for it in (1, 3):
                            want = orp.simulate_engine(tr, ref, sim_bw, duplex=duplex, iterations=it, chunk_bytes=chunk, urgent_first=uf)
                            got = tio.tio_plan_simulate_engine(lt, pl, sim_bw, duplex=duplex, iterations=it, chunk_bytes=chunk, urgent_first=uf)
                            assert got == (want["step_ns"], want["compute_ns"]), (bw, duplex, sim_bw, chunk, uf, it)


def test_engine_model_bit_exact_on_random_traces_and_invariants():
    rng = np.random.default_rng(17)
    n = 0
    for trial in range(60):
        tr = random_trace(rng, N=int(rng.integers(6, 30)), n_pers=int(rng.integers(1, 5)), n_trans=int(rng.integers(3, 25)))
        life = op.analyze_lifetimes(tr)
        cap = int(max(life["M"]) * rng.uniform(0.3, 0.95))
        bw = int(10 ** rng.uniform(8, 11))
        try:
            ref = op.build_plan(tr, life, cap, bw)
        except ValueError:
            continue
        lt = tio.tio_trace_import(tr["n_persistent"], [ops for _, ops, _ in tr["kernels"]], [t[0] for t in tr["tensors"]],
                                  tr["tau"], [t[1] for t in tr["tensors"]], [k[0] for k in tr["kernels"]])
        pl = tio.tio_build_plan(lt, tio.tio_analyze_lifetimes(lt), cap, bw, arena_bytes=1 << 30)
        if pl.export()["planning_cap"] != cap:
            continue
        assert pl.export()["entries"] == ref["entries"]
        chunk = int(rng.choice([0, 64, 256, 1 << 20]))
        for uf in (True, False):
            want = orp.simulate_engine(tr, ref, bw, chunk_bytes=chunk, urgent_first=uf)
            assert tio.tio_plan_simulate_engine(lt, pl, bw, chunk_bytes=chunk, urgent_first=uf) == (want["step_ns"], want["compute_ns"])
            assert want["step_ns"] >= want["compute_ns"]
        # instantaneous transfers: the compute time, whatever the policy
        assert orp.simulate_engine(tr, ref, 0)["step_ns"] == sum(tr["tau"])
        n += 1
    assert n > 20


def test_engine_model_golden_through_the_c_abi():
    tr, plan = _overtaking_case()
    lt = tio.tio_trace_import(tr["n_persistent"], [ops for _, ops, _ in tr["kernels"]], [t[0] for t in tr["tensors"]],
                              tr["tau"], [t[1] for t in tr["tensors"]], [k[0] for k in tr["kernels"]])
    # the library only simulates plans it built: plan example e instead (urgent and ordinary entries, three pairs)
    tr, cap, bw, entries, Mp, _ = load_golden("plan_example_e.txt")
    lt = tio.tio_trace_import(tr["n_persistent"], [ops for _, ops, _ in tr["kernels"]], [t[0] for t in tr["tensors"]],
                              tr["tau"], [t[1] for t in tr["tensors"]], [k[0] for k in tr["kernels"]])
    pl = tio.tio_build_plan(lt, tio.tio_analyze_lifetimes(lt), cap, bw, arena_bytes=1 << 20)
    ref = dict(entries=entries)
    for chunk in (0, 100, 250):
        for uf in (True, False):
            want = orp.simulate_engine(tr, ref, bw, chunk_bytes=chunk, urgent_first=uf)
            assert tio.tio_plan_simulate_engine(lt, pl, bw, chunk_bytes=chunk, urgent_first=uf) == (want["step_ns"], want["compute_ns"])
    with pytest.raises(tio.TioError):
        tio.tio_plan_simulate_engine(lt, pl, bw, iterations=0)


def test_pick_order_of_the_runtime_engine():
    """The runtime's paced engine chooses like the model: first ready urgent request, else first ready request, in the
    order submitted; without the ready queue only the oldest request may go."""
    ch = tio.tio_engine_choose
    assert ch([], []) == -1
    assert ch([0, 0, 0], [1, 1, 0]) == -1
    assert ch([0, 1, 1, 1], [0, 0, 1, 1]) == 2                       # an urgent ready one overtakes the ready one before it
    assert ch([0, 1, 1, 1], [1, 0, 0, 0]) == 1                       # a blocked urgent one does not hold the others up
    assert ch([1, 1], [0, 0]) == 0
    assert ch([0, 1, 1, 1], [0, 0, 1, 1], urgent_first=False) == 1
    assert ch([0, 1, 1], [0, 1, 1], ready_queue=False) == -1         # first come first served: waits for the oldest
    assert ch([1, 1, 1], [0, 1, 1], ready_queue=False) == 0
    # the same choice as the oracle's model makes on random queues
    rng = np.random.default_rng(1)
    for _ in range(200):
        n = int(rng.integers(1, 9))
        ready, urgent = rng.integers(0, 2, n).tolist(), rng.integers(0, 2, n).tolist()
        want = next((i for i in range(n) if ready[i] and urgent[i]), next((i for i in range(n) if ready[i]), -1))
        assert ch(ready, urgent) == want
