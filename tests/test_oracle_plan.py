"""Pins for oracle/trace.py, oracle/plan.py and oracle/replay.py."""
import itertools

import numpy as np
import pytest

from oracle import plan as op
from oracle import replay as orp
from oracle import trace as ot
from oracle.model import param_specs
from synth import CONFIGS
from planlib import golden_options, load_golden, mini_trace, random_trace


# ------------------------------------------------------------------ hand-worked cases
@pytest.mark.parametrize("name", ["plan_example_a.txt", "plan_example_b.txt", "plan_example_c.txt", "plan_example_e.txt",
                                  "plan_example_f.txt"])
def test_hand_worked_examples(name):
    tr, cap, bw, entries, Mp, err = load_golden(name)
    kw = golden_options(name)
    life = op.analyze_lifetimes(tr)
    if err:
        with pytest.raises(ValueError):
            op.build_plan(tr, life, cap, bw, **kw)
        return
    pl = op.build_plan(tr, life, cap, bw, **kw)
    assert pl["entries"] == entries
    assert pl["Mp"] == Mp
    orp.check_plan(tr, life, pl, cap)


def test_performance_model_by_hand():
    # example c: the one pair is fully exposed: 8 kernels of 100 ns + 150 ns offload + 150 ns prefetch
    tr, cap, bw, entries, Mp, _ = load_golden("plan_example_c.txt")
    life = op.analyze_lifetimes(tr)
    pl = op.build_plan(tr, life, cap, bw)
    sim = orp.simulate(tr, pl, bw)
    assert sim["compute_ns"] == 800 and sim["per_iteration"] == [1100, 1100, 1100]
    # empty plan: exactly the compute time
    pl0 = op.build_plan(tr, life, 10**6, bw)
    assert pl0["entries"] == [] and orp.simulate(tr, pl0, bw)["step_ns"] == 800
    # example a, both pairs, by hand: W hides completely (20 ns transfers inside idle windows);
    # X: offload issued after kernel 0 (t=100) takes 100 ns and blocks kernel 1 until 200;
    #    prefetch issued after kernel 4 takes 100 ns and blocks kernel 5: 600 + 100 + 100
    tr, cap, bw, entries, Mp, _ = load_golden("plan_example_a.txt")
    life = op.analyze_lifetimes(tr)
    pl = op.build_plan(tr, life, cap, bw)
    assert orp.simulate(tr, pl, bw)["per_iteration"][-1] == 800


# ------------------------------------------------------------------ trace
def _n_params(cfg):
    return sum(int(np.prod(s)) for _, s, _ in param_specs(cfg))


@pytest.mark.parametrize("name", list(CONFIGS))
def test_trace_counts_and_persistent_bytes(name):
    cfg = CONFIGS[name]
    tr = ot.build_trace(cfg)
    L = cfg["L"]
    N = len(tr["kernels"])
    assert N == (35 * L + 16 if cfg["arch"] == "gpt" else 31 * L + 13)
    bpp = 14 if cfg["precision"] == "bf16" else 12
    S = cfg["B"] * cfg["T"]
    pers = sum(t[0] for t in tr["tensors"][:tr["n_persistent"]])
    slack = 256 * tr["n_persistent"]                      # rounding of each tensor to 256 B
    assert bpp * _n_params(cfg) + 8 * S <= pers <= bpp * _n_params(cfg) + 8 * S + slack
    assert len(tr["tau"]) == N and min(tr["tau"]) >= ot.MODEL_LAUNCH_NS
    # every transient tensor is written before it is read, ids follow first-write order
    seen = set(range(tr["n_persistent"]))
    nxt = tr["n_persistent"]
    for op_, operands, _ in tr["kernels"]:
        for t, fl in operands:
            if t not in seen:
                assert fl & ot.WRITE, (t, fl)      # workspaces are written and read by one record
        for t in sorted(t for t, _ in operands if t not in seen):
            assert t == nxt
            nxt += 1
            seen.add(t)
    assert nxt == len(tr["tensors"])
    assert all(t[0] % 256 == 0 for t in tr["tensors"])


def test_config4_persistent_plus_grads_is_about_208_GB():
    tr = ot.build_trace(CONFIGS["llama_13b_bf16"])
    pers = sum(t[0] for t in tr["tensors"][:tr["n_persistent"]])
    grads = sum(t[0] for t in tr["tensors"] if t[1] == ot.K_PGRAD)
    assert abs((pers + grads) / 1e9 - 208.3) < 0.1


def test_lifetimes_closed_form_on_the_layer_chain():
    cfg = CONFIGS["tiny_gpt_fp32"]
    tr = ot.build_trace(cfg)
    life = op.analyze_lifetimes(tr)
    L, N = cfg["L"], len(tr["kernels"])
    bwd0 = 1 + 8 * L + 4 + 7               # first kernel of the last layer's backward (head: dX, dW, AdamW; final norm: 2 + 2 AdamW)
    for i in range(L):
        t = tr["ids"][f"l{i}.act"]
        s = tr["tensors"][t][0]
        gelu = 1 + 8 * i + 6
        assert life["active"][t] == [gelu, gelu + 1, bwd0 + 27 * (L - 1 - i) + 1]
        assert (t, s, gelu + 1, bwd0 + 27 * (L - 1 - i) + 1) in life["periods"]
        # x entering layer i: written by the previous kernel chain, read by ln1, the out-projection
        # residual and ln1's backward (the last kernel of the layer's backward)
        t = tr["ids"][f"l{i - 1}.xo" if i else "x0"]
        assert life["active"][t][-1] == bwd0 + 27 * (L - 1 - i) + 23
    # optimizer moments are touched once per iteration: one wrap-around period of length N
    t = tr["ids"]["l0.w_fc1.m"]
    (k,) = life["active"][t]
    assert [p for p in life["periods"] if p[0] == t] == [(t, tr["tensors"][t][0], k, k + N)]
    # weights of layer 0: forward use, two backward uses (dX, AdamW); wrap period closes the cycle
    t = tr["ids"]["l0.w_fc1"]
    a = life["active"][t]
    assert len(a) == 3 and [p[2:] for p in life["periods"] if p[0] == t] == [(a[0], a[1]), (a[1], a[2]), (a[2], a[0] + N)]
    # token and label buffers never become candidates
    assert not [p for p in life["periods"] if p[0] in (tr["ids"]["tokens"], tr["ids"]["labels"])]


def test_memory_vector_against_a_direct_recount():
    cfg = CONFIGS["tiny_llama_fp32"]
    tr = ot.build_trace(cfg)
    life = op.analyze_lifetimes(tr)
    N = len(tr["kernels"])
    first, last = {}, {}
    for k, (_, operands, _) in enumerate(tr["kernels"]):
        for t, _ in operands:
            first.setdefault(t, k)
            last[t] = k
    for k in range(N):
        tot = 0
        for t, (s, kind, _) in enumerate(tr["tensors"]):
            if t < tr["n_persistent"] or first[t] <= k <= last[t]:
                tot += s
        assert life["M"][k] == tot
    # peak of a GPT trace in closed form: at the head's weight-gradient kernel everything saved by
    # the forward pass (h1, qkv, ao, xm, h2, u, act, xo, statistics per layer), the logits, dhf and
    # the head gradient are live
    cfg = CONFIGS["tiny_gpt_fp32"]
    tr = ot.build_trace(cfg)
    life = op.analyze_lifetimes(tr)
    k = int(np.argmax(life["M"]))
    assert tr["kernels"][k][0] == ot.GEMM_DW and k == 1 + 8 * cfg["L"] + 4 + 1
    pers = sum(t[0] for t in tr["tensors"][:tr["n_persistent"]])
    S, d, f, V, H, L = 128, 128, 512, 1024, 4, 2
    r = lambda n: (n + 255) // 256 * 256
    per_layer = 4 * (5 * S * d + 3 * S * d + 2 * S * f) + 2 * r(S * 2 * 4) + r(2 * H * 64 * 4)
    saved = r(4 * S * d) + L * per_layer + r(4 * S * d) + r(S * 2 * 4)       # x0, layers, hf, stf
    live = pers + saved + 4 * S * V + 4 * S * d + 4 * V * d     # logits, dhf, g.w_head (row losses are dead)
    assert life["M"][k] == live


# ------------------------------------------------------------------ planner properties
def test_capacity_at_least_peak_gives_empty_plan():
    tr = ot.build_trace(CONFIGS["tiny_gpt_fp32"])
    life = op.analyze_lifetimes(tr)
    pl = op.build_plan(tr, life, max(life["M"]), 25 * 10**9)
    assert pl["entries"] == [] and pl["Mp"] == life["M"]


def test_infinite_bandwidth_first_choice_by_naive_scoring():
    rng = np.random.default_rng(5)
    for trial in range(30):
        tr = random_trace(rng, N=10, n_pers=2, n_trans=6)
        life = op.analyze_lifetimes(tr)
        N = 10
        cap = int(max(life["M"]) * 0.8)
        try:
            pl = op.build_plan(tr, life, cap, 0)
        except ValueError:
            continue
        # with unlimited bandwidth the window of a period is every kernel strictly inside it
        best = None
        for (t, s, a, b) in life["periods"]:
            score = sum(tr["tau"][k % N] for k in range(a + 1, b) if life["M"][k % N] > cap)
            if score > 0 and (best is None or (score, s, -a, -t, -b) > best[0]):
                best = ((score, s, -a, -t, -b), (t, a, b))
        first = [e for e in pl["entries"] if e[5] == 0]
        if best is None:
            assert not first or first[0][4] == 1
            continue
        t, a, b = best[1]
        off = [e for e in first if e[1] == op.OFFLOAD][0]
        pre = [e for e in first if e[1] == op.PREFETCH][0]
        assert (off[0], off[2], off[3]) == (t, a + 1, a + 1) and (pre[2], pre[3]) == (b, b)
        orp.check_plan(tr, life, pl, cap)


def test_infinite_bandwidth_needs_no_stalls_and_exhaustive_minimum():
    rng = np.random.default_rng(11)
    gaps = []
    for trial in range(25):
        tr = random_trace(rng, N=8, n_pers=2, n_trans=5)
        life = op.analyze_lifetimes(tr)
        N = 8
        P = life["periods"]
        if len(P) > 12:
            continue
        cap = int(max(life["M"]) * 0.75)
        # exhaustive search over subsets of periods, whole-period windows
        best_bytes = None
        for r in range(len(P) + 1):
            for sub in itertools.combinations(P, r):
                M2 = list(life["M"])
                for (t, s, a, b) in sub:
                    for k in range(a + 1, b):
                        M2[k % N] -= s
                if max(M2) <= cap:
                    tot = sum(p[1] for p in sub)
                    best_bytes = tot if best_bytes is None else min(best_bytes, tot)
        if best_bytes is None:
            with pytest.raises(ValueError):
                op.build_plan(tr, life, cap, 0)
            continue
        pl = op.build_plan(tr, life, cap, 0)
        st = orp.check_plan(tr, life, pl, cap)
        assert pl["n_forced"] == 0            # a feasible subset exists => the greedy loop finds one
        assert st["bytes_per_direction"] >= best_bytes
        gaps.append(st["bytes_per_direction"] / max(1, best_bytes))
    assert gaps and np.median(gaps) < 2.0     # heuristic, not optimal: report-level sanity only


@pytest.mark.parametrize("duplex", [True, False])
def test_random_traces_satisfy_the_residency_invariants(duplex):
    rng = np.random.default_rng(2)
    n_ok = 0
    for trial in range(60):
        tr = random_trace(rng, N=int(rng.integers(6, 30)), n_pers=int(rng.integers(1, 5)),
                          n_trans=int(rng.integers(3, 25)))
        life = op.analyze_lifetimes(tr)
        cap = int(max(life["M"]) * rng.uniform(0.3, 0.95))
        bw = int(10 ** rng.uniform(8, 11))
        try:
            pl = op.build_plan(tr, life, cap, bw, duplex=duplex)
        except ValueError:
            act = max(sum(tr["tensors"][t][0] for t, _ in ops) for _, ops, _ in tr["kernels"])
            continue
        st = orp.check_plan(tr, life, pl, cap)
        sim = orp.simulate(tr, pl, bw, duplex=duplex)
        assert sim["step_ns"] >= sim["compute_ns"]
        if pl["n_forced"] == 0 and pl["entries"]:
            # every transfer was placed inside an idle window of the modelled timeline
            assert st["bytes_per_direction"] * 10**9 // bw <= sim["compute_ns"] + len(pl["entries"])
        n_ok += 1
    assert n_ok > 20


def test_error_when_operands_alone_exceed_capacity():
    tr = mini_trace([100, 100, 100], [("a", 800, False, [0, 1, 2]), ("b", 400, False, [1])])
    life = op.analyze_lifetimes(tr)
    with pytest.raises(ValueError):
        op.build_plan(tr, life, 1000, 10**9)


def test_plan_does_not_depend_on_the_order_of_the_period_list():
    tr = ot.build_trace(CONFIGS["tiny_gpt_fp32"])
    life = op.analyze_lifetimes(tr)
    cap = max(life["M"]) // 2
    pl = op.build_plan(tr, life, cap, 25 * 10**9)
    rng = np.random.default_rng(0)
    life2 = dict(life, periods=[life["periods"][i] for i in rng.permutation(len(life["periods"]))])
    assert op.build_plan(tr, life2, cap, 25 * 10**9) == pl
    orp.check_plan(tr, life, pl, cap)


@pytest.mark.parametrize("name,bw", [("tiny_gpt_fp32", 25 * 10**9), ("tiny_gpt_fp32", 10**8),
                                     ("tiny_llama_fp32", 25 * 10**9), ("tiny_llama_fp32", 10**12)])
def test_model_traces_plan_validly_at_half_peak(name, bw):
    tr = ot.build_trace(CONFIGS[name])
    life = op.analyze_lifetimes(tr)
    cap = max(life["M"]) // 2
    for min_bytes in (0, 65536):
        pl = op.build_plan(tr, life, cap, bw, min_bytes=min_bytes)
        st = orp.check_plan(tr, life, pl, cap)
        assert st["bytes_per_direction"] >= max(life["M"]) - cap
    # tiny bandwidth: nothing fits the modelled timeline, so every entry is forced and urgent
    if bw == 10**8:
        pl = op.build_plan(tr, life, cap, 10**5)
        assert pl["n_greedy"] == 0 and all(e[4] == 1 for e in pl["entries"])


def test_channel_gap_search():
    ch = op.Channel(1000)
    ch.insert(100, 200)
    ch.insert(900, 1050)                   # wraps: [900,1000) and [0,50)
    assert list(zip(ch.b, ch.e)) == [(0, 50), (100, 200), (900, 1000)]
    assert ch.earliest_gap(0, 1000, 50) == 50
    assert ch.earliest_gap(0, 1000, 60) == 200
    assert ch.earliest_gap(60, 1000, 40) == 60
    assert ch.earliest_gap(150, 400, 100) == 200
    assert ch.earliest_gap(150, 290, 100) is None
    assert ch.latest_gap(0, 1000, 100) == 800
    assert ch.latest_gap(0, 950, 100) == 800
    assert ch.latest_gap(0, 150, 50) == 50
    assert ch.latest_gap(0, 150, 51) is None
    assert ch.earliest_gap(950, 1300, 60) == 1200        # second cycle: [1000,1050) and [1100,1200) busy
    assert ch.latest_gap(950, 2100, 60) == 1840          # [2050,2100) is only 50 long, [1900,2050) busy


# ------------------------------------------------------------------ the schedule against hand-written launch lists
OP_NAMES = ["EMBED_FWD", "NORM_FWD", "GEMM", "ROPE_FWD", "ATTN_FWD", "GELU_FWD", "SWIGLU_FWD", "CE_FWD_BWD", "LOSS_REDUCE",
            "GEMM_DX", "GEMM_DW", "BIAS_GRAD", "GELU_BWD", "SWIGLU_BWD", "NORM_BWD", "NORM_BWD_PARAMS", "ATTN_BWD_PRE",
            "ATTN_BWD", "ROPE_BWD", "EMBED_BWD", "POSEMB_BWD", "ADAMW"]


def _launch_list(path):
    import os
    from planlib import GOLDEN
    out = []
    for line in open(os.path.join(GOLDEN, path)):
        if line.startswith("#") or not line.strip():
            continue
        op_, r, w, rw = [x.strip() for x in line.split("|")]
        out.append((op_, sorted(r.split()), sorted(w.split()), sorted(rw.split())))
    return out


@pytest.mark.parametrize("golden,cfg", [
    ("trace_gpt_one_layer.txt", dict(arch="gpt", L=1, d=64, H=2, f=256, V=300, T=32, B=2, precision="fp32")),
    ("trace_llama_one_layer.txt", dict(arch="llama", L=1, d=64, H=2, f=176, V=300, T=64, B=2, precision="bf16"))])
def test_schedule_against_the_hand_written_launch_list(golden, cfg):
    """Every launch of a one-layer model, with the names of the tensors it reads, writes and updates, against a list
    written by hand from the dataflow; the same layer pattern repeats for deeper models (checked below by comparing
    layer 0 of a two-layer trace with the list, tensor names shifted)."""
    tr = ot.build_trace(cfg)
    names = [t[2] for t in tr["tensors"]]
    got = []
    for op_, operands, _ in tr["kernels"]:
        r = sorted(names[t] for t, fl in operands if fl == ot.READ)
        w = sorted(names[t] for t, fl in operands if fl == ot.WRITE)
        rw = sorted(names[t] for t, fl in operands if fl == (ot.READ | ot.WRITE))
        got.append((OP_NAMES[op_], r, w, rw))
    want = _launch_list(golden)
    assert len(got) == len(want)
    for i, (g, w) in enumerate(zip(got, want)):
        assert g == w, (i, g, w)
    # two layers: layer 1's launches are layer 0's with "l0." -> "l1.", its input x0 -> l0.xo, and the gradient that
    # enters it from above (dxf) -> stays; layer 0's backward takes l1.dx where the one-layer list has dxf
    tr2 = ot.build_trace(dict(cfg, L=2))
    names2 = [t[2] for t in tr2["tensors"]]
    fwd1 = [k for k in tr2["kernels"] if any(names2[t].startswith("l1.") for t, _ in k[1])]
    fwd0 = [k for k in tr["kernels"] if any(names[t].startswith("l0.") for t, _ in k[1])]
    ren = lambda n: "l0.xo" if n == "x0" else n.replace("l0.", "l1.") if n.startswith(("l0.", "g.l0.")) or ".l0." in n else n
    per_layer_one = [(k[0], sorted(ren(names[t]).replace("g.l0.", "g.l1.") for t, _ in k[1])) for k in fwd0
                     if k[0] not in (ot.EMBED_FWD, ot.EMBED_BWD, ot.POSEMB_BWD) and not (k[0] == ot.NORM_FWD and "hf" in [names[t] for t, _ in k[1]])
                     and not (k[0] == ot.NORM_BWD and "dxf" in [names[t] for t, _ in k[1]] and "partf" in [names[t] for t, _ in k[1]])]
    per_layer_two = [(k[0], sorted(names2[t] for t, _ in k[1])) for k in fwd1
                     if not (k[0] == ot.NORM_FWD and "hf" in [names2[t] for t, _ in k[1]])
                     and not (k[0] == ot.NORM_BWD and "partf" in [names2[t] for t, _ in k[1]])
                     and not any(names2[t].startswith("l0.") and names2[t] != "l0.xo" for t, _ in k[1])]
    assert per_layer_two == per_layer_one
