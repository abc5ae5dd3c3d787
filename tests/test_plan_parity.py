"""Library (C ABI, pure-CPU half) against the oracle, bit for bit: trace, lifetimes, plan."""
import numpy as np
import pytest

import paper_2506_06472_amd as tio
from oracle import plan as op
from oracle import replay as orp
from oracle import trace as ot
from synth import CONFIGS
from planlib import golden_options, load_golden, random_trace


def lib_trace_from_oracle(tr):
    return tio.tio_trace_import(tr["n_persistent"], [ops for _, ops, _ in tr["kernels"]],
                                [t[0] for t in tr["tensors"]], tr["tau"], [t[1] for t in tr["tensors"]],
                                [k[0] for k in tr["kernels"]])


def assert_same_plan(tr, lt, ll, cap, bw, **kw):
    """Library plan == oracle plan at the planning capacity the library settled on."""
    try:
        pl = tio.tio_build_plan(lt, ll, cap, bw, **kw).export()
    except tio.TioError as e:
        assert e.code == -3, e
        with pytest.raises(ValueError):
            op.build_plan(tr, op.analyze_lifetimes(tr), cap, bw, duplex=kw.get("duplex", True),
                          min_bytes=kw.get("min_bytes", 0), clamp_benefit=kw.get("clamp_benefit", False))
        return None
    life = op.analyze_lifetimes(tr)
    ref = op.build_plan(tr, life, pl["planning_cap"], bw, duplex=kw.get("duplex", True), min_bytes=kw.get("min_bytes", 0),
                        clamp_benefit=kw.get("clamp_benefit", False))
    assert pl["entries"] == ref["entries"]
    assert pl["Mp"] == ref["Mp"]
    assert (pl["n_greedy"], pl["n_forced"]) == (ref["n_greedy"], ref["n_forced"])
    st = orp.check_plan(tr, life, ref, pl["planning_cap"])
    assert st["bytes_per_direction"] == pl["bytes_per_direction"]
    arena = kw.get("arena_bytes") or cap
    assert pl["arena_needed"] <= arena
    orp.check_layout(tr, life, ref, pl["allocs"], arena)
    return pl


@pytest.mark.parametrize("name", list(CONFIGS))
def test_trace_and_lifetimes_bit_exact(name):
    cfg = CONFIGS[name]
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    v = lt.export()
    assert (v["n_kernels"], v["n_tensors"], v["n_persistent"]) == (len(tr["kernels"]), len(tr["tensors"]), tr["n_persistent"])
    assert v["op"].tolist() == [k[0] for k in tr["kernels"]]
    assert v["flops"].tolist() == [k[2] for k in tr["kernels"]]
    assert v["tau"].tolist() == tr["tau"]
    assert v["tensor_bytes"].tolist() == [t[0] for t in tr["tensors"]]
    assert v["tensor_kind"].tolist() == [t[1] for t in tr["tensors"]]
    off = [0]
    flat = []
    for _, ops, _ in tr["kernels"]:
        flat += ops
        off.append(len(flat))
    assert v["operand_off"].tolist() == off
    assert v["operand_tensor"].tolist() == [t for t, _ in flat]
    assert v["operand_flags"].tolist() == [f for _, f in flat]
    life = op.analyze_lifetimes(tr)
    lv = tio.tio_analyze_lifetimes(lt).export()
    assert lv["M"].tolist() == life["M"]
    got = sorted(zip(lv["tensor"].tolist(), lv["bytes"].tolist(), lv["start"].tolist(), lv["end"].tolist()))
    assert got == sorted(life["periods"])
    # parameter list
    from oracle.model import param_specs
    assert [(n, int(np.prod(s))) for n, s, _ in param_specs(cfg)] == [(n, r * c) for n, r, c in tio.tio_param_list(cfg)]


@pytest.mark.parametrize("name", ["plan_example_a.txt", "plan_example_c.txt", "plan_example_e.txt", "plan_example_f.txt"])
def test_golden_examples_through_the_c_abi(name):
    tr, cap, bw, entries, Mp, _ = load_golden(name)
    lt = lib_trace_from_oracle(tr)
    ll = tio.tio_analyze_lifetimes(lt)
    pl = tio.tio_build_plan(lt, ll, cap, bw, arena_bytes=1 << 20, **golden_options(name)).export()
    assert pl["planning_cap"] == cap and pl["entries"] == entries and pl["Mp"] == Mp


def test_golden_infeasible_through_the_c_abi():
    tr, cap, bw, *_ = load_golden("plan_example_b.txt")
    lt = lib_trace_from_oracle(tr)
    with pytest.raises(tio.TioError) as e:
        tio.tio_build_plan(lt, tio.tio_analyze_lifetimes(lt), cap, bw)
    assert e.value.code == -3


@pytest.mark.parametrize("name,frac,bw,min_bytes", [
    ("tiny_gpt_fp32", 0.5, 25 * 10**9, 0), ("tiny_gpt_fp32", 0.5, 10**8, 0), ("tiny_gpt_fp32", 0.3, 0, 0),
    ("tiny_gpt_fp32", 0.7, 10**12, 65536), ("tiny_llama_fp32", 0.5, 25 * 10**9, 0),
    ("tiny_llama_fp32", 0.4, 10**9, 32768), ("tiny_llama_fp32", 0.9, 10**10, 0)])
def test_model_plans_bit_exact(name, frac, bw, min_bytes):
    cfg = CONFIGS[name]
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    cap = int(max(op.analyze_lifetimes(tr)["M"]) * frac)
    for duplex in (True, False):
        pl = assert_same_plan(tr, lt, ll, cap, bw, min_bytes=min_bytes, duplex=duplex)
        assert pl is not None
        tio.tio_plan_validate(lt, ll, tio.tio_build_plan(lt, ll, cap, bw, min_bytes=min_bytes, duplex=duplex))


def test_random_synthetic_traces_bit_exact():
    rng = np.random.default_rng(9)
    n = 0
    for trial in range(80):
        tr = random_trace(rng, N=int(rng.integers(5, 40)), n_pers=int(rng.integers(1, 6)),
                          n_trans=int(rng.integers(3, 30)))
        # the library rounds nothing itself, but addresses are 256-aligned: use 256-multiples
        tr["tensors"] = [(s * 32, k, nme) for s, k, nme in tr["tensors"]]
        lt = lib_trace_from_oracle(tr)
        ll = tio.tio_analyze_lifetimes(lt)
        life = op.analyze_lifetimes(tr)
        cap = int(max(life["M"]) * rng.uniform(0.3, 1.0)) // 256 * 256
        bw = int(10 ** rng.uniform(9, 12.5))
        pl = assert_same_plan(tr, lt, ll, cap, bw, duplex=bool(trial % 2), arena_bytes=4 * max(life["M"]))
        n += pl is not None
    assert n > 30


def test_hand_worked_example_where_the_two_benefit_readings_differ():
    """tests/golden/plan_example_g.txt: the formula of Algorithm 1 takes the larger of two tensors that tie, the prose
    reading the one that is just large enough; both oracles and the library through the C ABI."""
    from oracle import plan_plain as opp
    tr, cap, bw, entries, _, _ = load_golden("plan_example_g.txt")
    formula, prose = entries[:2], entries[2:]
    life = op.analyze_lifetimes(tr)
    lt = lib_trace_from_oracle(tr)
    ll = tio.tio_analyze_lifetimes(lt)
    for clamp, want, Mp in ((False, formula, [500, 300, 300, 500]), (True, prose, [500, 600, 600, 500])):
        ref = op.build_plan(tr, life, cap, bw, clamp_benefit=clamp)
        assert ref["entries"] == want and ref["Mp"] == Mp
        assert opp.build_plan(tr, cap, bw, clamp_benefit=clamp)["entries"] == want
        pl = tio.tio_build_plan(lt, ll, cap, bw, arena_bytes=4 * cap, clamp_benefit=clamp).export()
        assert pl["entries"] == want and pl["Mp"] == Mp


def test_prose_benefit_variant_bit_exact_and_different_from_the_formula():
    """clamp_benefit (a kernel counts only with the bytes it is over capacity, the prose of "Quantify the benefit and
    cost") through the C ABI against the oracle's exact-fraction ranking: random traces, where the two variants do pick
    different periods, and the small model traces."""
    rng = np.random.default_rng(21)
    n = differ = 0
    for trial in range(80):
        tr = random_trace(rng, N=int(rng.integers(5, 40)), n_pers=int(rng.integers(1, 6)),
                          n_trans=int(rng.integers(3, 30)))
        tr["tensors"] = [(s * 32, k, nme) for s, k, nme in tr["tensors"]]
        lt = lib_trace_from_oracle(tr)
        ll = tio.tio_analyze_lifetimes(lt)
        life = op.analyze_lifetimes(tr)
        cap = int(max(life["M"]) * rng.uniform(0.5, 1.0)) // 256 * 256
        bw = int(10 ** rng.uniform(9, 12.5))
        kw = dict(duplex=bool(trial % 2), arena_bytes=4 * max(life["M"]))
        pl = assert_same_plan(tr, lt, ll, cap, bw, clamp_benefit=True, **kw)
        if pl is None:
            continue
        n += 1
        try:
            plain = tio.tio_build_plan(lt, ll, cap, bw, **kw).export()
            differ += plain["entries"] != pl["entries"]
        except tio.TioError:
            pass
    assert n > 30 and differ >= 5, (n, differ)
    for name, frac, bw in (("tiny_gpt_fp32", 0.5, 25 * 10**9), ("tiny_llama_fp32", 0.4, 10**9), ("tiny_llama_fp32", 0.8, 10**10)):
        cfg = CONFIGS[name]
        tr = ot.build_trace(cfg)
        lt = tio.tio_trace_build(cfg)
        ll = tio.tio_analyze_lifetimes(lt)
        cap = int(max(op.analyze_lifetimes(tr)["M"]) * frac)
        for duplex in (True, False):
            assert assert_same_plan(tr, lt, ll, cap, bw, duplex=duplex, clamp_benefit=True) is not None


def test_uncapped_plan_is_empty_and_layout_valid():
    cfg = CONFIGS["tiny_gpt_fp32"]
    tr = ot.build_trace(cfg)
    life = op.analyze_lifetimes(tr)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    pl = tio.tio_build_plan(lt, ll, 2**62, 0).export()
    assert pl["entries"] == [] and pl["Mp"] == life["M"]
    assert max(life["M"]) <= pl["arena_needed"] <= int(1.3 * max(life["M"]))
    orp.check_layout(tr, life, dict(entries=[]), pl["allocs"], pl["arena_needed"])


def test_stale_and_invalid_arguments_are_reported():
    lt = tio.tio_trace_build(CONFIGS["tiny_gpt_fp32"])
    lt2 = tio.tio_trace_build(CONFIGS["tiny_llama_fp32"])
    with pytest.raises(tio.TioError) as e:
        tio.tio_build_plan(lt, tio.tio_analyze_lifetimes(lt2), 10**6, 10**9)
    assert e.value.code == -5
    with pytest.raises(tio.TioError):
        tio.tio_trace_build(dict(CONFIGS["tiny_gpt_fp32"], d=130))
    with pytest.raises(tio.TioError):
        lt.set_tau([1, 2, 3])


@pytest.mark.parametrize("name", ["llama_7b_bf16", "llama_13b_bf16", "llama_30b_bf16"])
def test_large_configurations_plan_bit_exact_at_full_size(name):
    """The three Llama-shaped workloads at their stated capacities and bandwidth (modelled kernel times)."""
    cfg = CONFIGS[name]
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    life = op.analyze_lifetimes(tr)
    pl = assert_same_plan(tr, lt, ll, cfg["cap_bytes"], cfg.get("slow_tier_bw", 25 * 10**9), min_bytes=1 << 20)
    assert pl["bytes_per_direction"] >= max(life["M"]) - cfg["cap_bytes"]
    assert pl["arena_needed"] <= cfg["cap_bytes"]


@pytest.mark.slow
def test_gpt2_small_plan_bit_exact_at_full_size():
    cfg = CONFIGS["gpt2_small_bf16"]
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    cap = int(max(op.analyze_lifetimes(tr)["M"]) * cfg["cap_frac"])
    pl = assert_same_plan(tr, lt, ll, cap, 25 * 10**9, min_bytes=1 << 20)
    assert pl["bytes_per_direction"] >= max(op.analyze_lifetimes(tr)["M"]) - cap


def test_library_exports_every_declared_symbol():
    import os
    import re
    hdr = open(os.path.join(os.path.dirname(__file__), "..", "include", "teraio.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(tio_[a-z0-9_]+)\s*\(", hdr)))
    assert len(names) >= 30 and "tio_train_step" in names and "tio_plan_simulate" in names
    lib = tio.binding.lib()
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing
    assert lib.tio_version().decode().strip() and lib.tio_last_error() is not None


@pytest.mark.parametrize("name,frac", [("tiny_gpt_fp32", 0.5), ("tiny_llama_fp32", 0.4), ("gpt2_small_bf16", 0.4)])
def test_performance_model_bit_exact(name, frac):
    """tio_plan_simulate against the oracle's model (itself pinned by the hand-worked examples): same integer
    nanoseconds for every bandwidth, duplex or not, and for one to three iterations."""
    cfg = CONFIGS[name] if name != "gpt2_small_bf16" else dict(CONFIGS[name], L=3)
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    life = op.analyze_lifetimes(tr)
    cap = int(max(life["M"]) * frac) // 256 * 256
    for bw in (10**9, 25 * 10**9, 0):
        for duplex in (True, False):
            pl = tio.tio_build_plan(lt, ll, cap, bw, duplex=duplex)
            pe = pl.export()
            ref = op.build_plan(tr, life, pe["planning_cap"], bw, duplex=duplex)
            assert pe["entries"] == ref["entries"]
            for sim_bw in (bw, 5 * 10**9):
                for it in (1, 3):
                    want = orp.simulate(tr, ref, sim_bw, duplex=duplex, iterations=it)
                    got = tio.tio_plan_simulate(lt, pl, sim_bw, duplex=duplex, iterations=it)
                    assert got == (want["step_ns"], want["compute_ns"]), (bw, duplex, sim_bw, it)


def test_performance_model_golden_through_the_c_abi():
    tr, cap, bw, entries, Mp, _ = load_golden("plan_example_c.txt")
    lt = lib_trace_from_oracle(tr)
    ll = tio.tio_analyze_lifetimes(lt)
    pl = tio.tio_build_plan(lt, ll, cap, bw, arena_bytes=1 << 20)
    # the one pair is fully exposed: 8 kernels of 100 ns + 150 ns offload + 150 ns prefetch
    assert tio.tio_plan_simulate(lt, pl, bw) == (1100, 800)
    assert tio.tio_plan_simulate(lt, tio.tio_build_plan(lt, ll, 10**6, bw, arena_bytes=1 << 21), bw) == (800, 800)
    with pytest.raises(tio.TioError):
        tio.tio_plan_simulate(lt, pl, bw, iterations=0)


def test_performance_model_invariants_and_sweep_tool():
    """For a fixed plan the predicted step time never grows with bandwidth, equals the compute time when
    transfers are instantaneous, and is at least max(compute, bytes / bandwidth); the sweep tool runs."""
    import io
    from paper_2506_06472_amd import sweep as sw
    cfg = dict(CONFIGS["gpt2_small_bf16"], L=4, V=8192)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    cap = int(ll.export()["M"].max() * 0.5) // 256 * 256
    pl = tio.tio_build_plan(lt, ll, cap, 25 * 10**9)
    moved = pl.export()["bytes_per_direction"]
    prev = None
    for bw in (10**9, 4 * 10**9, 25 * 10**9, 10**11, 10**13):
        step, comp = tio.tio_plan_simulate(lt, pl, bw)
        assert step >= comp and step >= moved * 10**9 // bw
        assert prev is None or step <= prev
        prev = step
    assert tio.tio_plan_simulate(lt, pl, 0) == (comp, comp)
    out = io.StringIO()
    rows = sw.sweep("tiny_gpt_fp32", [10**9, 25 * 10**9], out=out)
    sw.characterize("tiny_gpt_fp32", out=out)
    assert len(rows) == 2 and rows[0][2] >= rows[0][3] and "inactive periods" in out.getvalue()
    # a host-memory tier beside the slow tier, and one channel shared by both directions
    rows = sw.sweep("tiny_gpt_fp32", [10**9], out=out, host_bw=2 * 10**10, host_budgets=(0, 10**5, 10**7))
    assert [r[1] for r in rows] == [0, 10**5, 10**7] and rows[2][2] <= rows[0][2] and sum(rows[2][4]["tier"]) > 0
    shared = sw.sweep("tiny_gpt_fp32", [10**9], out=out, shared_channel=True)
    assert shared[0][2] >= rows[0][2]
