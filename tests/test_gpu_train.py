"""GPU parity of whole training steps (C ABI: tio_ctx_create, tio_params_load, tio_train_step, ...)
against the CPU oracle, and bitwise equality of runs with and without offloading."""
import numpy as np
import pytest

from oracle import model as om
from synth import CONFIGS
from gpulib import make_inputs, plans_for, read_state

pytestmark = pytest.mark.gpu

# 512 tokens: the weight-gradient GEMMs of this shape run with a split contraction
SMALL_BF16 = dict(arch="gpt", L=2, d=256, H=4, f=1024, V=1000, T=256, B=2, precision="bf16", lr=3e-4)
SMALL_LLAMA_BF16 = dict(arch="llama", L=2, d=256, H=2, f=688, V=520, T=96, B=2, precision="bf16", lr=3e-4)


def _ctx(cfg, plan_export, extra_arena=0, bw=0):
    import paper_2506_06472_amd as tio
    return tio.tio_ctx_create(cfg, plan_export["arena_needed"] + extra_arena, plan_export["host_needed"] + (1 << 20), bw)


@pytest.mark.parametrize("name", ["tiny_gpt_fp32", "tiny_llama_fp32"])
def test_fp32_steps_match_oracle(name):
    cfg = CONFIGS[name]
    params, tok, lab = make_inputs(cfg, seed=0)
    lt, ll, up, _, peak = plans_for(cfg)
    ctx = _ctx(cfg, up.export())
    ctx.tio_params_load(params)
    ref = om.Trainer(cfg, params)
    for step in range(3):
        print(f"{name} step {step}", flush=True)
        st = ctx.tio_train_step(tok, lab, None, capture_grads=True)
        rl = ref.step(tok, lab)
        assert abs(st["loss"] - rl) <= 1e-5 * abs(rl), (step, st["loss"], rl)
        for n, _, _ in ctx.params:
            g = ctx.tio_grads_read(n).astype(np.float64)
            gr = ref.last_grads[n].reshape(g.shape)
            scale = np.abs(gr).max()
            if scale < 1e-12:       # e.g. the key bias: its exact gradient is zero
                assert np.abs(g).max() <= 1e-7, n
            else:
                assert np.abs(g - gr).max() <= 1e-4 * scale, (step, n, np.abs(g - gr).max() / scale)
    # parameters after three steps: tight where the update is well conditioned, 2*lr per step elsewhere
    for n, _, _ in ctx.params:
        w = ctx.tio_params_read(n, 0).astype(np.float64)
        wr = ref.p[n].reshape(w.shape)
        assert np.abs(w - wr).max() <= 3 * 2 * cfg["lr"] + 1e-6, n
        m = ctx.tio_params_read(n, 2).astype(np.float64)
        mr = ref.m[n].reshape(m.shape)
        assert np.abs(m - mr).max() <= 1e-4 * max(np.abs(mr).max(), 1e-12) + 1e-9, n
    frac_close = np.mean([np.mean(np.abs(ctx.tio_params_read(n, 0) - ref.p[n].reshape(-1).reshape(ctx.tio_params_read(n, 0).shape)) < 1e-5)
                          for n, _, _ in ctx.params if n.startswith("l0.w_")])
    assert frac_close > 0.99
    ctx.close()


@pytest.mark.parametrize("name,cap_frac,bw,min_bytes", [
    ("tiny_gpt_fp32", 0.5, 25 * 10**9, 0), ("tiny_gpt_fp32", 0.3, 10**9, 0), ("tiny_llama_fp32", 0.5, 25 * 10**9, 0),
    ("tiny_llama_fp32", 0.45, 0, 16384)])
def test_offloading_leaves_numerics_bitwise_unchanged(name, cap_frac, bw, min_bytes):
    _bitwise_under_cap(name, cap_frac, bw, min_bytes, 0)


@pytest.mark.parametrize("name,cap_frac,bw,passes", [("tiny_gpt_fp32", 0.3, 10**8, 4), ("tiny_llama_fp32", 0.5, 10**9, 3)])
def test_re_timed_plans_leave_numerics_bitwise_unchanged(name, cap_frac, bw, passes):
    """Plans from the re-timing loop (Algorithm 1 run again on the stalled timeline) at bandwidths where a later pass
    wins: the capped run still gives the bits of the uncapped one and moves exactly the planned bytes."""
    ce = _bitwise_under_cap(name, cap_frac, bw, 0, passes)
    assert ce["retime_pass"] > 0


def _bitwise_under_cap(name, cap_frac, bw, min_bytes, passes):
    cfg = CONFIGS[name]
    params, tok, lab = make_inputs(cfg, seed=1)
    lt, ll, up, cp, peak = plans_for(cfg, cap_frac, bw, min_bytes, retime_passes=passes)
    ce = cp.export()
    print(f"{name}: peak {peak} cap {ce['cap']} planning cap {ce['planning_cap']} entries {len(ce['entries'])} "
          f"forced {ce['n_forced']} arena {ce['arena_needed']}", flush=True)
    assert ce["arena_needed"] <= ce["cap"] < peak
    names = [n for n, _, _ in __import__("paper_2506_06472_amd").tio_param_list(cfg)]
    runs = []
    for plan, arena in ((None, up.export()), (cp, ce)):
        ctx = _ctx(cfg, dict(arena_needed=arena["arena_needed"] if plan is None else ce["cap"],
                             host_needed=max(arena["host_needed"], ce["host_needed"])), bw=bw)
        ctx.tio_params_load(params)
        losses = []
        for step in range(4):
            print(f"  plan={'capped' if plan else 'none'} step {step}", flush=True)
            st = ctx.tio_train_step(tok, lab, plan)
            losses.append(st["loss"])
            if plan is not None:
                # steady state moves exactly the planned bytes; the first iteration after the plan is
                # installed skips offloads that belong to the end of a previous iteration
                assert st["h2d_bytes"] == ce["bytes_per_direction"]
                assert (st["d2h_bytes"] == ce["bytes_per_direction"]) if step else (st["d2h_bytes"] <= ce["bytes_per_direction"])
        state = read_state(ctx, names, cfg["precision"] == "bf16")
        runs.append((losses, state))
        ctx.close()
    (l0, s0), (l1, s1) = runs
    assert np.array(l0, dtype=np.float32).tobytes() == np.array(l1, dtype=np.float32).tobytes(), (l0, l1)
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key
    assert l0[-1] < l0[0]
    return ce


@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_LLAMA_BF16], ids=["gpt", "llama"])
def test_bf16_loss_and_grads_against_oracle_and_bitwise_offload(cfg):
    import paper_2506_06472_amd as tio
    params, tok, lab = make_inputs(cfg, seed=2)
    lt, ll, up, cp, peak = plans_for(cfg, 0.4, 25 * 10**9, 0)
    ce = cp.export()
    ctx = _ctx(cfg, up.export())
    ctx.tio_params_load(params)
    ref = om.Trainer(cfg, params)
    losses = []
    for step in range(3):
        print(f"bf16 {cfg['arch']} step {step}", flush=True)
        st = ctx.tio_train_step(tok, lab, None, capture_grads=(step == 0))
        rl = ref.step(tok, lab)
        losses.append(st["loss"])
        assert abs(st["loss"] - rl) <= 2e-2 * abs(rl), (step, st["loss"], rl)
        if step == 0:
            for n, _, _ in ctx.params:
                g = ctx.tio_grads_read(n).astype(np.float64)
                gr = ref.last_grads[n].reshape(g.shape)
                scale = np.abs(gr).max()
                if scale > 1e-9:
                    assert np.abs(g - gr).max() <= 6e-2 * scale, (n, np.abs(g - gr).max() / scale)
    names = [n for n, _, _ in ctx.params]
    s0 = read_state(ctx, names, True)
    ctx.close()
    ctx = tio.tio_ctx_create(cfg, ce["cap"], ce["host_needed"] + (1 << 20), 25 * 10**9)
    ctx.tio_params_load(params)
    l1 = [ctx.tio_train_step(tok, lab, cp)["loss"] for _ in range(3)]
    s1 = read_state(ctx, names, True)
    ctx.close()
    assert np.array(losses, dtype=np.float32).tobytes() == np.array(l1, dtype=np.float32).tobytes(), (losses, l1)
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key


def test_measured_profile_gives_the_same_structure_and_positive_times():
    import paper_2506_06472_amd as tio
    cfg = CONFIGS["tiny_gpt_fp32"]
    params, tok, lab = make_inputs(cfg, seed=0)
    lt, ll, up, _, peak = plans_for(cfg)
    ctx = _ctx(cfg, up.export())
    ctx.tio_params_load(params)
    tr = ctx.tio_profile_iteration(tok, lab, tio.PROFILE_MEASURED).export()
    # the structure the launcher recorded while it ran the kernels, against the oracle's trace of the same model
    from oracle import trace as ot
    otr = ot.build_trace(cfg)
    assert (tr["n_kernels"], tr["n_tensors"], tr["n_persistent"]) == (len(otr["kernels"]), len(otr["tensors"]), otr["n_persistent"])
    assert tr["op"].tolist() == [k[0] for k in otr["kernels"]]
    flat, off = [], [0]
    for _, ops, _ in otr["kernels"]:
        flat += ops
        off.append(len(flat))
    assert tr["operand_off"].tolist() == off
    assert tr["operand_tensor"].tolist() == [t for t, _ in flat] and tr["operand_flags"].tolist() == [f for _, f in flat]
    assert tr["tensor_bytes"].tolist() == [t[0] for t in otr["tensors"]] and tr["tensor_kind"].tolist() == [t[1] for t in otr["tensors"]]
    assert tr["tau"].min() > 0 and tr["tau"].sum() < 10**9
    # a plan built from measured times runs and still matches the uncapped numerics
    ctx.tio_params_load(params)
    l0 = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(2)]
    lt.set_tau(tr["tau"])
    cap = int(peak * 0.5) // 256 * 256
    cp = tio.tio_build_plan(lt, ll, cap, 25 * 10**9, arena_bytes=up.export()["arena_needed"])
    ctx2 = tio.tio_ctx_create(cfg, up.export()["arena_needed"], cp.export()["host_needed"] + (1 << 20), 0)
    ctx2.tio_params_load(params)
    l1 = [ctx2.tio_train_step(tok, lab, cp)["loss"] for _ in range(2)]
    assert l0 == l1
    ctx.close(); ctx2.close()


def test_profile_of_an_iteration_that_does_not_fit_the_arena():
    """A context whose arena holds 55 % of the iteration's peak: the plain measured profile is refused, the
    offloaded profile runs the iteration under a plan of its own and returns positive times for every launch;
    the state it leaves is the state four plain steps leave (warm-up and three measured iterations)."""
    import paper_2506_06472_amd as tio
    cfg = CONFIGS["tiny_llama_fp32"]
    params, tok, lab = make_inputs(cfg, seed=0)
    lt, ll, up, cp, peak = plans_for(cfg, 0.55, 25 * 10**9, 0)
    ce, ue = cp.export(), up.export()
    hb = 2 * max(ue["host_needed"], ce["host_needed"]) + (1 << 20)
    ctx = tio.tio_ctx_create(cfg, ce["cap"], hb, 25 * 10**9)
    ctx.tio_params_load(params)
    with pytest.raises(tio.TioError) as ei:
        ctx.tio_profile_iteration(tok, lab, tio.PROFILE_MEASURED)
    assert ei.value.code == -7
    tr = ctx.tio_profile_iteration(tok, lab, tio.PROFILE_OFFLOADED).export()
    ref = lt.export()
    for key in ("op", "operand_off", "operand_tensor", "operand_flags", "tensor_bytes", "tensor_kind"):
        assert np.array_equal(tr[key], ref[key]), key
    assert tr["tau"].min() > 0 and tr["tau"].sum() < 10**9
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    s1 = read_state(ctx, names, False)
    ctx.close()
    ctx = _ctx(cfg, ue)
    ctx.tio_params_load(params)
    for _ in range(4):
        ctx.tio_train_step(tok, lab, None)
    s0 = read_state(ctx, names, False)
    ctx.close()
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key


def test_errors_are_reported_not_faulted():
    import paper_2506_06472_amd as tio
    cfg = CONFIGS["tiny_gpt_fp32"]
    params, tok, lab = make_inputs(cfg, seed=0)
    lt, ll, up, cp, peak = plans_for(cfg, 0.5)
    ctx = tio.tio_ctx_create(cfg, cp.export()["cap"], cp.export()["host_needed"] + (1 << 20), 0)
    ctx.tio_params_load(params)
    with pytest.raises(tio.TioError) as e:            # uncapped layout does not fit a capped arena
        ctx.tio_train_step(tok, lab, None)
    assert e.value.code == -7
    bad = tok.copy(); bad[0, 0] = cfg["V"]
    with pytest.raises(tio.TioError):
        ctx.tio_train_step(bad, lab, cp)
    other = tio.tio_trace_build(CONFIGS["tiny_llama_fp32"])
    ol = tio.tio_analyze_lifetimes(other)
    with pytest.raises(tio.TioError) as e:
        ctx.tio_train_step(tok, lab, tio.tio_build_plan(other, ol, 2**62, 0))
    assert e.value.code == -5
    assert ctx.tio_train_step(tok, lab, cp)["loss"] > 0
    ctx.close()


def test_slow_tier_in_device_memory_gives_the_same_bits():
    """The slow-tier pool may be a device buffer outside the arena (hosts that cannot pin enough memory)."""
    import paper_2506_06472_amd as tio
    cfg = SMALL_BF16
    params, tok, lab = make_inputs(cfg, seed=4)
    lt, ll, up, cp, peak = plans_for(cfg, 0.4, 25 * 10**9, 0)
    ce = cp.export()
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    out = []
    for on_dev, bw in ((False, 25 * 10**9), (True, 25 * 10**9), (True, 0)):
        ctx = tio.tio_ctx_create(cfg, ce["cap"], ce["host_needed"] + (1 << 20), bw, pool_on_device=on_dev)
        ctx.tio_params_load(params)
        losses = [ctx.tio_train_step(tok, lab, cp)["loss"] for _ in range(3)]
        out.append((losses, read_state(ctx, names, True)))
        ctx.close()
    for losses, state in out[1:]:
        assert losses == out[0][0]
        for key in state:
            assert state[key].tobytes() == out[0][1][key].tobytes(), key


@pytest.mark.parametrize("mode", ["plain", "paced", "two_tier", "file"])
def test_vacated_ranges_can_be_poisoned(mode, tmp_path):
    """poison_freed overwrites every arena range an offload has vacated with NaN patterns: a kernel that still
    read such a range would turn the loss into NaN.  The run stays bitwise equal to the uncapped one for every
    kind of slow tier, and the timeline statistics of a step add up."""
    import paper_2506_06472_amd as tio
    cfg = dict(arch="gpt", L=2, d=256, H=4, f=1024, V=1000, T=256, B=2, precision="bf16", lr=3e-4)
    params, tok, lab = make_inputs(cfg, seed=9)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    peak = int(ll.export()["M"].max())
    up = tio.tio_build_plan(lt, ll, 2**62, 0)
    two = mode == "two_tier"
    cp = tio.tio_build_plan(lt, ll, int(peak * 0.4) // 256 * 256, 4 * 10**9, host_bw=4 * 10**10 if two else 0,
                            host_budget=peak // 4 if two else 0)
    ue, ce = up.export(), cp.export()
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    ctx = tio.tio_ctx_create(cfg, ue["arena_needed"], ue["host_needed"] + (1 << 20), 0)
    ctx.tio_params_load(params)
    l0 = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(4)]
    s0 = read_state(ctx, names, True)
    ctx.close()
    kw = dict(poison_freed=True)
    if two:
        kw.update(host_tier_bytes=ce["host_tier_needed"] + 4096, host_tier_bw=4 * 10**10)
    if mode == "file":
        ctx = tio.tio_ctx_create(cfg, ce["cap"], 1 << 30, 0, slow_tier_file=str(tmp_path / "slow_tier.bin"),
                                 staging_bytes=2 << 20, file_chunk_bytes=128 << 10, **kw)
    else:
        ctx = tio.tio_ctx_create(cfg, ce["cap"], ce["host_needed"] + (1 << 20), 0 if mode == "plain" else 4 * 10**9, **kw)
    ctx.tio_params_load(params)
    l1 = [ctx.tio_train_step(tok, lab, cp)["loss"] for _ in range(3)]
    st = ctx.tio_train_step(tok, lab, cp, timeline=True)
    l1.append(st["loss"])
    s1 = read_state(ctx, names, True)
    ctx.close()
    assert np.isfinite(l1).all()
    assert np.array(l0, np.float32).tobytes() == np.array(l1, np.float32).tobytes(), (l0, l1)
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key
    # begin-to-end time of the step's transfers: positive, and at a paced tier at least bytes / bandwidth
    assert st["d2h_busy_ns"] > 0 and st["h2d_busy_ns"] > 0
    if mode == "paced":
        assert st["h2d_busy_ns"] >= 0.98 * ce["bytes_per_direction"] / 4e9 * 1e9


def test_bandwidth_can_change_between_steps_and_one_launch_can_be_timed():
    """tio_set_slow_tier_bw moves the slow tier between plain copies and its paced engine without touching the
    numbers; a lower bandwidth makes the capped step slower; tio_op_bench times one launch of the schedule."""
    import paper_2506_06472_amd as tio
    cfg = dict(arch="gpt", L=2, d=256, H=4, f=1024, V=1000, T=256, B=2, precision="bf16", lr=3e-4)
    params, tok, lab = make_inputs(cfg, seed=10)
    lt, ll, up, cp, peak = plans_for(cfg, 0.4, 2 * 10**9)
    ue, ce = up.export(), cp.export()
    ctx = _ctx(cfg, dict(arena_needed=ue["arena_needed"], host_needed=max(ue["host_needed"], ce["host_needed"])), bw=0)
    ctx.tio_params_load(params)
    l0 = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(6)]
    ctx.tio_params_load(params)
    l1, wall = [], []
    for bw in (0, 2 * 10**9, 2 * 10**9, 0, 10**9, 10**9):
        ctx.tio_set_slow_tier_bw(bw)
        st = ctx.tio_train_step(tok, lab, cp)
        l1.append(st["loss"])
        wall.append(st["wall_ns"])
    assert np.array(l0, np.float32).tobytes() == np.array(l1, np.float32).tobytes(), (l0, l1)
    # steady-state steps: half the bandwidth, about twice the transfer time
    floor = ce["bytes_per_direction"] / 2e9 * 1e9
    assert wall[2] >= 0.9 * floor and wall[5] >= 1.8 * floor and wall[3] < wall[2]
    ops = lt.export()["op"]
    k = int(np.nonzero(ops == 2)[0][0])                # first GEMM launch of the schedule
    ns = ctx.tio_op_bench(k, 5)
    assert 0 < ns < 1e8
    with pytest.raises(tio.TioError):
        ctx.tio_op_bench(len(ops), 1)
    ctx.close()
    small = _ctx(cfg, dict(arena_needed=ce["cap"], host_needed=ce["host_needed"]), bw=0)
    small.tio_params_load(params)
    with pytest.raises(tio.TioError) as ei:            # the uncapped layout does not fit this arena
        small.tio_op_bench(k, 1)
    assert ei.value.code == -7
    small.close()


@pytest.mark.parametrize("bw", [0, 2 * 10**9])
def test_one_copy_stream_shared_by_both_directions(bw):
    """d2h_stream == h2d_stream: offloads and prefetches form one queue (the planner's duplex = 0 channel).  The
    numbers stay those of the uncapped run, and at an emulated bandwidth a step takes at least the time of all its
    bytes, both directions, through the one channel."""
    import paper_2506_06472_amd as tio
    cfg = SMALL_BF16
    params, tok, lab = make_inputs(cfg, seed=11)
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    peak = int(ll.export()["M"].max())
    up = tio.tio_build_plan(lt, ll, 2**62, 0)
    cp = tio.tio_build_plan(lt, ll, int(peak * 0.4) // 256 * 256, bw or 2 * 10**9, duplex=False)
    ue, ce = up.export(), cp.export()
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    ctx = tio.tio_ctx_create(cfg, ue["arena_needed"], ue["host_needed"] + (1 << 20), 0)
    ctx.tio_params_load(params)
    l0 = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(4)]
    s0 = read_state(ctx, names, True)
    ctx.close()
    ctx = tio.tio_ctx_create(cfg, ce["cap"], ce["host_needed"] + (1 << 20), bw, single_copy_stream=True)
    ctx.tio_params_load(params)
    stats = [ctx.tio_train_step(tok, lab, cp) for _ in range(4)]
    s1 = read_state(ctx, names, True)
    ctx.close()
    l1 = [st["loss"] for st in stats]
    assert np.array(l0, np.float32).tobytes() == np.array(l1, np.float32).tobytes(), (l0, l1)
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key
    if bw:
        assert stats[-1]["wall_ns"] >= 0.95 * 2 * ce["bytes_per_direction"] / bw * 1e9


def test_kernel_times_of_the_full_model_from_one_measured_layer():
    """sweep.measure_layer_tau: every launch of the full trace gets the measured time of a one-layer launch with
    the same operator, flops and operand sizes; the result drives the planner and the performance model."""
    import io
    import paper_2506_06472_amd as tio
    from paper_2506_06472_amd import sweep as sw
    name = "tiny_llama_fp32"
    cfg = CONFIGS[name]
    tau = sw.measure_layer_tau(name, out=io.StringIO())
    lt = tio.tio_trace_build(cfg)
    assert len(tau) == lt.export()["n_kernels"] and (tau > 0).all()
    rows = sw.sweep(name, [10**9, 10**10], tau=tau, out=io.StringIO())
    assert rows[0][2] >= rows[1][2] >= int(tau.sum())


@pytest.mark.parametrize("cfg", [SMALL_BF16, SMALL_LLAMA_BF16, CONFIGS["tiny_gpt_fp32"], CONFIGS["tiny_llama_fp32"]],
                         ids=["gpt_bf16", "llama_bf16", "gpt_fp32", "llama_fp32"])
def test_optimizer_state_follows_the_oracle_from_the_gpu_gradients(cfg):
    """Three steps; after each one the oracle's AdamW (float64) is fed the gradients the GPU produced, so the two sides
    differ only by the optimizer arithmetic: master copy (bf16 recipe) or weights (fp32), first and second moment agree
    element by element to 1e-6 relative, and the bf16 weights are the master copy rounded to nearest even."""
    from synth import to_bf16_round
    params, tok, lab = make_inputs(cfg, seed=5)
    lt, ll, up, _, peak = plans_for(cfg)
    ctx = _ctx(cfg, up.export())
    ctx.tio_params_load(params)
    bf16 = cfg["precision"] == "bf16"
    names = [n for n, _, _ in ctx.params]
    th = {n: np.asarray(params[n], np.float64).reshape(-1) for n in names}
    m = {n: np.zeros_like(th[n]) for n in names}
    v = {n: np.zeros_like(th[n]) for n in names}
    gmax = {n: np.zeros_like(th[n]) for n in names}
    # the hyperparameters as the library receives them: single-precision fields of the model description
    f32 = lambda x: float(np.float32(x))
    hp = dict(lr=f32(cfg["lr"]), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), wd=f32(0.01))
    for step in range(3):
        print(f"optimizer state {cfg['arch']} {cfg['precision']} step {step}", flush=True)
        ctx.tio_train_step(tok, lab, None, capture_grads=True)
        for n in names:
            g = ctx.tio_grads_read(n).astype(np.float64).reshape(-1)
            gmax[n] = np.maximum(gmax[n], np.abs(g))
            th[n], m[n], v[n] = om.adamw_step(th[n], g, m[n], v[n], step + 1, **hp)
    worst = 0.0
    for n in names:
        got_th = ctx.tio_params_read(n, 1 if bf16 else 0).astype(np.float64).reshape(-1)
        got_m = ctx.tio_params_read(n, 2).astype(np.float64).reshape(-1)
        got_v = ctx.tio_params_read(n, 3).astype(np.float64).reshape(-1)
        # 1e-6 of what each element is made of: the parameter and its three updates of at most lr each; the moment and
        # the largest gradient term that went into it (terms of either sign cancel); the second moment itself (all its
        # terms are positive), with the smallest normal fp32 for squares that underflow
        for what, got, ref, scale in (("theta", got_th, th[n], np.abs(th[n]) + 3 * hp["lr"]),
                                      ("m", got_m, m[n], np.abs(m[n]) + 0.1 * gmax[n]),
                                      ("v", got_v, v[n], np.abs(v[n]))):
            err = np.abs(got - ref)
            bound = 1e-6 * scale + 1.2e-38
            assert np.all(err <= bound), (n, what, float((err / (scale + 1e-300)).max()))
            worst = max(worst, float((err / (scale + 1e-30)).max()))
        if bf16:
            w = ctx.tio_params_read(n, 0).astype(np.float32).reshape(-1)
            assert np.array_equal(w, to_bf16_round(ctx.tio_params_read(n, 1).astype(np.float32)).reshape(-1)), n
    print("largest relative deviation of the optimizer state", worst, flush=True)
    ctx.close()
