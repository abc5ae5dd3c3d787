"""GPU: plans with a host-memory tier beside the slow tier run through the C ABI and leave every bit of the
training state as the uncapped run produces it; both tiers carry traffic; a context without the second pool
refuses such a plan."""
import numpy as np
import pytest

from synth import CONFIGS
from gpulib import make_inputs, read_state

pytestmark = pytest.mark.gpu

BF16 = dict(arch="gpt", L=2, d=256, H=4, f=1024, V=1000, T=256, B=2, precision="bf16", lr=3e-4)


def _plans(cfg, frac, bw, hbw, bfrac, min_bytes=0):
    import paper_2506_06472_amd as tio
    lt = tio.tio_trace_build(cfg)
    ll = tio.tio_analyze_lifetimes(lt)
    peak = int(ll.export()["M"].max())
    up = tio.tio_build_plan(lt, ll, 2**62, 0)
    cp = tio.tio_build_plan(lt, ll, int(peak * frac) // 256 * 256, bw, min_bytes=min_bytes, host_bw=hbw,
                            host_budget=int(peak * bfrac))
    return lt, ll, up, cp, peak


@pytest.mark.parametrize("cfg,frac,bw,hbw,bfrac,pace", [
    (CONFIGS["tiny_gpt_fp32"], 0.5, 2 * 10**9, 2 * 10**10, 0.3, True),
    (CONFIGS["tiny_llama_fp32"], 0.45, 10**9, 8 * 10**9, 1.0, False),
    (BF16, 0.4, 4 * 10**9, 4 * 10**10, 0.25, True),
], ids=["gpt_fp32", "llama_fp32", "gpt_bf16"])
def test_two_tier_plan_is_bitwise_neutral(cfg, frac, bw, hbw, bfrac, pace):
    import paper_2506_06472_amd as tio
    params, tok, lab = make_inputs(cfg, seed=3)
    lt, ll, up, cp, peak = _plans(cfg, frac, bw, hbw, bfrac)
    ue, ce = up.export(), cp.export()
    n1 = sum(ce["tier"])
    print(f"pairs {len(ce['tier'])} on the host tier {n1} host pool {ce['host_tier_needed']} peak {ce['host_peak']}", flush=True)
    assert 0 < n1 < len(ce["tier"]) and ce["host_peak"] <= int(peak * bfrac)
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    bf = cfg["precision"] == "bf16"
    hb = max(ue["host_needed"], ce["host_needed"]) + (1 << 20)
    ctx = tio.tio_ctx_create(cfg, ue["arena_needed"], hb, 0)
    ctx.tio_params_load(params)
    l0 = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(4)]
    s0 = read_state(ctx, names, bf)
    ctx.close()
    ctx = tio.tio_ctx_create(cfg, ce["cap"], hb, bw if pace else 0, host_tier_bytes=ce["host_tier_needed"] + 4096,
                             host_tier_bw=hbw if pace else 0)
    ctx.tio_params_load(params)
    l1 = []
    for step in range(4):
        st = ctx.tio_train_step(tok, lab, cp)
        l1.append(st["loss"])
        assert st["h2d_bytes"] == ce["bytes_per_direction"]
    s1 = read_state(ctx, names, bf)        # some tensors are read back from their host-tier slots
    ctx.close()
    assert np.array(l0, np.float32).tobytes() == np.array(l1, np.float32).tobytes(), (l0, l1)
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key


def test_switching_between_single_and_two_tier_plans_keeps_the_bits():
    import paper_2506_06472_amd as tio
    cfg = BF16
    params, tok, lab = make_inputs(cfg, seed=5)
    lt, ll, up, cp2, peak = _plans(cfg, 0.4, 4 * 10**9, 4 * 10**10, 0.25)
    cp1 = tio.tio_build_plan(lt, ll, int(peak * 0.5) // 256 * 256, 4 * 10**9)
    ue, e1, e2 = up.export(), cp1.export(), cp2.export()
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    hb = max(ue["host_needed"], e1["host_needed"], e2["host_needed"]) + (1 << 20)
    ctx = tio.tio_ctx_create(cfg, ue["arena_needed"], hb, 0)
    ctx.tio_params_load(params)
    l0 = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(6)]
    s0 = read_state(ctx, names, True)
    ctx.close()
    ctx = tio.tio_ctx_create(cfg, ue["arena_needed"], hb, 0, host_tier_bytes=e2["host_tier_needed"] + 4096)
    ctx.tio_params_load(params)
    l1 = [ctx.tio_train_step(tok, lab, pl)["loss"] for pl in (cp2, cp2, cp1, cp2, None, cp2)]
    s1 = read_state(ctx, names, True)
    ctx.close()
    assert np.array(l0, np.float32).tobytes() == np.array(l1, np.float32).tobytes(), (l0, l1)
    for key in s0:
        assert s0[key].tobytes() == s1[key].tobytes(), key


def test_two_tier_plan_needs_the_second_pool():
    import paper_2506_06472_amd as tio
    cfg = CONFIGS["tiny_gpt_fp32"]
    params, tok, lab = make_inputs(cfg, seed=0)
    lt, ll, up, cp, peak = _plans(cfg, 0.5, 2 * 10**9, 2 * 10**10, 0.3)
    ce = cp.export()
    ctx = tio.tio_ctx_create(cfg, ce["cap"], ce["host_needed"] + (1 << 20), 0)
    ctx.tio_params_load(params)
    with pytest.raises(tio.TioError) as ei:
        ctx.tio_train_step(tok, lab, cp)
    assert ei.value.code == -2
    ctx.close()
