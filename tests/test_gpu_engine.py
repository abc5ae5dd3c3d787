"""GPU: the paced engine's ready queue (chunked transfers, urgent first; Section 3.2 "Minimize kernel stalls").
Every service policy leaves losses and optimizer state bitwise equal to the uncapped run, and the measured step follows
the engine model."""
import time

import numpy as np
import pytest

from synth import CONFIGS
from gpulib import make_inputs, plans_for, read_state

pytestmark = pytest.mark.gpu

SMALL_BF16 = dict(arch="gpt", L=2, d=256, H=4, f=1024, V=1000, T=256, B=2, precision="bf16", lr=3e-4)


@pytest.mark.parametrize("cfg,cap_frac", [(CONFIGS["tiny_llama_fp32"], 0.45), (SMALL_BF16, 0.4)], ids=["llama_fp32", "gpt_bf16"])
def test_every_engine_policy_is_bitwise_neutral(cfg, cap_frac):
    import paper_2506_06472_amd as tio
    bw = 2 * 10**9
    params, tok, lab = make_inputs(cfg, seed=3)
    lt, ll, up, cp, peak = plans_for(cfg, cap_frac, bw)
    ce = cp.export()
    assert any(e[4] for e in ce["entries"]) and not all(e[4] for e in ce["entries"]), "want urgent and ordinary entries"
    names = [n for n, _, _ in tio.tio_param_list(cfg)]
    ctx = tio.tio_ctx_create(cfg, up.export()["arena_needed"], max(up.export()["host_needed"], ce["host_needed"]) + (1 << 20), bw)
    ctx.tio_params_load(params)
    ref_losses = [ctx.tio_train_step(tok, lab, None)["loss"] for _ in range(3)]
    ref_state = read_state(ctx, names, cfg["precision"] == "bf16")
    ctx.close()
    biggest = int(lt.export()["tensor_bytes"].max())
    for chunk, urgent_first, ready_queue in ((16 << 20, True, True), (4096, True, True), (biggest // 3 + 256, True, True),
                                            (0, True, True), (4096, False, True), (0, False, False), (65536, True, False)):
        print(f"policy chunk={chunk} urgent_first={urgent_first} ready_queue={ready_queue}", flush=True)
        ctx = tio.tio_ctx_create(cfg, ce["cap"], max(up.export()["host_needed"], ce["host_needed"]) + (1 << 20), bw, poison_freed=True)
        ctx.tio_set_engine_policy(chunk, urgent_first, ready_queue)
        ctx.tio_params_load(params)
        losses = []
        for step in range(3):
            st = ctx.tio_train_step(tok, lab, cp)
            losses.append(st["loss"])
            assert st["h2d_bytes"] == ce["bytes_per_direction"]
        state = read_state(ctx, names, cfg["precision"] == "bf16")
        ctx.close()
        assert np.array(losses, np.float32).tobytes() == np.array(ref_losses, np.float32).tobytes(), (losses, ref_losses)
        for key in ref_state:
            assert state[key].tobytes() == ref_state[key].tobytes(), key


def test_measured_step_follows_the_engine_model():
    """GPT-2-small-shaped workload, four layers, 40 % cap, slow tier paced to 25 GB/s: the measured step is within a few
    per cent of tio_plan_simulate_engine fed with the measured kernel times, for the default policy and for first come
    first served."""
    import torch
    import paper_2506_06472_amd as tio
    cfg = dict(CONFIGS["gpt2_small_bf16"], L=4)
    bw = 25 * 10**9
    params, tok, lab = make_inputs(cfg, seed=0)
    lt, ll, up, _, peak = plans_for(cfg)
    ue = up.export()
    ctx = tio.tio_ctx_create(cfg, ue["arena_needed"], ue["host_needed"] + (1 << 20), 0)
    ctx.tio_params_load(params)
    tau = ctx.tio_profile_iteration(tok, lab).export()["tau"]
    ctx.close()
    lt.set_tau(tau)
    cap = int(peak * 0.4) // 256 * 256
    cp = tio.tio_build_plan(lt, ll, cap, bw, min_bytes=1 << 20)
    ce = cp.export()
    ctx = tio.tio_ctx_create(cfg, ce["cap"], ce["host_needed"] + (1 << 20), bw)
    ctx.tio_params_load(params)
    for chunk, urgent_first, ready_queue in ((16 << 20, True, True), (0, False, False)):
        ctx.tio_set_engine_policy(chunk, urgent_first, ready_queue)
        for _ in range(2):
            ctx.tio_train_step(tok, lab, cp)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = 5
        for _ in range(n):
            ctx.tio_train_step(tok, lab, cp)
        torch.cuda.synchronize()
        measured = (time.perf_counter() - t0) / n * 1e9
        if ready_queue:
            model = tio.tio_plan_simulate_engine(lt, cp, bw, chunk_bytes=chunk, urgent_first=urgent_first)[0]
        else:
            model = tio.tio_plan_simulate(lt, cp, bw)[0]
        print(f"policy chunk={chunk} urgent_first={urgent_first} ready_queue={ready_queue}: measured {measured / 1e6:.2f} ms, "
              f"model {model / 1e6:.2f} ms", flush=True)
        assert abs(measured - model) <= 0.06 * model, (measured, model)
    ctx.close()
