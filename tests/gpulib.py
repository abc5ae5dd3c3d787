"""Helpers for the GPU parity tests (marshalling only)."""
import numpy as np

import paper_2506_06472_amd as tio
from oracle import model as om
from synth import gen_params, gen_tokens, to_bf16_round


def make_inputs(cfg, seed=0):
    params = gen_params(om.param_specs(cfg), seed)
    if cfg["precision"] == "bf16":
        params = {k: to_bf16_round(v) for k, v in params.items()}
    tok, lab = gen_tokens(cfg["B"], cfg["T"], cfg["V"], seed)
    return params, tok, lab


def plans_for(cfg, cap_frac=None, bw=25 * 10**9, min_bytes=0, tau=None, retime_passes=0):
    """(trace, lifetimes, uncapped plan, capped plan or None)"""
    lt = tio.tio_trace_build(cfg)
    if tau is not None:
        lt.set_tau(tau)
    ll = tio.tio_analyze_lifetimes(lt)
    peak = int(ll.export()["M"].max())
    up = tio.tio_build_plan(lt, ll, 2**62, 0)
    cp = None
    if cap_frac is not None:
        cap = int(peak * cap_frac) // 256 * 256
        cp = tio.tio_build_plan(lt, ll, cap, bw, min_bytes=min_bytes, retime_passes=retime_passes)
    return lt, ll, up, cp, peak


def read_state(ctx, names, bf16):
    out = {}
    for n in names:
        for which in ((0, 1, 2, 3) if bf16 else (0, 2, 3)):
            out[(n, which)] = ctx.tio_params_read(n, which)
    return out
