"""Seeded synthetic workloads.

The paper trains Llama3/Granite on C4; throughput and the tensor-access
structure depend on shapes only, so seeded inputs of the same shapes stand in:
weights N(0, 0.02^2), norm gains 1, biases 0, token ids uniform over the
vocabulary, next-token labels.  Nothing here implements any step of the method.
"""
from __future__ import annotations

import numpy as np

# name -> model/workload shape.  arch: "gpt" (LayerNorm, GELU, biases, learned
# positions) or "llama" (RMSNorm, RoPE, SwiGLU, no biases).
CONFIGS = {
    "tiny_gpt_fp32": dict(arch="gpt", L=2, d=128, H=4, f=512, V=1024, T=64, B=2,
                          precision="fp32", lr=1e-3, cap_frac=0.5),
    "gpt2_small_bf16": dict(arch="gpt", L=12, d=768, H=12, f=3072, V=50257, T=1024, B=8,
                            precision="bf16", lr=3e-4, cap_frac=0.4),
    "llama_7b_bf16": dict(arch="llama", L=32, d=4096, H=32, f=11008, V=32000, T=2048, B=4,
                          precision="bf16", lr=3e-4, cap_bytes=96 * 10**9),
    "llama_13b_bf16": dict(arch="llama", L=40, d=5120, H=40, f=13824, V=32000, T=2048, B=4,
                           precision="bf16", lr=3e-4, cap_bytes=128 * 10**9),
    "llama_30b_bf16": dict(arch="llama", L=60, d=6656, H=52, f=17920, V=32000, T=4096, B=2,
                           precision="bf16", lr=3e-4, cap_bytes=256 * 10**9,
                           slow_tier_bw=25 * 10**9),
    # small Llama-shaped case for parity tests (not one of the benchmark configs)
    "tiny_llama_fp32": dict(arch="llama", L=2, d=128, H=4, f=352, V=512, T=64, B=2,
                            precision="fp32", lr=1e-3, cap_frac=0.5),
}


def gen_params(specs, seed: int):
    """specs: iterable of (name, shape, init) with init in {"normal", "ones", "zeros"}.

    Returns {name: float32 array}.  One generator, drawn in the order given.
    """
    rng = np.random.default_rng(seed)
    out = {}
    for name, shape, init in specs:
        if init == "normal":
            out[name] = (rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02))
        elif init == "ones":
            out[name] = np.ones(shape, dtype=np.float32)
        elif init == "zeros":
            out[name] = np.zeros(shape, dtype=np.float32)
        else:
            raise ValueError(init)
    return out


def gen_tokens(B: int, T: int, V: int, seed: int):
    """Returns (inputs [B,T] int32, labels [B,T] int32): labels are the next token."""
    rng = np.random.default_rng(seed + 1_000_003)
    seq = rng.integers(0, V, size=(B, T + 1), dtype=np.int64)
    return seq[:, :T].astype(np.int32).copy(), seq[:, 1:].astype(np.int32).copy()


def to_bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returned as float32.

    Input conditioning only (both sides start from weights that are exactly
    representable in bf16 when the workload is bf16).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def iter_params_pooled(specs, seed: int, pool_elems: int = 1 << 27):
    """Yields (name, float32 array) one tensor at a time for very large models.

    Normal tensors are cut from one seeded pool of N(0, 0.02^2) values at a rotating offset (wrapping
    around), so a 30-billion-parameter model needs seconds, not minutes, of host time.  The values of
    different tensors are then not independent, which is irrelevant for what these workloads measure
    (throughput and tensor traffic depend on shapes only).
    """
    rng = np.random.default_rng(seed)
    pool = rng.standard_normal(pool_elems, dtype=np.float32) * np.float32(0.02)
    off = 0
    for name, shape, init in specs:
        n = int(np.prod(shape))
        if init == "ones":
            yield name, np.ones(shape, dtype=np.float32)
        elif init == "zeros":
            yield name, np.zeros(shape, dtype=np.float32)
        else:
            out = np.empty(n, dtype=np.float32)
            done = 0
            while done < n:
                take = min(n - done, pool_elems - off)
                out[done:done + take] = pool[off:off + take]
                done += take
                off = (off + take) % pool_elems
            off = (off + 7919) % pool_elems
            yield name, out.reshape(shape)
