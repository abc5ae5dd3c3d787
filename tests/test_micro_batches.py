"""Micro-batches with gradient accumulation (Sections 4.1 and 4.2 of the paper train with micro-batches).

Oracle pins: the micro-batched loss and gradients equal the whole-batch ones (the loss is a mean over tokens,
so the result does not depend on how the batch is cut); the trace has the closed-form kernel and tensor
counts, its gradient tensors live from the first micro-batch's backward pass to their AdamW launch, and a
single micro-batch reproduces the plain trace.  Library: trace, lifetimes and plan bit-exact against the
oracle."""
import numpy as np
import pytest

import paper_2506_06472_amd as tio
from oracle import model as om
from oracle import plan as op
from oracle import trace as ot
from synth import CONFIGS, gen_params, gen_tokens
from test_plan_parity import assert_same_plan

TINY = [dict(CONFIGS["tiny_gpt_fp32"], B=4), dict(CONFIGS["tiny_llama_fp32"], B=4)]


@pytest.mark.parametrize("cfg", TINY, ids=["gpt", "llama"])
@pytest.mark.parametrize("n", [2, 4])
def test_oracle_accumulated_gradient_equals_whole_batch_gradient(cfg, n):
    params = gen_params(om.param_specs(cfg), 3)
    tok, lab = gen_tokens(cfg["B"], cfg["T"], cfg["V"], 3)
    l1, g1 = om.forward_backward(cfg, params, tok, lab)
    ln, gn = om.forward_backward(dict(cfg, micro_batches=n), params, tok, lab)
    assert abs(l1 - ln) <= 1e-12 * abs(l1)
    for k in g1:
        scale = np.abs(g1[k]).max()
        assert np.abs(g1[k] - gn[k]).max() <= 1e-11 * max(scale, 1e-30), k


def test_oracle_unequal_group_losses_average_to_the_batch_loss():
    """Two groups with very different losses: the batch loss is their plain average (equal token counts)."""
    cfg = dict(CONFIGS["tiny_gpt_fp32"], B=2)
    params = gen_params(om.param_specs(cfg), 5)
    tok, lab = gen_tokens(2, cfg["T"], cfg["V"], 5)
    la, _ = om.forward_backward(cfg, params, tok[:1], lab[:1], want_grads=False)
    lb, _ = om.forward_backward(cfg, params, tok[1:], lab[1:], want_grads=False)
    l2, _ = om.forward_backward(dict(cfg, micro_batches=2), params, tok, lab, want_grads=False)
    assert abs(l2 - 0.5 * (la + lb)) <= 1e-12


@pytest.mark.parametrize("cfg", TINY + [dict(CONFIGS["gpt2_small_bf16"], L=2)], ids=["gpt", "llama", "gpt_bf16"])
def test_trace_structure(cfg):
    one = ot.build_trace(cfg)
    assert ot.build_trace(dict(cfg, micro_batches=1)) == one
    n = 2
    tr = ot.build_trace(dict(cfg, micro_batches=n))
    half = ot.build_trace(dict(cfg, B=cfg["B"] // n))
    n_adamw = sum(1 for k in half["kernels"] if k[0] == ot.ADAMW)
    # every launch of the half-size schedule twice, the AdamW launches once
    assert len(tr["kernels"]) == n * len(half["kernels"]) - (n - 1) * n_adamw
    # tensors: persistent ones once, one more token and label buffer, the transients twice except the
    # parameter gradients and the loss
    npers = half["n_persistent"]
    n_pgrad = sum(1 for t in half["tensors"] if t[1] == ot.K_PGRAD)
    assert tr["n_persistent"] == npers + 2 * (n - 1)
    assert len(tr["tensors"]) == npers + 2 * (n - 1) + n * (len(half["tensors"]) - npers) - (n - 1) * (n_pgrad + 1)
    # the second micro-batch's launches are the first one's on tensors of the same sizes
    first = [k for k in half["kernels"] if k[0] != ot.ADAMW]
    second = [k for k in tr["kernels"][len(first):] if k[0] != ot.ADAMW]
    # (operands are listed by tensor id, and the shared loss scalar has a smaller id than the second
    # micro-batch's transients: compare the operand sizes as multisets)
    assert [(k[0], k[2], sorted(half["tensors"][t][0] for t, _ in k[1])) for k in first] == \
           [(k[0], k[2], sorted(tr["tensors"][t][0] for t, _ in k[1])) for k in second]
    # a gradient tensor: written first in micro-batch 0, read and written in micro-batch 1, read by its AdamW
    life = op.analyze_lifetimes(tr)
    g = tr["ids"]["g.w_head"]
    uses = [(i, fl) for i, k in enumerate(tr["kernels"]) for t, fl in k[1] if t == g]
    assert [fl for _, fl in uses] == [ot.WRITE, ot.READ | ot.WRITE, ot.READ]
    assert tr["kernels"][uses[-1][0]][0] == ot.ADAMW and uses[0][0] < len(first) <= uses[1][0]
    # it is inactive (and can be offloaded) between the micro-batches
    assert any(t == g and s == uses[0][0] and e == uses[1][0] for t, _, s, e in life["periods"])


@pytest.mark.parametrize("cfg", [dict(CONFIGS["tiny_gpt_fp32"], B=4, micro_batches=2),
                                 dict(CONFIGS["tiny_llama_fp32"], B=4, micro_batches=4),
                                 dict(CONFIGS["gpt2_small_bf16"], L=3, micro_batches=2)], ids=["gpt2", "llama4", "gpt_bf16"])
def test_library_trace_lifetimes_and_plan_bit_exact(cfg):
    tr = ot.build_trace(cfg)
    lt = tio.tio_trace_build(cfg)
    v = lt.export()
    assert (v["n_kernels"], v["n_tensors"], v["n_persistent"]) == (len(tr["kernels"]), len(tr["tensors"]), tr["n_persistent"])
    assert v["op"].tolist() == [k[0] for k in tr["kernels"]]
    assert v["flops"].tolist() == [k[2] for k in tr["kernels"]]
    assert v["tau"].tolist() == tr["tau"]
    assert v["tensor_bytes"].tolist() == [t[0] for t in tr["tensors"]]
    assert v["tensor_kind"].tolist() == [t[1] for t in tr["tensors"]]
    flat = [o for _, ops, _ in tr["kernels"] for o in ops]
    assert v["operand_tensor"].tolist() == [t for t, _ in flat]
    assert v["operand_flags"].tolist() == [f for _, f in flat]
    life = op.analyze_lifetimes(tr)
    ll = tio.tio_analyze_lifetimes(lt)
    lv = ll.export()
    assert lv["M"].tolist() == life["M"]
    assert sorted(zip(lv["tensor"].tolist(), lv["bytes"].tolist(), lv["start"].tolist(), lv["end"].tolist())) == sorted(life["periods"])
    peak = max(life["M"])
    for frac in (0.5, 0.7):
        assert_same_plan(tr, lt, ll, int(peak * frac) // 256 * 256, 25 * 10**9)


def test_batch_must_divide():
    with pytest.raises(tio.TioError):
        tio.tio_trace_build(dict(CONFIGS["tiny_gpt_fp32"], B=3, micro_batches=2))
