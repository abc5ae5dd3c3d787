"""Pins for oracle/model.py: things fixed by mathematics or by a library routine,
not by the oracle itself."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import model as om
from synth import CONFIGS, gen_params, gen_tokens

TINY = {
    "gpt": dict(arch="gpt", L=2, d=16, H=2, f=24, V=29, T=5, B=2, lr=1e-3),
    "llama": dict(arch="llama", L=2, d=16, H=2, f=20, V=29, T=5, B=2, lr=1e-3),
}


def _setup(cfg, seed=0, scale=10.0):
    p = gen_params(om.param_specs(cfg), seed)
    rng = np.random.default_rng(seed + 7)
    # move away from the symmetric init so that every term of the gradient is exercised
    p = {k: (v * scale + 0.1 * rng.standard_normal(v.shape)).astype(np.float64) for k, v in p.items()}
    tok, lab = gen_tokens(cfg["B"], cfg["T"], cfg["V"], seed)
    return p, tok, lab


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_end_to_end_gradient_matches_central_differences(arch):
    cfg = TINY[arch]
    p, tok, lab = _setup(cfg)
    loss, G = om.forward_backward(cfg, p, tok, lab)
    rng = np.random.default_rng(1)
    h = 1e-6
    for name, w in p.items():
        flat = w.reshape(-1)
        idx = rng.choice(flat.size, size=min(6, flat.size), replace=False)
        if name == "wte":  # rows that are actually looked up
            idx = np.array([int(t) * cfg["d"] + j for t, j in zip(tok.reshape(-1)[:4], range(4))])
        for i in idx:
            old = flat[i]
            flat[i] = old + h
            lp, _ = om.forward_backward(cfg, p, tok, lab, want_grads=False)
            flat[i] = old - h
            lm, _ = om.forward_backward(cfg, p, tok, lab, want_grads=False)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            an = G[name].reshape(-1)[i]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 2e-9, (name, i, fd, an)


def _fd_op(fwd, bwd, x, rng, h=1e-6, n=10):
    """Checks sum(fwd(x) * r) against bwd(r) by central differences."""
    y = fwd(x)
    r = rng.standard_normal(y.shape)
    dx = bwd(r)
    flat = x.reshape(-1)
    for i in rng.choice(flat.size, size=min(n, flat.size), replace=False):
        old = flat[i]
        flat[i] = old + h
        fp = (fwd(x) * r).sum()
        flat[i] = old - h
        fm = (fwd(x) * r).sum()
        flat[i] = old
        fd = (fp - fm) / (2 * h)
        assert abs(fd - dx.reshape(-1)[i]) <= 1e-6 * max(1.0, abs(fd)), (i, fd, dx.reshape(-1)[i])


def test_operator_gradients_by_central_differences():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 12))
    g = rng.standard_normal(12)
    b = rng.standard_normal(12)
    _fd_op(lambda a: om.layernorm_fwd(a, g, b, 1e-5)[0],
           lambda r: om.layernorm_bwd(r, g, om.layernorm_fwd(x, g, b, 1e-5)[1])[0], x, rng)
    _fd_op(lambda a: om.rmsnorm_fwd(a, g, 1e-5)[0],
           lambda r: om.rmsnorm_bwd(r, g, om.rmsnorm_fwd(x, g, 1e-5)[1])[0], x, rng)
    _fd_op(om.gelu_fwd, lambda r: om.gelu_bwd(r, x), x, rng)
    _fd_op(om.swiglu_fwd, lambda r: om.swiglu_bwd(r, x), x, rng)
    q, k, v = (rng.standard_normal((2, 3, 6, 4)) for _ in range(3))
    _fd_op(lambda a: om.attention_fwd(a, k, v)[0],
           lambda r: om.attention_bwd(r, q, k, v, om.attention_fwd(q, k, v)[1])[0], q, rng)
    _fd_op(lambda a: om.attention_fwd(q, a, v)[0],
           lambda r: om.attention_bwd(r, q, k, v, om.attention_fwd(q, k, v)[1])[1], k, rng)
    _fd_op(lambda a: om.attention_fwd(q, k, a)[0],
           lambda r: om.attention_bwd(r, q, k, v, om.attention_fwd(q, k, v)[1])[2], v, rng)
    # norm parameter gradients
    gg = g.copy()
    _fd_op(lambda a: om.layernorm_fwd(x, a, b, 1e-5)[0],
           lambda r: om.layernorm_bwd(r, gg, om.layernorm_fwd(x, gg, b, 1e-5)[1])[1], gg, rng)
    _fd_op(lambda a: om.rmsnorm_fwd(x, a, 1e-5)[0],
           lambda r: om.rmsnorm_bwd(r, gg, om.rmsnorm_fwd(x, gg, 1e-5)[1])[1], gg, rng)


# ---------------------------------------------------------------- library cross-check
def _torch_loss(cfg, P, tok, lab):
    a, L, d, H = cfg["arch"], cfg["L"], cfg["d"], cfg["H"]
    B, T = tok.shape
    dh = d // H
    t = torch.from_numpy(tok.astype(np.int64))
    x = P["wte"][t]
    if a == "gpt":
        x = x + P["wpe"][:T][None]
    else:
        inv = 10000.0 ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
        ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None]
        rot = torch.polar(torch.ones_like(ang), ang)          # complex rotation

        def rope(z):  # [B,T,H,dh]
            zc = torch.view_as_complex(z.reshape(B, T, H, dh // 2, 2).contiguous())
            return torch.view_as_real(zc * rot[None, :, None, :]).reshape(B, T, H, dh)
    for i in range(L):
        p = f"l{i}."
        if a == "gpt":
            h = F.layer_norm(x, (d,), P[p + "ln1_g"], P[p + "ln1_b"], 1e-5)
            qkv = F.linear(h, P[p + "w_qkv"], P[p + "b_qkv"])
        else:
            h = F.rms_norm(x, (d,), P[p + "rms1_g"], 1e-5)
            qkv = F.linear(h, P[p + "w_qkv"])
        q, k, v = (z.reshape(B, T, H, dh) for z in qkv.split(d, dim=-1))
        if a == "llama":
            q, k = rope(q), rope(k)
        o = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2), is_causal=True)
        o = o.transpose(1, 2).reshape(B, T, d)
        x = x + F.linear(o, P[p + "w_o"], P[p + "b_o"] if a == "gpt" else None)
        if a == "gpt":
            h = F.layer_norm(x, (d,), P[p + "ln2_g"], P[p + "ln2_b"], 1e-5)
            x = x + F.linear(F.gelu(F.linear(h, P[p + "w_fc1"], P[p + "b_fc1"]), approximate="tanh"),
                             P[p + "w_fc2"], P[p + "b_fc2"])
        else:
            h = F.rms_norm(x, (d,), P[p + "rms2_g"], 1e-5)
            g, u = F.linear(h, P[p + "w_gu"]).chunk(2, dim=-1)
            x = x + F.linear(F.silu(g) * u, P[p + "w_down"])
    if a == "gpt":
        x = F.layer_norm(x, (d,), P["lnf_g"], P["lnf_b"], 1e-5)
    else:
        x = F.rms_norm(x, (d,), P["rmsf_g"], 1e-5)
    logits = F.linear(x, P["w_head"])
    return F.cross_entropy(logits.reshape(B * T, -1), torch.from_numpy(lab.astype(np.int64)).reshape(-1))


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_against_torch_autograd_and_adamw(arch):
    cfg = dict(TINY[arch], T=9, B=3)
    p, tok, lab = _setup(cfg, seed=3)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    opt = torch.optim.AdamW(list(P.values()), lr=cfg["lr"], betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    tr = om.Trainer(cfg, p)
    for step in range(3):
        opt.zero_grad()
        tl = _torch_loss(cfg, P, tok, lab)
        tl.backward()
        loss = tr.step(tok, lab)
        assert abs(loss - tl.item()) <= 1e-12 * abs(tl.item())
        for k in p:
            g_ref = P[k].grad.numpy()
            assert np.abs(tr.last_grads[k] - g_ref).max() <= 1e-11 * max(1e-30, np.abs(g_ref).max()), (step, k)
        grads = {k: P[k].grad.numpy().copy() for k in p}
        opt.step()
        for k in p:
            # where |g| is at rounding level (e.g. the key bias, whose true gradient is 0)
            # m/(sqrt(v)+eps) is ill-conditioned: those entries get the bound 2*lr per step
            well = np.abs(grads[k]) > 1e-9
            err = np.abs(tr.p[k] - P[k].detach().numpy())
            assert (err[well].max() if well.any() else 0.0) <= 1e-12, (step, k)
            assert err.max() <= 2 * cfg["lr"] * (step + 1), (step, k)


# ---------------------------------------------------------------- closed forms and invariants
def test_loss_at_init_is_log_vocab():
    for name in ("tiny_gpt_fp32", "tiny_llama_fp32"):
        cfg = CONFIGS[name]
        p = gen_params(om.param_specs(cfg), 0)
        tok, lab = gen_tokens(cfg["B"], cfg["T"], cfg["V"], 0)
        loss, _ = om.forward_backward(cfg, p, tok, lab, want_grads=False)
        assert abs(loss - math.log(cfg["V"])) < 1e-2 * math.log(cfg["V"])


def test_attention_single_position_is_identity_on_v_and_rows_sum_to_one():
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal((2, 3, 1, 4)) for _ in range(3))
    o, p = om.attention_fwd(q, k, v)
    assert np.array_equal(o, v)
    q, k, v = (rng.standard_normal((2, 3, 6, 4)) for _ in range(3))
    o, p = om.attention_fwd(q, k, v)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(p[0, 0], 1) == 0.0)
    # first row attends only to position 0
    assert np.allclose(o[:, :, 0], v[:, :, 0])
    # uniform scores -> running mean of v
    o2, _ = om.attention_fwd(np.zeros_like(q), k, v)
    assert np.allclose(o2[0, 0, 3], v[0, 0, :4].mean(0))


def test_causality_of_logits():
    cfg = TINY["gpt"]
    p, tok, lab = _setup(cfg)
    _, _, lg = om.forward_backward(cfg, p, tok, lab, want_grads=False, return_logits=True)
    tok2 = tok.copy()
    tok2[:, 3] = (tok2[:, 3] + 1) % cfg["V"]
    _, _, lg2 = om.forward_backward(cfg, p, tok2, lab, want_grads=False, return_logits=True)
    T = cfg["T"]
    lg, lg2 = lg.reshape(cfg["B"], T, -1), lg2.reshape(cfg["B"], T, -1)
    assert np.array_equal(lg[:, :3], lg2[:, :3])
    assert not np.array_equal(lg[:, 3:], lg2[:, 3:])


def test_rope_is_a_rotation():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 3, 7, 8))
    cos, sin = om.rope_tables(7, 8, 10000.0, np.float64)
    y = om.rope_apply(x, cos, sin)
    assert np.array_equal(y[:, :, 0], x[:, :, 0])                      # position 0: identity
    n0 = (x.reshape(2, 3, 7, 4, 2) ** 2).sum(-1)
    n1 = (y.reshape(2, 3, 7, 4, 2) ** 2).sum(-1)
    assert np.allclose(n0, n1, rtol=1e-13)                              # each pair keeps its norm
    assert np.allclose(om.rope_apply(y, cos, sin, inverse=True), x, atol=1e-14)
    # pair 0 at position 1 rotates by exactly 1 radian; the last pair by theta^(-(dh-2)/dh)
    v = np.zeros((1, 1, 2, 8)); v[0, 0, 1, 0] = 1.0; v[0, 0, 1, 6] = 1.0
    r = om.rope_apply(v, *om.rope_tables(2, 8, 10000.0, np.float64))
    assert np.allclose(r[0, 0, 1, :2], [math.cos(1.0), math.sin(1.0)])
    a = 10000.0 ** (-6.0 / 8.0)
    assert np.allclose(r[0, 0, 1, 6:], [math.cos(a), math.sin(a)])
    # relative-position property: <rope(q)_i, rope(k)_j> depends on i-j only
    q = rng.standard_normal(8); k = rng.standard_normal(8)
    Q = np.tile(q, (1, 1, 7, 1)); K = np.tile(k, (1, 1, 7, 1))
    Qr, Kr = om.rope_apply(Q, cos, sin), om.rope_apply(K, cos, sin)
    assert np.isclose(Qr[0, 0, 5] @ Kr[0, 0, 3], Qr[0, 0, 4] @ Kr[0, 0, 2])


def test_layernorm_statistics_and_rmsnorm_scale():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64)) * 3 + 2
    y, _ = om.layernorm_fwd(x, np.ones(64), np.zeros(64), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-13) and np.allclose(y.var(-1), 1, atol=1e-12)
    y, _ = om.rmsnorm_fwd(x, np.ones(64), 0.0)
    assert np.allclose((y * y).mean(-1), 1, atol=1e-12)


def test_gelu_values():
    # tanh form at a few points, written from the definition with math.tanh
    for x in (-3.0, -1.0, 0.0, 0.5, 2.0):
        ref = 0.5 * x * (1 + math.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))
        assert om.gelu_fwd(np.array([x]))[0] == pytest.approx(ref, rel=1e-15, abs=1e-300)
    assert om.gelu_fwd(np.array([10.0]))[0] == pytest.approx(10.0, rel=1e-12)
    assert abs(om.gelu_fwd(np.array([-10.0]))[0]) < 1e-12


def test_cross_entropy_uniform_and_peaked():
    S, V = 4, 10
    loss, dl = om.cross_entropy(np.zeros((S, V)), np.arange(S))
    assert loss == pytest.approx(math.log(V))
    assert np.allclose(dl.sum(-1), 0)
    assert dl[0, 0] == pytest.approx((1 / V - 1) / S) and dl[0, 1] == pytest.approx(1 / V / S)
    lg = np.zeros((1, 3)); lg[0, 2] = 1000.0
    assert om.cross_entropy(lg, np.array([2]))[0] == pytest.approx(0.0, abs=1e-12)
    assert om.cross_entropy(lg, np.array([0]))[0] == pytest.approx(1000.0)


def test_adamw_first_step_closed_form():
    g = np.array([0.5, -2.0, 1e-3]); th = np.array([1.0, -1.0, 0.3])
    lr, wd, eps = 1e-3, 0.01, 1e-8
    t1, m1, v1 = om.adamw_step(th, g, np.zeros(3), np.zeros(3), 1, lr)
    # at t=1 the bias-corrected moments are g and g^2
    assert np.allclose(t1, th - lr * (g / (np.abs(g) + eps) + wd * th), rtol=1e-14)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)
    # zero gradient: pure decay
    t2, _, _ = om.adamw_step(th, np.zeros(3), np.zeros(3), np.zeros(3), 1, lr)
    assert np.allclose(t2, th * (1 - lr * wd))


def test_param_counts_match_published_model_sizes():
    n = lambda c: sum(int(np.prod(s)) for _, s, _ in om.param_specs(CONFIGS[c]))
    assert n("tiny_gpt_fp32") == 667_136
    assert n("gpt2_small_bf16") == 163_037_184
    assert n("llama_7b_bf16") == 6_738_415_616       # Llama-7B has 6.74e9 parameters
    assert n("llama_13b_bf16") == 13_015_864_320
    assert n("llama_30b_bf16") == 32_528_943_616
