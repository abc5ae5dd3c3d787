"""CPU oracle for the model arithmetic of one training iteration.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference against which
the HIP path is checked; only tests, the smoke check and the benchmark's
cpu_baseline leg may import it.  It shares no code with the HIP library.

The paper (Section 4.1) trains decoder-only transformers with stock framework
operators and gives no arithmetic of its own, so each function below is the
textbook definition of the operator written out with numpy, in float64 unless
another dtype is asked for.  Forward, exact backward (analytic gradient of the
mean next-token cross-entropy) and the AdamW update.

Pins (tests/test_oracle_model.py): central finite differences in float64 for
every operator and end to end; torch CPU autograd of the same network built
from library operators; loss at initialisation ~ ln V; single-position
attention is the identity on V; causality; RoPE is a rotation (norm
preserving, identity at position 0); LayerNorm output has mean 0 and variance
1; AdamW first step in closed form and against torch.optim.AdamW.
Parity with the paper's own numerics is unpinned: the paper prints no losses.
"""
from __future__ import annotations

import math

import numpy as np

GELU_C = math.sqrt(2.0 / math.pi)
GELU_A = 0.044715


# ----------------------------------------------------------------------------
# parameter list (order is part of the trace specification)
# ----------------------------------------------------------------------------
def param_specs(cfg):
    """[(name, shape, init)] in parameter-list order."""
    a, L, d, f, V, T = cfg["arch"], cfg["L"], cfg["d"], cfg["f"], cfg["V"], cfg["T"]
    out = [("wte", (V, d), "normal")]
    if a == "gpt":
        out.append(("wpe", (T, d), "normal"))
    for i in range(L):
        p = f"l{i}."
        if a == "gpt":
            out += [(p + "ln1_g", (d,), "ones"), (p + "ln1_b", (d,), "zeros"),
                    (p + "w_qkv", (3 * d, d), "normal"), (p + "b_qkv", (3 * d,), "zeros"),
                    (p + "w_o", (d, d), "normal"), (p + "b_o", (d,), "zeros"),
                    (p + "ln2_g", (d,), "ones"), (p + "ln2_b", (d,), "zeros"),
                    (p + "w_fc1", (f, d), "normal"), (p + "b_fc1", (f,), "zeros"),
                    (p + "w_fc2", (d, f), "normal"), (p + "b_fc2", (d,), "zeros")]
        else:
            out += [(p + "rms1_g", (d,), "ones"), (p + "w_qkv", (3 * d, d), "normal"),
                    (p + "w_o", (d, d), "normal"), (p + "rms2_g", (d,), "ones"),
                    (p + "w_gu", (2 * f, d), "normal"), (p + "w_down", (d, f), "normal")]
    if a == "gpt":
        out += [("lnf_g", (d,), "ones"), ("lnf_b", (d,), "zeros")]
    else:
        out += [("rmsf_g", (d,), "ones")]
    out.append(("w_head", (V, d), "normal"))
    return out


# ----------------------------------------------------------------------------
# operators: forward and backward
# ----------------------------------------------------------------------------
def layernorm_fwd(x, g, b, eps):
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)          # biased variance
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * rstd
    return xh * g + b, (xh, rstd)


def layernorm_bwd(dy, g, cache):
    xh, rstd = cache
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(-1, keepdims=True) - xh * (dxh * xh).mean(-1, keepdims=True))
    return dx, (dy * xh).sum(0), dy.sum(0)


def rmsnorm_fwd(x, g, eps):
    rstd = 1.0 / np.sqrt((x * x).mean(-1, keepdims=True) + eps)
    xh = x * rstd
    return xh * g, (xh, rstd)


def rmsnorm_bwd(dy, g, cache):
    xh, rstd = cache
    dxh = dy * g
    dx = rstd * (dxh - xh * (dxh * xh).mean(-1, keepdims=True))
    return dx, (dy * xh).sum(0)


def gelu_fwd(x):
    """tanh form: 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    u = GELU_C * (x + GELU_A * x ** 3)
    return 0.5 * x * (1.0 + np.tanh(u))


def gelu_bwd(dy, x):
    u = GELU_C * (x + GELU_A * x ** 3)
    t = np.tanh(u)
    return dy * (0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * GELU_C * (1.0 + 3.0 * GELU_A * x * x))


def swiglu_fwd(gu):
    """gu [...,2f]: gate = first f columns, up = last f; silu(gate) * up."""
    f = gu.shape[-1] // 2
    g, u = gu[..., :f], gu[..., f:]
    return g / (1.0 + np.exp(-g)) * u


def swiglu_bwd(dy, gu):
    f = gu.shape[-1] // 2
    g, u = gu[..., :f], gu[..., f:]
    s = 1.0 / (1.0 + np.exp(-g))
    dg = dy * u * (s + g * s * (1.0 - s))
    du = dy * g * s
    return np.concatenate([dg, du], axis=-1)


def rope_tables(T, dh, theta, dtype):
    i = np.arange(dh // 2, dtype=np.float64)
    inv = theta ** (-2.0 * i / dh)
    ang = np.arange(T, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def rope_apply(x, cos, sin, inverse=False):
    """x [B,H,T,dh]; rotates adjacent pairs (2i, 2i+1) by pos * theta^(-2i/dh)."""
    x0, x1 = x[..., 0::2], x[..., 1::2]
    s = -sin if inverse else sin
    y = np.empty_like(x)
    y[..., 0::2] = x0 * cos - x1 * s
    y[..., 1::2] = x0 * s + x1 * cos
    return y


def attention_fwd(q, k, v):
    """q,k,v [B,H,T,dh]; causal softmax(q k^T / sqrt(dh)) v."""
    T, dh = q.shape[-2], q.shape[-1]
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / math.sqrt(dh)
    mask = np.triu(np.ones((T, T), dtype=bool), 1)
    s = np.where(mask, -np.inf, s)
    s = s - s.max(-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(-1, keepdims=True)
    return np.matmul(p, v), p


def attention_bwd(do, q, k, v, p):
    dh = q.shape[-1]
    dv = np.matmul(np.swapaxes(p, -1, -2), do)
    dp = np.matmul(do, np.swapaxes(v, -1, -2))
    ds = p * (dp - (dp * p).sum(-1, keepdims=True))
    dq = np.matmul(ds, k) / math.sqrt(dh)
    dk = np.matmul(np.swapaxes(ds, -1, -2), q) / math.sqrt(dh)
    return dq, dk, dv


def cross_entropy(logits, labels):
    """mean over rows of -log softmax(logits)[label]; returns loss, dlogits."""
    S = logits.shape[0]
    z = logits - logits.max(-1, keepdims=True)
    e = np.exp(z)
    se = e.sum(-1, keepdims=True)
    logp = z - np.log(se)
    loss = -logp[np.arange(S), labels].mean()
    dl = e / se
    dl[np.arange(S), labels] -= 1.0
    return loss, dl / S


# ----------------------------------------------------------------------------
# network
# ----------------------------------------------------------------------------
def _heads(x, B, T, H):          # [S, d] -> [B,H,T,dh]
    return x.reshape(B, T, H, -1).transpose(0, 2, 1, 3)


def _unheads(x):                 # [B,H,T,dh] -> [S, d]
    B, H, T, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * T, H * dh)


def forward_backward(cfg, params, tokens, labels, dtype=np.float64, want_grads=True,
                     return_logits=False):
    """One forward (and backward) pass.  params: {name: array}; tokens/labels [B,T] int.

    Returns (loss, grads) with grads {name: array} in `dtype`.  With cfg["micro_batches"] = n > 1 the batch
    is cut into n groups of B/n sequences that are run one after the other; the loss is the mean over all
    tokens, so every group contributes its mean loss and mean gradient weighted by its share of the tokens,
    and the gradients are added up group by group (gradient accumulation; Section 4.1 of the paper trains
    with micro-batches).
    """
    n_mb = int(cfg.get("micro_batches", 1) or 1)
    if n_mb == 1:
        return _forward_backward_batch(cfg, params, tokens, labels, dtype, want_grads, return_logits)
    assert not return_logits
    B = tokens.shape[0]
    assert B % n_mb == 0
    g = B // n_mb
    loss, grads = dtype(0.0), None
    for j in range(n_mb):
        lj, gj = _forward_backward_batch(cfg, params, tokens[j * g:(j + 1) * g], labels[j * g:(j + 1) * g], dtype,
                                         want_grads, False)
        share = dtype(1.0) / dtype(n_mb)
        loss = loss + lj * share
        if want_grads:
            if grads is None:
                grads = {k: v * share for k, v in gj.items()}
            else:
                for k, v in gj.items():
                    grads[k] = grads[k] + v * share
    return loss, grads


def _forward_backward_batch(cfg, params, tokens, labels, dtype, want_grads, return_logits):
    a, L, d, H, V = cfg["arch"], cfg["L"], cfg["d"], cfg["H"], cfg["V"]
    eps = cfg.get("eps", 1e-5)
    B, T = tokens.shape
    S = B * T
    dh = d // H
    P = {k: np.asarray(v, dtype=dtype) for k, v in params.items()}
    tok = tokens.reshape(-1).astype(np.int64)
    lab = labels.reshape(-1).astype(np.int64)
    gpt = a == "gpt"
    if not gpt:
        cos, sin = rope_tables(T, dh, cfg.get("rope_theta", 10000.0), dtype)

    x = P["wte"][tok]
    if gpt:
        x = x + np.tile(P["wpe"][:T], (B, 1))
    C = []
    for i in range(L):
        p = f"l{i}."
        c = {"x": x}
        if gpt:
            h, c["n1"] = layernorm_fwd(x, P[p + "ln1_g"], P[p + "ln1_b"], eps)
            qkv = h @ P[p + "w_qkv"].T + P[p + "b_qkv"]
        else:
            h, c["n1"] = rmsnorm_fwd(x, P[p + "rms1_g"], eps)
            qkv = h @ P[p + "w_qkv"].T
        c["h1"] = h
        q, k, v = (_heads(qkv[:, j * d:(j + 1) * d], B, T, H) for j in range(3))
        if not gpt:
            q, k = rope_apply(q, cos, sin), rope_apply(k, cos, sin)
        o, pr = attention_fwd(q, k, v)
        c.update(q=q, k=k, v=v, p=pr)
        ao = _unheads(o)
        c["ao"] = ao
        x = x + ao @ P[p + "w_o"].T + (P[p + "b_o"] if gpt else 0.0)
        c["xm"] = x
        if gpt:
            h, c["n2"] = layernorm_fwd(x, P[p + "ln2_g"], P[p + "ln2_b"], eps)
            u = h @ P[p + "w_fc1"].T + P[p + "b_fc1"]
            act = gelu_fwd(u)
            x = x + act @ P[p + "w_fc2"].T + P[p + "b_fc2"]
        else:
            h, c["n2"] = rmsnorm_fwd(x, P[p + "rms2_g"], eps)
            u = h @ P[p + "w_gu"].T
            act = swiglu_fwd(u)
            x = x + act @ P[p + "w_down"].T
        c.update(h2=h, u=u, act=act)
        C.append(c)
    if gpt:
        hf, nf = layernorm_fwd(x, P["lnf_g"], P["lnf_b"], eps)
    else:
        hf, nf = rmsnorm_fwd(x, P["rmsf_g"], eps)
    logits = hf @ P["w_head"].T
    loss, dlogits = cross_entropy(logits, lab)
    if not want_grads:
        return (float(loss), None, logits) if return_logits else (float(loss), None)

    G = {}
    G["w_head"] = dlogits.T @ hf
    dhf = dlogits @ P["w_head"]
    if gpt:
        dx, G["lnf_g"], G["lnf_b"] = layernorm_bwd(dhf, P["lnf_g"], nf)
    else:
        dx, G["rmsf_g"] = rmsnorm_bwd(dhf, P["rmsf_g"], nf)
    for i in reversed(range(L)):
        p = f"l{i}."
        c = C[i]
        if gpt:
            G[p + "w_fc2"] = dx.T @ c["act"]
            G[p + "b_fc2"] = dx.sum(0)
            du = gelu_bwd(dx @ P[p + "w_fc2"], c["u"])
            G[p + "w_fc1"] = du.T @ c["h2"]
            G[p + "b_fc1"] = du.sum(0)
            dn, G[p + "ln2_g"], G[p + "ln2_b"] = layernorm_bwd(du @ P[p + "w_fc1"], P[p + "ln2_g"], c["n2"])
        else:
            G[p + "w_down"] = dx.T @ c["act"]
            du = swiglu_bwd(dx @ P[p + "w_down"], c["u"])
            G[p + "w_gu"] = du.T @ c["h2"]
            dn, G[p + "rms2_g"] = rmsnorm_bwd(du @ P[p + "w_gu"], P[p + "rms2_g"], c["n2"])
        dx = dx + dn                                   # gradient at x_mid
        G[p + "w_o"] = dx.T @ c["ao"]
        if gpt:
            G[p + "b_o"] = dx.sum(0)
        do = _heads(dx @ P[p + "w_o"], B, T, H)
        dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], c["p"])
        if not gpt:
            dq, dk = rope_apply(dq, cos, sin, inverse=True), rope_apply(dk, cos, sin, inverse=True)
        dqkv = np.concatenate([_unheads(dq), _unheads(dk), _unheads(dv)], axis=1)
        G[p + "w_qkv"] = dqkv.T @ c["h1"]
        if gpt:
            G[p + "b_qkv"] = dqkv.sum(0)
            dn, G[p + "ln1_g"], G[p + "ln1_b"] = layernorm_bwd(dqkv @ P[p + "w_qkv"], P[p + "ln1_g"], c["n1"])
        else:
            dn, G[p + "rms1_g"] = rmsnorm_bwd(dqkv @ P[p + "w_qkv"], P[p + "rms1_g"], c["n1"])
        dx = dx + dn
        c.clear()
    gw = np.zeros_like(P["wte"])
    np.add.at(gw, tok, dx)
    G["wte"] = gw
    if gpt:
        G["wpe"] = np.zeros_like(P["wpe"])
        G["wpe"][:T] = dx.reshape(B, T, d).sum(0)
    if return_logits:
        return float(loss), G, logits
    return float(loss), G


# ----------------------------------------------------------------------------
# optimizer
# ----------------------------------------------------------------------------
def adamw_step(theta, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01):
    """Decoupled-weight-decay Adam, step index t starting at 1.

    m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
    theta <- theta - lr ( m/(1-b1^t) / (sqrt(v/(1-b2^t)) + eps) + wd theta ).
    Returns new (theta, m, v).
    """
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mh = m / (1.0 - beta1 ** t)
    vh = v / (1.0 - beta2 ** t)
    theta = theta - lr * (mh / (np.sqrt(vh) + eps) + wd * theta)
    return theta, m, v


class Trainer:
    """Holds parameters and AdamW state; step() = forward, backward, update."""

    def __init__(self, cfg, params, dtype=np.float64):
        self.cfg, self.dtype = cfg, dtype
        self.p = {k: np.asarray(v, dtype=dtype).copy() for k, v in params.items()}
        self.m = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.v = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.t = 0
        self.last_grads = None

    def step(self, tokens, labels):
        loss, G = forward_backward(self.cfg, self.p, tokens, labels, dtype=self.dtype)
        self.t += 1
        lr = self.cfg.get("lr", 1e-3)
        for k in self.p:
            self.p[k], self.m[k], self.v[k] = adamw_step(self.p[k], G[k], self.m[k], self.v[k], self.t, lr)
        self.last_grads = G
        return loss
