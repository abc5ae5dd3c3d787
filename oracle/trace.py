"""CPU oracle for the tensor access trace of one training iteration.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

The paper's profiler (Section 3.1) marks every input and output tensor of a GPU
operator active while the operator runs and records tensor sizes and kernel
times.  In this build the operators are the library's own kernel launches, so
the trace is a function of the model shape alone: this file writes that
function out from the canonical kernel schedule (one record per launch, in
launch order), independently of the library's launcher.

A trace is
  tensors: list of (bytes, kind, name); bytes = payload rounded up to 256
  kernels: list of (op, operands, flops); operands = sorted list of
           (tensor id, flags), flags bit0 = read, bit1 = written
  tau:     modelled kernel times in ns (a deterministic stand-in for measured
           times: max(flops/F, bytes/W) + c with integer constants)

Tensor ids: persistent tensors first (parameter-list order; per parameter the
compute weight, then the fp32 master copy when the precision is bf16, then the
two AdamW moments), then the token and label buffers, then transient tensors
in order of first write.

Micro-batches (cfg["micro_batches"] = n > 1; the paper splits each batch into
micro-batches, Section 4.1 and 4.2): the batch is cut into n groups of B/n
sequences; the forward and backward schedule runs once per group on tensors of
that group's size (one token and one label buffer per group, all listed after
the persistent tensors); parameter gradients and the scalar loss are written by
the first group and accumulated in place by the later ones; the AdamW launches
follow the gradient-completing launches of the last group only.

Pins (tests/test_oracle_plan.py): the complete launch list of a one-layer GPT-shaped
and a one-layer Llama-shaped model, with the names of the tensors every launch reads,
writes and updates, against lists written by hand from the dataflow
(tests/golden/trace_*_one_layer.txt), and the repetition of that pattern in a second
layer; kernel and tensor counts in closed form, persistent bytes = 12 or 14 bytes per
parameter, every transient written before read, peak memory at the loss kernel in
closed form.  The schedule itself is a reading of this build (the paper names no
kernels); the contraction-splitting rule of the weight-gradient products (dw_splits)
and the norm-backward row count are launch parameters of the library restated here:
their values are pinned only by the library's trace being equal to this one.
"""
from __future__ import annotations

from .model import param_specs

# op codes (shared numbering is part of the written specification, not shared code)
(EMBED_FWD, NORM_FWD, GEMM, ROPE_FWD, ATTN_FWD, GELU_FWD, SWIGLU_FWD, CE_FWD_BWD, LOSS_REDUCE,
 GEMM_DX, GEMM_DW, BIAS_GRAD, GELU_BWD, SWIGLU_BWD, NORM_BWD, NORM_BWD_PARAMS, ATTN_BWD_PRE,
 ATTN_BWD, ROPE_BWD, EMBED_BWD, POSEMB_BWD, ADAMW) = range(22)

# tensor kinds
K_WEIGHT, K_MASTER, K_M, K_V, K_INPUT, K_ACT, K_GRAD, K_PGRAD = range(8)

READ, WRITE = 1, 2
NORM_BWD_ROWS = 8           # rows of the token dimension handled by one norm-backward workgroup

# modelled kernel time constants
MODEL_FLOPS_PER_S = 1_250_000_000_000_000     # half of the dense bf16 MFMA peak
MODEL_BYTES_PER_S = 4_000_000_000_000         # half of the HBM peak
MODEL_LAUNCH_NS = 4_000


def _r256(n):
    return (n + 255) // 256 * 256


def dw_splits(M, N, K):
    """Contraction ranges of a bf16 weight-gradient GEMM dW[M,N] over K tokens: doubled (at most 8, at least
    256 tokens per range) while fewer than about 512 workgroups of 128x128 output tiles would exist."""
    tiles = ((M + 127) // 128) * ((N + 127) // 128)
    s = 1
    while s < 8 and tiles * s * 2 <= 512 and K // (s * 2) >= 256:
        s *= 2
    return s


def vocab_ld(V):
    """Leading dimension of the logits matrix: vocabulary rounded up to 64 columns."""
    return (V + 63) // 64 * 64


class _Builder:
    def __init__(self):
        self.tensors, self.kernels, self.ids = [], [], {}

    def tensor(self, name, nbytes, kind):
        assert name not in self.ids, name
        self.ids[name] = len(self.tensors)
        self.tensors.append((_r256(nbytes), kind, name))
        return self.ids[name]

    def kernel(self, op, reads=(), writes=(), inouts=(), flops=0):
        fl = {}
        for n in reads:
            fl[self.ids[n]] = fl.get(self.ids[n], 0) | READ
        for n in writes:
            fl[self.ids[n]] = fl.get(self.ids[n], 0) | WRITE
        for n in inouts:
            fl[self.ids[n]] = fl.get(self.ids[n], 0) | READ | WRITE
        self.kernels.append((op, sorted(fl.items()), int(flops)))


def build_trace(cfg):
    a, L, d, H, f, V, T, B = (cfg[k] for k in ("arch", "L", "d", "H", "f", "V", "T", "B"))
    n_mb = int(cfg.get("micro_batches", 1) or 1)
    assert n_mb >= 1 and B % n_mb == 0, "batch must divide into the micro-batches"
    B //= n_mb                           # from here on: sequences and tokens of one micro-batch
    gpt = a == "gpt"
    bf16 = cfg["precision"] == "bf16"
    e = 2 if bf16 else 4                 # element size of weights, activations, gradients
    S = B * T
    Vp = vocab_ld(V)
    b = _Builder()
    specs = param_specs(cfg)

    # ---- persistent tensors
    for name, shape, _ in specs:
        n = 1
        for s in shape:
            n *= s
        b.tensor(name, n * e, K_WEIGHT)
        if bf16:
            b.tensor(name + ".master", n * 4, K_MASTER)
        b.tensor(name + ".m", n * 4, K_M)
        b.tensor(name + ".v", n * 4, K_V)
    for j in range(n_mb):
        pre = "" if n_mb == 1 else f"mb{j}."
        b.tensor(pre + "tokens", S * 4, K_INPUT)
        b.tensor(pre + "labels", S * 4, K_INPUT)
    n_persistent = len(b.tensors)
    for j in range(n_mb):
        _micro_batch(b, cfg, j, n_mb, B, S, Vp, e, specs)

    tau = []
    for op, operands, flops in b.kernels:
        nbytes = sum(b.tensors[t][0] for t, _ in operands)
        tf = -(-flops * 10**9 // MODEL_FLOPS_PER_S)
        tb = -(-nbytes * 10**9 // MODEL_BYTES_PER_S)
        tau.append(max(tf, tb) + MODEL_LAUNCH_NS)
    return dict(tensors=b.tensors, kernels=b.kernels, tau=tau, ids=b.ids, n_persistent=n_persistent)


def _micro_batch(b, cfg, j, n_mb, B, S, Vp, e, specs):
    """Appends the forward and backward launches of micro-batch j (B sequences, S tokens)."""
    a, L, d, H, f, V, T = (cfg[k] for k in ("arch", "L", "d", "H", "f", "V", "T"))
    gpt = a == "gpt"
    bf16 = cfg["precision"] == "bf16"
    first, last = j == 0, j == n_mb - 1
    pre = "" if n_mb == 1 else f"mb{j}."          # transient tensors of this micro-batch
    shared = set()
    for name, _, _ in specs:
        shared.update((name, name + ".master", name + ".m", name + ".v"))
    # names of persistent tensors, gradients and the loss are shared by all micro-batches
    q = lambda n: n if (n in shared or n.startswith("g.") or n == "loss") else pre + n

    class _Scoped:
        ids = b.ids
        tensors = b.tensors

        @staticmethod
        def tensor(name, nbytes, kind):
            return b.tensor(q(name), nbytes, kind)

        @staticmethod
        def kernel(op, reads=(), writes=(), inouts=(), flops=0):
            b.kernel(op, [q(n) for n in reads], [q(n) for n in writes], [q(n) for n in inouts], flops)

    _schedule(_Scoped, cfg, first, last, B, S, Vp, e)


def _schedule(b, cfg, first, last, B, S, Vp, e):
    a, L, d, H, f, V, T = (cfg[k] for k in ("arch", "L", "d", "H", "f", "V", "T"))
    gpt = a == "gpt"
    bf16 = cfg["precision"] == "bf16"

    act = lambda name, n, es=e: b.tensor(name, n * es, K_ACT)
    grd = lambda name, n, es=e: b.tensor(name, n * es, K_GRAD)
    nb = (S + NORM_BWD_ROWS - 1) // NORM_BWD_ROWS
    nstat = 2 if gpt else 1              # LayerNorm keeps mean and rstd, RMSNorm rstd
    norm_p = (lambda p, k: [p + k + "_g", p + k + "_b"]) if gpt else (lambda p, k: [p + k + "_g"])
    nk = "ln" if gpt else "rms"
    attn_flops = 2 * B * H * T * T * (d // H)       # two T x T x dh products, causal half

    # ---- forward
    act("x0", S * d)
    b.kernel(EMBED_FWD, reads=["tokens", "wte"] + (["wpe"] if gpt else []), writes=["x0"])
    x = "x0"
    for i in range(L):
        p = f"l{i}."
        act(p + "h1", S * d); act(p + "st1", S * nstat, 4)
        b.kernel(NORM_FWD, reads=[x] + norm_p(p, nk + "1"), writes=[p + "h1", p + "st1"])
        act(p + "qkv", S * 3 * d)
        b.kernel(GEMM, reads=[p + "h1", p + "w_qkv"] + ([p + "b_qkv"] if gpt else []),
                 writes=[p + "qkv"], flops=2 * S * 3 * d * d)
        if not gpt:
            b.kernel(ROPE_FWD, inouts=[p + "qkv"])
        act(p + "ao", S * d); act(p + "lse", B * H * T, 4)
        b.kernel(ATTN_FWD, reads=[p + "qkv"], writes=[p + "ao", p + "lse"], flops=attn_flops)
        act(p + "xm", S * d)
        b.kernel(GEMM, reads=[p + "ao", p + "w_o", x] + ([p + "b_o"] if gpt else []),
                 writes=[p + "xm"], flops=2 * S * d * d)
        act(p + "h2", S * d); act(p + "st2", S * nstat, 4)
        b.kernel(NORM_FWD, reads=[p + "xm"] + norm_p(p, nk + "2"), writes=[p + "h2", p + "st2"])
        if gpt:
            act(p + "u", S * f)
            b.kernel(GEMM, reads=[p + "h2", p + "w_fc1", p + "b_fc1"], writes=[p + "u"], flops=2 * S * f * d)
            act(p + "act", S * f)
            b.kernel(GELU_FWD, reads=[p + "u"], writes=[p + "act"])
            w2, b2 = p + "w_fc2", [p + "b_fc2"]
        else:
            act(p + "u", S * 2 * f)
            b.kernel(GEMM, reads=[p + "h2", p + "w_gu"], writes=[p + "u"], flops=2 * S * 2 * f * d)
            act(p + "act", S * f)
            b.kernel(SWIGLU_FWD, reads=[p + "u"], writes=[p + "act"])
            w2, b2 = p + "w_down", []
        act(p + "xo", S * d)
        b.kernel(GEMM, reads=[p + "act", w2, p + "xm"] + b2, writes=[p + "xo"], flops=2 * S * d * f)
        x = p + "xo"
    fin = "lnf" if gpt else "rmsf"
    fin_p = [fin + "_g"] + ([fin + "_b"] if gpt else [])
    act("hf", S * d); act("stf", S * nstat, 4)
    b.kernel(NORM_FWD, reads=[x] + fin_p, writes=["hf", "stf"])
    act("logits", S * Vp)
    b.kernel(GEMM, reads=["hf", "w_head"], writes=["logits"], flops=2 * S * V * d)
    act("losses", S, 4)
    b.kernel(CE_FWD_BWD, reads=["labels"], inouts=["logits"], writes=["losses"])
    if first:
        act("loss", 1, 4)
        b.kernel(LOSS_REDUCE, reads=["losses"], writes=["loss"])
    else:                                # adds this micro-batch's share to the running loss
        b.kernel(LOSS_REDUCE, reads=["losses"], inouts=["loss"])

    # ---- backward
    def pgrad(name):
        # gradient tensor of a parameter: created by the first micro-batch, accumulated into by the others
        if first:
            b.tensor("g." + name, b.tensors[b.ids[name]][0], K_PGRAD)

    def gout(names):
        """operand lists of a launch that produces parameter gradients: (writes, inouts)"""
        return (names, []) if first else ([], names)

    def adamw(name):
        # the update of a parameter follows the launch that completes its gradient (no later kernel of the
        # iteration reads the parameter), so gradients die at once and optimizer traffic overlaps the backward pass
        if not last:
            return
        state = [name] + ([name + ".master"] if bf16 else []) + [name + ".m", name + ".v"]
        b.kernel(ADAMW, reads=["g." + name], inouts=state)

    def norm_bwd(dy, xin, st, pnames, dres, dx, part):
        grd(dx, S * d); grd(part, nb * len(pnames) * d, 4)
        b.kernel(NORM_BWD, reads=[dy, xin, st, pnames[0]] + ([dres] if dres else []), writes=[dx, part])
        for n in pnames:
            pgrad(n)
        gw, gio = gout(["g." + n for n in pnames])
        b.kernel(NORM_BWD_PARAMS, reads=[part], writes=gw, inouts=gio)
        for n in pnames:
            adamw(n)

    def gemm_dw(dy, xin, w, bias, n_out, n_in):
        pgrad(w)
        if bias:
            pgrad(bias)
        ws = []
        splits = dw_splits(n_out, n_in, S) if bf16 else 1
        if splits > 1:                                   # fp32 partial tiles and partial row sums
            grd("ws." + w, splits * (n_out * n_in + n_out), 4)
            ws = ["ws." + w]
        gw, gio = gout(["g." + w] + (["g." + bias] if bias else []))
        b.kernel(GEMM_DW, reads=[dy, xin], writes=gw, inouts=ws + gio, flops=2 * S * n_in * n_out)
        adamw(w)
        if bias:
            adamw(bias)

    grd("dhf", S * d)
    b.kernel(GEMM_DX, reads=["logits", "w_head"], writes=["dhf"], flops=2 * S * V * d)
    gemm_dw("logits", "hf", "w_head", None, V, d)
    norm_bwd("dhf", x, "stf", fin_p, None, "dxf", "partf")
    dx = "dxf"
    for i in reversed(range(L)):
        p = f"l{i}."
        xin = f"l{i - 1}.xo" if i > 0 else "x0"
        w2 = p + ("w_fc2" if gpt else "w_down")
        w1 = p + ("w_fc1" if gpt else "w_gu")
        f1 = f if gpt else 2 * f
        grd(p + "dact", S * f)
        b.kernel(GEMM_DX, reads=[dx, w2], writes=[p + "dact"], flops=2 * S * d * f)
        gemm_dw(dx, p + "act", w2, p + "b_fc2" if gpt else None, d, f)
        if gpt:
            b.kernel(GELU_BWD, reads=[p + "u"], inouts=[p + "dact"])
            du = p + "dact"
        else:
            grd(p + "du", S * 2 * f)
            b.kernel(SWIGLU_BWD, reads=[p + "dact", p + "u"], writes=[p + "du"])
            du = p + "du"
        grd(p + "dh2", S * d)
        b.kernel(GEMM_DX, reads=[du, w1], writes=[p + "dh2"], flops=2 * S * f1 * d)
        gemm_dw(du, p + "h2", w1, p + "b_fc1" if gpt else None, f1, d)
        norm_bwd(p + "dh2", p + "xm", p + "st2", norm_p(p, nk + "2"), dx, p + "dxm", p + "part2")
        grd(p + "dao", S * d)
        b.kernel(GEMM_DX, reads=[p + "dxm", p + "w_o"], writes=[p + "dao"], flops=2 * S * d * d)
        gemm_dw(p + "dxm", p + "ao", p + "w_o", p + "b_o" if gpt else None, d, d)
        grd(p + "delta", B * H * T, 4)
        b.kernel(ATTN_BWD_PRE, reads=[p + "dao", p + "ao"], writes=[p + "delta"])
        grd(p + "dqkv", S * 3 * d)
        b.kernel(ATTN_BWD, reads=[p + "dao", p + "qkv", p + "lse", p + "delta"], writes=[p + "dqkv"],
                 flops=attn_flops * 5 // 2)
        if not gpt:
            b.kernel(ROPE_BWD, inouts=[p + "dqkv"])
        grd(p + "dh1", S * d)
        b.kernel(GEMM_DX, reads=[p + "dqkv", p + "w_qkv"], writes=[p + "dh1"], flops=2 * S * 3 * d * d)
        gemm_dw(p + "dqkv", p + "h1", p + "w_qkv", p + "b_qkv" if gpt else None, 3 * d, d)
        norm_bwd(p + "dh1", xin, p + "st1", norm_p(p, nk + "1"), p + "dxm", p + "dx", p + "part1")
        dx = p + "dx"
    pgrad("wte")
    gw, gio = gout(["g.wte"])
    b.kernel(EMBED_BWD, reads=[dx, "tokens"], writes=gw, inouts=gio)
    adamw("wte")
    if gpt:
        pgrad("wpe")
        gw, gio = gout(["g.wpe"])
        b.kernel(POSEMB_BWD, reads=[dx], writes=gw, inouts=gio)
        adamw("wpe")
