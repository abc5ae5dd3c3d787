// Builds the canonical kernel schedule of one iteration (forward, backward, AdamW) for the
// GPT-shaped and Llama-shaped decoders.  One KernelRec per HIP launch, in launch order; tensor
// ids: persistent tensors first (parameter-list order; weight, [master], m, v), then the token and
// label buffers, then transient tensors in order of first write.
//
// Micro-batches (cfg.micro_batches = n > 1; Sections 4.1 and 4.2 of the paper train with micro-batches):
// the batch is cut into n groups of batch/n sequences; the forward and backward schedule runs once per
// group on tensors of that group's size (one token and one label buffer per group); parameter gradients
// and the scalar loss are written by the first group and accumulated in place by the later ones; the
// AdamW launches follow the gradient-completing launches of the last group only.
#include "program.h"

#include <stdexcept>

namespace tio {

namespace {

struct Builder {
    Program P;
    int64_t e;  // element size of weights / activations / gradients

    int tensor(const std::string &name, int64_t payload, int kind) {
        TensorInfo t;
        t.bytes = (uint64_t)((payload + 255) / 256 * 256);
        t.kind = kind;
        t.name = name;
        P.tensors.push_back(t);
        return (int)P.tensors.size() - 1;
    }
    int act(const std::string &n, int64_t numel) { return tensor(n, numel * e, KIND_ACT); }
    int act32(const std::string &n, int64_t numel) { return tensor(n, numel * 4, KIND_ACT); }
    int grd(const std::string &n, int64_t numel) { return tensor(n, numel * e, KIND_GRAD); }
    int grd32(const std::string &n, int64_t numel) { return tensor(n, numel * 4, KIND_GRAD); }

    KernelRec &kernel(int op) {
        KernelRec k;
        k.op = op;
        for (int i = 0; i < kMaxRoles; ++i) { k.t[i] = -1; k.fl[i] = 0; }
        for (auto &x : k.p) x = 0;
        k.flops = 0;
        P.kernels.push_back(k);
        return P.kernels.back();
    }
};

void set(KernelRec &k, int role, int tensor, int flags) { k.t[role] = tensor; k.fl[role] = (uint8_t)flags; }
constexpr int R = 1, W = 2, RW = 3;

}  // namespace

std::vector<ParamInfo> list_params(const tio_model_cfg &c) {
    std::vector<ParamInfo> out;
    auto add = [&](const std::string &n, int64_t r, int64_t cc, int init) {
        ParamInfo p;
        p.name = n; p.rows = r; p.cols = cc; p.w = p.master = p.m = p.v = p.grad = -1; p.init = init;
        out.push_back(p);
    };
    const int64_t d = c.d_model, f = c.d_ff, V = c.vocab, T = c.seq_len;
    const bool gpt = c.arch == TIO_ARCH_GPT;
    add("wte", V, d, 0);
    if (gpt) add("wpe", T, d, 0);
    for (int i = 0; i < c.n_layers; ++i) {
        std::string p = "l" + std::to_string(i) + ".";
        if (gpt) {
            add(p + "ln1_g", 1, d, 1); add(p + "ln1_b", 1, d, 2);
            add(p + "w_qkv", 3 * d, d, 0); add(p + "b_qkv", 1, 3 * d, 2);
            add(p + "w_o", d, d, 0); add(p + "b_o", 1, d, 2);
            add(p + "ln2_g", 1, d, 1); add(p + "ln2_b", 1, d, 2);
            add(p + "w_fc1", f, d, 0); add(p + "b_fc1", 1, f, 2);
            add(p + "w_fc2", d, f, 0); add(p + "b_fc2", 1, d, 2);
        } else {
            add(p + "rms1_g", 1, d, 1);
            add(p + "w_qkv", 3 * d, d, 0);
            add(p + "w_o", d, d, 0);
            add(p + "rms2_g", 1, d, 1);
            add(p + "w_gu", 2 * f, d, 0);
            add(p + "w_down", d, f, 0);
        }
    }
    if (gpt) { add("lnf_g", 1, d, 1); add("lnf_b", 1, d, 2); }
    else add("rmsf_g", 1, d, 1);
    add("w_head", V, d, 0);
    return out;
}

Program build_program(const tio_model_cfg &c) {
    if (c.arch != TIO_ARCH_GPT && c.arch != TIO_ARCH_LLAMA) throw std::invalid_argument("arch");
    if (c.precision != TIO_PREC_FP32 && c.precision != TIO_PREC_BF16) throw std::invalid_argument("precision");
    if (c.n_layers < 1 || c.d_model < 8 || c.n_heads < 1 || c.d_ff < 8 || c.vocab < 2 || c.seq_len < 1 || c.batch < 1)
        throw std::invalid_argument("non-positive dimension");
    if (c.d_model % c.n_heads) throw std::invalid_argument("d_model must be a multiple of n_heads");
    if (c.d_model % 8 || c.d_ff % 8 || (c.d_model / c.n_heads) % 8)
        throw std::invalid_argument("d_model, d_ff and the head dimension must be multiples of 8");
    const int nmb = c.micro_batches > 1 ? c.micro_batches : 1;
    if (c.micro_batches < 0 || c.batch % nmb) throw std::invalid_argument("batch must be a multiple of micro_batches");

    Builder b;
    b.P.cfg = c;
    const bool gpt = c.arch == TIO_ARCH_GPT;
    const bool bf16 = c.precision == TIO_PREC_BF16;
    b.e = bf16 ? 2 : 4;
    // B, S: sequences and tokens of one micro-batch
    const int64_t L = c.n_layers, d = c.d_model, H = c.n_heads, f = c.d_ff, V = c.vocab, T = c.seq_len, B = c.batch / nmb;
    const int64_t S = B * T, Vp = vocab_ld(V), dh = d / H, S_total = S * nmb;

    // ---- persistent tensors
    b.P.params = list_params(c);
    for (auto &p : b.P.params) {
        int64_t n = p.rows * p.cols;
        p.w = b.tensor(p.name, n * b.e, KIND_WEIGHT);
        if (bf16) p.master = b.tensor(p.name + ".master", n * 4, KIND_MASTER);
        p.m = b.tensor(p.name + ".m", n * 4, KIND_M);
        p.v = b.tensor(p.name + ".v", n * 4, KIND_V);
    }
    for (int j = 0; j < nmb; ++j) {
        const std::string pre = nmb == 1 ? "" : "mb" + std::to_string(j) + ".";
        b.P.tokens_ids.push_back(b.tensor(pre + "tokens", S * 4, KIND_INPUT));
        b.P.labels_ids.push_back(b.tensor(pre + "labels", S * 4, KIND_INPUT));
    }
    b.P.n_persistent = (int)b.P.tensors.size();
    b.P.tokens_id = b.P.tokens_ids[0];
    b.P.labels_id = b.P.labels_ids[0];

    auto pidx = [&](const std::string &name) -> ParamInfo & {
        for (auto &p : b.P.params) if (p.name == name) return p;
        throw std::logic_error("no parameter " + name);
    };
    // parameters are looked up by position to avoid the linear search in the layer loop
    const int per_layer = gpt ? 12 : 6;
    const int first_layer_param = gpt ? 2 : 1;
    auto LP = [&](int layer, int j) -> ParamInfo & { return b.P.params[first_layer_param + layer * per_layer + j]; };
    // GPT layer slots: 0 ln1_g 1 ln1_b 2 w_qkv 3 b_qkv 4 w_o 5 b_o 6 ln2_g 7 ln2_b 8 w_fc1 9 b_fc1 10 w_fc2 11 b_fc2
    // Llama layer slots: 0 rms1_g 1 w_qkv 2 w_o 3 rms2_g 4 w_gu 5 w_down
    const int64_t nstat = gpt ? 2 : 1;
    const int64_t nb = (S + kNormBwdRows - 1) / kNormBwdRows;
    const int64_t attn_flops = 2 * B * H * T * T * dh;

    struct LayerT { int x_in, h1, st1, qkv, ao, lse, xm, h2, st2, u, act, xo; };
    int loss = -1;
    for (int mb = 0; mb < nmb; ++mb) {
    const bool first = mb == 0, last = mb == nmb - 1;
    const std::string pre = nmb == 1 ? "" : "mb" + std::to_string(mb) + ".";   // transient tensors of this micro-batch
    const int tokens_id = b.P.tokens_ids[mb], labels_id = b.P.labels_ids[mb];
    const int GW = first ? W : RW;            // gradient outputs: written by the first micro-batch, accumulated by the rest
    std::vector<LayerT> LT(L);

    auto norm_fwd = [&](int x, ParamInfo &g, ParamInfo *bias, int y, int st) {
        KernelRec &k = b.kernel(OP_NORM_FWD);
        set(k, 0, x, R); set(k, 1, g.w, R); if (bias) set(k, 2, bias->w, R);
        set(k, 3, y, W); set(k, 4, st, W);
        k.p[0] = S; k.p[1] = d;
    };
    auto gemm = [&](int A, ParamInfo &Wt, ParamInfo *bias, int resid, int C, int64_t N, int64_t K, int64_t ldc) {
        KernelRec &k = b.kernel(OP_GEMM);
        set(k, 0, A, R); set(k, 1, Wt.w, R); if (bias) set(k, 2, bias->w, R); if (resid >= 0) set(k, 3, resid, R);
        set(k, 4, C, W);
        k.p[0] = S; k.p[1] = N; k.p[2] = K; k.p[3] = ldc;
        k.flops = 2 * S * N * K;
    };

    // ---- forward
    int x0 = b.act(pre + "x0", S * d);
    {
        KernelRec &k = b.kernel(OP_EMBED_FWD);
        set(k, 0, tokens_id, R); set(k, 1, pidx("wte").w, R); if (gpt) set(k, 2, pidx("wpe").w, R);
        set(k, 3, x0, W);
        k.p[0] = S; k.p[1] = d; k.p[2] = T;
    }
    int x = x0;
    for (int i = 0; i < L; ++i) {
        std::string p = pre + "l" + std::to_string(i) + ".";
        LayerT &t = LT[i];
        t.x_in = x;
        t.h1 = b.act(p + "h1", S * d); t.st1 = b.act32(p + "st1", S * nstat);
        norm_fwd(x, LP(i, 0), gpt ? &LP(i, 1) : nullptr, t.h1, t.st1);
        t.qkv = b.act(p + "qkv", S * 3 * d);
        gemm(t.h1, LP(i, gpt ? 2 : 1), gpt ? &LP(i, 3) : nullptr, -1, t.qkv, 3 * d, d, 3 * d);
        if (!gpt) {
            KernelRec &k = b.kernel(OP_ROPE_FWD);
            set(k, 0, t.qkv, RW);
        }
        t.ao = b.act(p + "ao", S * d); t.lse = b.act32(p + "lse", B * H * T);
        {
            KernelRec &k = b.kernel(OP_ATTN_FWD);
            set(k, 0, t.qkv, R); set(k, 1, t.ao, W); set(k, 2, t.lse, W);
            k.flops = attn_flops;
        }
        t.xm = b.act(p + "xm", S * d);
        gemm(t.ao, LP(i, gpt ? 4 : 2), gpt ? &LP(i, 5) : nullptr, x, t.xm, d, d, d);
        t.h2 = b.act(p + "h2", S * d); t.st2 = b.act32(p + "st2", S * nstat);
        norm_fwd(t.xm, LP(i, gpt ? 6 : 3), gpt ? &LP(i, 7) : nullptr, t.h2, t.st2);
        if (gpt) {
            t.u = b.act(p + "u", S * f);
            gemm(t.h2, LP(i, 8), &LP(i, 9), -1, t.u, f, d, f);
            t.act = b.act(p + "act", S * f);
            KernelRec &k = b.kernel(OP_GELU_FWD);
            set(k, 0, t.u, R); set(k, 1, t.act, W);
            k.p[0] = S * f;
        } else {
            t.u = b.act(p + "u", S * 2 * f);
            gemm(t.h2, LP(i, 4), nullptr, -1, t.u, 2 * f, d, 2 * f);
            t.act = b.act(p + "act", S * f);
            KernelRec &k = b.kernel(OP_SWIGLU_FWD);
            set(k, 0, t.u, R); set(k, 1, t.act, W);
            k.p[0] = S; k.p[1] = f;
        }
        t.xo = b.act(p + "xo", S * d);
        gemm(t.act, LP(i, gpt ? 10 : 5), gpt ? &LP(i, 11) : nullptr, t.xm, t.xo, d, f, d);
        x = t.xo;
    }
    ParamInfo &fin_g = pidx(gpt ? "lnf_g" : "rmsf_g");
    ParamInfo *fin_b = gpt ? &pidx("lnf_b") : nullptr;
    ParamInfo &head = pidx("w_head");
    int hf = b.act(pre + "hf", S * d), stf = b.act32(pre + "stf", S * nstat);
    norm_fwd(x, fin_g, fin_b, hf, stf);
    int logits = b.act(pre + "logits", S * Vp);
    gemm(hf, head, nullptr, -1, logits, V, d, Vp);
    int losses = b.act32(pre + "losses", S);
    {
        KernelRec &k = b.kernel(OP_CE_FWD_BWD);
        set(k, 0, logits, RW); set(k, 1, labels_id, R); set(k, 2, losses, W);
        k.p[0] = S; k.p[1] = V; k.p[2] = Vp; k.p[3] = S_total;      // the loss is the mean over the whole batch
    }
    if (first) {
        loss = b.act32("loss", 1);
        b.P.loss_id = loss;
    }
    {
        KernelRec &k = b.kernel(OP_LOSS_REDUCE);
        set(k, 0, losses, R); set(k, 1, loss, GW);
        k.p[0] = S; k.p[1] = S_total; k.p[2] = first ? 0 : 1;       // later micro-batches add their share
    }

    // ---- backward
    auto pgrad = [&](ParamInfo &p) {
        if (first) p.grad = b.tensor("g." + p.name, p.rows * p.cols * b.e, KIND_PGRAD);
        return p.grad;
    };
    // A parameter is updated right after the launch that completes its gradient: nothing later in the
    // iteration reads it, the gradient dies at once, and the optimizer-state traffic overlaps the backward pass.
    auto adamw = [&](ParamInfo &p) {
        if (!last) return;
        KernelRec &k = b.kernel(OP_ADAMW);
        set(k, 0, p.grad, R); set(k, 1, p.w, RW); if (bf16) set(k, 2, p.master, RW);
        set(k, 3, p.m, RW); set(k, 4, p.v, RW);
        k.p[0] = p.rows * p.cols;
    };
    auto gemm_dx = [&](int dY, ParamInfo &Wt, int dX, int64_t n_in, int64_t n_out, int64_t ld_dy) {
        KernelRec &k = b.kernel(OP_GEMM_DX);
        set(k, 0, dY, R); set(k, 1, Wt.w, R); set(k, 2, dX, W);
        k.p[0] = S; k.p[1] = n_in; k.p[2] = n_out; k.p[3] = ld_dy;
        k.flops = 2 * S * n_in * n_out;
    };
    // the bias gradient (column sums of dY) is produced by the same launch as the weight gradient
    auto gemm_dw = [&](int dY, int X, ParamInfo &Wt, ParamInfo *bias, int64_t n_in, int64_t n_out, int64_t ld_dy) {
        pgrad(Wt);
        if (bias) pgrad(*bias);
        const int splits = bf16 ? dw_splits(n_out, n_in, S) : 1;
        int ws = -1;
        if (splits > 1) ws = b.grd32(pre + "ws." + Wt.name, splits * (n_out * n_in + n_out));   // fp32 partials + row sums
        KernelRec &k = b.kernel(OP_GEMM_DW);
        set(k, 0, dY, R); set(k, 1, X, R); set(k, 2, Wt.grad, GW);
        if (bias) set(k, 3, bias->grad, GW);
        if (ws >= 0) set(k, 4, ws, RW);
        k.p[0] = n_out; k.p[1] = n_in; k.p[2] = S; k.p[3] = ld_dy; k.p[4] = splits; k.p[5] = first ? 0 : 1;
        k.flops = 2 * S * n_in * n_out;
        adamw(Wt);
        if (bias) adamw(*bias);
    };
    auto norm_bwd = [&](int dy, int xin, int st, ParamInfo &g, ParamInfo *bias, int dres, const std::string &dxn,
                        const std::string &pn) {
        int dx = b.grd(dxn, S * d);
        int part = b.grd32(pn, nb * (bias ? 2 : 1) * d);
        {
            KernelRec &k = b.kernel(OP_NORM_BWD);
            set(k, 0, dy, R); set(k, 1, xin, R); set(k, 2, st, R); set(k, 3, g.w, R);
            if (dres >= 0) set(k, 4, dres, R);
            set(k, 5, dx, W); set(k, 6, part, W);
            k.p[0] = S; k.p[1] = d; k.p[2] = nb;
        }
        pgrad(g);
        if (bias) pgrad(*bias);
        {
            KernelRec &k = b.kernel(OP_NORM_BWD_PARAMS);
            set(k, 0, part, R); set(k, 1, g.grad, GW); if (bias) set(k, 2, bias->grad, GW);
            k.p[0] = nb; k.p[1] = d; k.p[2] = first ? 0 : 1;
        }
        adamw(g);
        if (bias) adamw(*bias);
        return dx;
    };

    int dhf = b.grd(pre + "dhf", S * d);
    gemm_dx(logits, head, dhf, d, V, Vp);
    gemm_dw(logits, hf, head, nullptr, d, V, Vp);
    int dx = norm_bwd(dhf, x, stf, fin_g, fin_b, -1, pre + "dxf", pre + "partf");
    for (int i = (int)L - 1; i >= 0; --i) {
        std::string p = pre + "l" + std::to_string(i) + ".";
        LayerT &t = LT[i];
        ParamInfo &w2 = LP(i, gpt ? 10 : 5);
        ParamInfo &w1 = LP(i, gpt ? 8 : 4);
        const int64_t f1 = gpt ? f : 2 * f;
        int dact = b.grd(p + "dact", S * f);
        gemm_dx(dx, w2, dact, f, d, d);
        gemm_dw(dx, t.act, w2, gpt ? &LP(i, 11) : nullptr, f, d, d);
        int du;
        if (gpt) {
            KernelRec &k = b.kernel(OP_GELU_BWD);
            set(k, 0, dact, RW); set(k, 1, t.u, R);
            k.p[0] = S * f;
            du = dact;
        } else {
            du = b.grd(p + "du", S * 2 * f);
            KernelRec &k = b.kernel(OP_SWIGLU_BWD);
            set(k, 0, dact, R); set(k, 1, t.u, R); set(k, 2, du, W);
            k.p[0] = S; k.p[1] = f;
        }
        int dh2 = b.grd(p + "dh2", S * d);
        gemm_dx(du, w1, dh2, d, f1, f1);
        gemm_dw(du, t.h2, w1, gpt ? &LP(i, 9) : nullptr, d, f1, f1);
        int dxm = norm_bwd(dh2, t.xm, t.st2, LP(i, gpt ? 6 : 3), gpt ? &LP(i, 7) : nullptr, dx, p + "dxm", p + "part2");
        ParamInfo &wo = LP(i, gpt ? 4 : 2);
        int dao = b.grd(p + "dao", S * d);
        gemm_dx(dxm, wo, dao, d, d, d);
        gemm_dw(dxm, t.ao, wo, gpt ? &LP(i, 5) : nullptr, d, d, d);
        int delta = b.grd32(p + "delta", B * H * T);
        {
            KernelRec &k = b.kernel(OP_ATTN_BWD_PRE);
            set(k, 0, dao, R); set(k, 1, t.ao, R); set(k, 2, delta, W);
        }
        int dqkv = b.grd(p + "dqkv", S * 3 * d);
        {
            KernelRec &k = b.kernel(OP_ATTN_BWD);
            set(k, 0, dao, R); set(k, 1, t.qkv, R); set(k, 2, t.lse, R); set(k, 3, delta, R); set(k, 4, dqkv, W);
            k.flops = attn_flops * 5 / 2;
        }
        if (!gpt) {
            KernelRec &k = b.kernel(OP_ROPE_BWD);
            set(k, 0, dqkv, RW);
        }
        ParamInfo &wqkv = LP(i, gpt ? 2 : 1);
        int dh1 = b.grd(p + "dh1", S * d);
        gemm_dx(dqkv, wqkv, dh1, d, 3 * d, 3 * d);
        gemm_dw(dqkv, t.h1, wqkv, gpt ? &LP(i, 3) : nullptr, d, 3 * d, 3 * d);
        dx = norm_bwd(dh1, t.x_in, t.st1, LP(i, 0), gpt ? &LP(i, 1) : nullptr, dxm, p + "dx", p + "part1");
    }
    {
        ParamInfo &wte = pidx("wte");
        pgrad(wte);
        {
            KernelRec &k = b.kernel(OP_EMBED_BWD);
            set(k, 0, dx, R); set(k, 1, tokens_id, R); set(k, 2, wte.grad, GW);
            k.p[0] = S; k.p[1] = d; k.p[2] = V; k.p[3] = first ? 0 : 1;
        }
        adamw(wte);
    }
    if (gpt) {
        ParamInfo &wpe = pidx("wpe");
        pgrad(wpe);
        {
            KernelRec &k = b.kernel(OP_POSEMB_BWD);
            set(k, 0, dx, R); set(k, 1, wpe.grad, GW);
            k.p[0] = B; k.p[1] = T; k.p[2] = d; k.p[3] = first ? 0 : 1;
        }
        adamw(wpe);
    }
    }   // micro-batches

    return b.P;
}

}  // namespace tio
