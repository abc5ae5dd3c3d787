// Kernel schedule ("program") of one training iteration: the tensors, the launches in launch
// order and the operands of every launch.  The profiler of the paper (Section 3.1) learns this by
// instrumenting framework operators; here the launcher itself is the instrumentation point, so the
// structural trace is exactly this list.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/teraio.h"

namespace tio {

enum Op : int32_t {
    OP_EMBED_FWD = 0, OP_NORM_FWD, OP_GEMM, OP_ROPE_FWD, OP_ATTN_FWD, OP_GELU_FWD, OP_SWIGLU_FWD,
    OP_CE_FWD_BWD, OP_LOSS_REDUCE, OP_GEMM_DX, OP_GEMM_DW, OP_BIAS_GRAD, OP_GELU_BWD, OP_SWIGLU_BWD,
    OP_NORM_BWD, OP_NORM_BWD_PARAMS, OP_ATTN_BWD_PRE, OP_ATTN_BWD, OP_ROPE_BWD, OP_EMBED_BWD,
    OP_POSEMB_BWD, OP_ADAMW, OP_COUNT
};   // OP_BIAS_GRAD is a reserved code: the bias gradient comes out of the weight-gradient GEMM

enum Kind : int32_t { KIND_WEIGHT = 0, KIND_MASTER, KIND_M, KIND_V, KIND_INPUT, KIND_ACT, KIND_GRAD, KIND_PGRAD };

constexpr int kMaxRoles = 8;
constexpr int kNormBwdRows = 8;    // token rows per norm-backward workgroup (fixes the partials size)

struct TensorInfo {
    uint64_t bytes;      // payload rounded up to 256
    int32_t kind;
    std::string name;
};

struct KernelRec {
    int32_t op;
    int32_t t[kMaxRoles];     // tensor id per operand role, -1 = absent
    uint8_t fl[kMaxRoles];    // bit0 read, bit1 written
    int64_t p[6];             // integer launch parameters (meaning per op, see runtime)
    int64_t flops;
};

struct ParamInfo {
    std::string name;
    int64_t rows, cols;       // vectors: rows = 1
    int32_t w, master, m, v;  // tensor ids (master = -1 in fp32 mode)
    int32_t grad;             // tensor id of the gradient
    int32_t init;             // 0 normal, 1 ones, 2 zeros (information for callers)
};

struct Program {
    tio_model_cfg cfg;
    std::vector<TensorInfo> tensors;
    std::vector<KernelRec> kernels;
    std::vector<ParamInfo> params;
    int32_t n_persistent = 0;
    int32_t tokens_id = -1, labels_id = -1, loss_id = -1;
    std::vector<int32_t> tokens_ids, labels_ids;     // one buffer per micro-batch (tokens_id / labels_id = the first)
};

// Throws std::invalid_argument on a bad configuration.
Program build_program(const tio_model_cfg &cfg);
std::vector<ParamInfo> list_params(const tio_model_cfg &cfg);
inline int64_t vocab_ld(int64_t V) { return (V + 63) / 64 * 64; }
// Number of contraction ranges of a bf16 weight-gradient GEMM dW[M,N] = dY^T.X over K tokens: small
// weight matrices give too few 128x128 output tiles to fill the GPU, so the token dimension is
// split (powers of two, at most 8, at least 256 tokens per range) until about 512 workgroups exist.
inline int dw_splits(int64_t M, int64_t N, int64_t K) {
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    int s = 1;
    while (s < 8 && tiles * s * 2 <= 512 && K / (s * 2) >= 256) s *= 2;
    return s;
}

}  // namespace tio
