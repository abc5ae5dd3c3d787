// Host-side launchers of the gfx950 kernels.  dtype: TIO_PREC_FP32 or TIO_PREC_BF16 (element type
// of activations / weights / gradients); statistics, softmax, loss and optimizer state are fp32.
// All pointers are device pointers, 16-byte aligned; row strides are multiples of 8 elements.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace tio {
namespace k {

void embed_fwd(hipStream_t s, int dtype, const int32_t *tok, const void *wte, const void *wpe, void *x,
               int64_t S, int64_t d, int64_t T);
void norm_fwd(hipStream_t s, int dtype, bool rms, const void *x, const void *g, const void *b, void *y,
              float *stats, int64_t S, int64_t d, float eps);
// C[M,N] = A.B^T (+bias[N]) (+resid[M,N]); a_km / b_km: operand stored [K][rows] instead of [rows][K];
// rowsum (optional, [M]): sum over k of A[m][k], produced by the same launch (bias gradient of dW);
// workspace/splits: with splits > 1 and an fp32 workspace of splits*(M*N+M) floats the contraction is
// cut into `splits` ranges whose partial results are added in order by a second launch
// pipelined bf16 MFMA GEMM (kernels_gemm_pipe.hip); cfg 0: 128x128 tiles, 1: 256x256 tiles.  Returns false
// without launching when an operand is too large for its 32-bit buffer offsets.  With ws != nullptr the
// fp32 split-K partials go to ws and the caller runs the reduction.
bool gemm_bf16_pipelined(hipStream_t s, int cfg, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A,
                         int64_t lda, const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr,
                         void *C, int64_t ldc, void *rowsum, float *ws, int splits, bool rowsum_accumulate);
// bf16 MFMA GEMM whose operand tiles are loaded from global memory straight into LDS (kernels_gemm_dl.hip); same
// arguments and tile configurations as gemm_bf16_pipelined.  Returns false without launching when K is not a multiple of 8
// (a partly valid 16-byte chunk cannot be masked on its way into LDS) or an operand is too large for 32-bit offsets.
bool gemm_bf16_direct(hipStream_t s, int cfg, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A,
                      int64_t lda, const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr,
                      void *C, int64_t ldc, void *rowsum, float *ws, int splits, bool rowsum_accumulate);
void gemm(hipStream_t s, int dtype, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A,
          int64_t lda, const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr, void *C,
          int64_t ldc, void *rowsum, void *workspace, int splits, bool accumulate = false);

void rope(hipStream_t s, int dtype, void *qkv, int64_t B, int64_t T, int64_t H, int64_t dh, float theta,
          bool inverse);
void attn_fwd(hipStream_t s, int dtype, const void *qkv, void *o, float *lse, int64_t B, int64_t T, int64_t H,
              int64_t dh);
// matrix-core attention (bf16, head dimension 64 or 128); attn_fwd / attn_bwd dispatch to it
bool attn_mfma_supported(int dtype, int64_t T, int64_t H, int64_t dh);
void attn_fwd_mfma(hipStream_t s, const void *qkv, void *o, float *lse, int64_t B, int64_t T, int64_t H, int64_t dh);
void attn_bwd_mfma(hipStream_t s, const void *dO, const void *qkv, const float *lse, const float *delta, void *dqkv,
                   int64_t B, int64_t T, int64_t H, int64_t dh);
void gelu_fwd(hipStream_t s, int dtype, const void *u, void *y, int64_t n);
void swiglu_fwd(hipStream_t s, int dtype, const void *gu, void *y, int64_t S, int64_t f);
// S rows of this launch; S_total: tokens of the whole batch (the loss is their mean)
void ce_fwd_bwd(hipStream_t s, int dtype, void *logits, const int32_t *labels, float *losses, int64_t S,
                int64_t V, int64_t ld, int64_t S_total);
// loss[0] (+)= sum(losses[0..S)) / S_total
void loss_reduce(hipStream_t s, const float *losses, float *loss, int64_t S, int64_t S_total, bool accumulate);
void gelu_bwd(hipStream_t s, int dtype, void *dact, const void *u, int64_t n);
void swiglu_bwd(hipStream_t s, int dtype, const void *dact, const void *gu, void *dgu, int64_t S, int64_t f);
void norm_bwd(hipStream_t s, int dtype, bool rms, const void *dy, const void *x, const float *stats,
              const void *g, const void *dres, void *dx, float *part, int64_t S, int64_t d, int64_t nb);
// accumulate (here and below): add to the gradient already in the output (later micro-batches)
void norm_bwd_params(hipStream_t s, int dtype, bool rms, const float *part, void *dg, void *db, int64_t nb,
                     int64_t d, bool accumulate);
void attn_bwd_pre(hipStream_t s, int dtype, const void *dO, const void *O, float *delta, int64_t B, int64_t T,
                  int64_t H, int64_t dh);
void attn_bwd(hipStream_t s, int dtype, const void *dO, const void *qkv, const float *lse, const float *delta,
              void *dqkv, int64_t B, int64_t T, int64_t H, int64_t dh);
void embed_bwd(hipStream_t s, int dtype, const void *dx, const int32_t *tok, void *dwte, int64_t S, int64_t d,
               int64_t V, bool accumulate);
void posemb_bwd(hipStream_t s, int dtype, const void *dx, void *dwpe, int64_t B, int64_t T, int64_t d, bool accumulate);
void adamw(hipStream_t s, int dtype, const void *g, void *w, float *master, float *m, float *v, int64_t n,
           float lr, float beta1, float beta2, float eps, float wd, float bc1, float bc2);
void fill_u32(hipStream_t s, void *p, uint32_t value, int64_t n_words);
// fp32 <-> storage conversion helpers used when parameters are loaded and read back
void convert_from_f32(hipStream_t s, int dtype, const float *src, void *dst, int64_t n);

}  // namespace k
}  // namespace tio
