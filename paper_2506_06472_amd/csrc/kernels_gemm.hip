// Dense contractions of the training step: C[M,N] = A . B^T (+bias) (+residual).
//
// bf16: the MFMA kernel of kernels_gemm_dl.hip (operand tiles loaded straight into LDS) does the work, the pipelined
// kernel of kernels_gemm_pipe.hip (tiles staged through registers) where that one does not apply; this file holds the dispatch,
// the split-K reduction and a plain MFMA kernel with 64-bit addressing that takes over when an operand is
// too large for the pipelined kernel's 32-bit buffer offsets.  In the plain kernel a workgroup owns a
// BM x BN tile of C; both operand tiles are staged through LDS in [row][k] order with a 16-byte row
// pad, so that every MFMA operand is one 16-byte LDS read.  Operands that are stored with the
// contraction index as the slow dimension ("k-major": the weight in dX = dY.W, both operands in
// dW = dY^T.X) are transposed in registers in 8x8 blocks on their way into LDS, so no transposed
// copy of any tensor ever exists in HBM.  The accumulator layout is chosen so that each lane owns
// 4 consecutive columns of a row of C: the epilogue (bias, residual, rounding to bf16) writes 8 bytes
// per store.
//
// fp32: plain LDS-tiled FMA kernel (used by the small fp32 configurations, which are launch bound).
#include <cstdlib>
#include <stdexcept>

#include "../../include/teraio.h"
#include "device_common.h"
#include "kernels.h"
#include "mfma_tiles.h"

namespace tio {
namespace k {

namespace {

template <int BM, int BN, int BK, int WGM, int WGN, int NBUF, bool AKM, bool BKM>
__global__ void __launch_bounds__(WGM *WGN * 64)
    gemm_bf16_k(const uint16_t *__restrict__ A, int64_t lda, const uint16_t *__restrict__ B, int64_t ldb,
                const uint16_t *__restrict__ bias, const uint16_t *__restrict__ resid, int64_t ldr,
                uint16_t *__restrict__ C, int64_t ldc, int64_t M, int64_t N, int64_t K, int tiles_m, int tiles_n,
                uint16_t *__restrict__ rowsum, float *__restrict__ ws, int64_t k_chunk, int rowsum_acc) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int TPR = NT / BM;           // threads that share one row of the A tile for the row sums
    static_assert(NT % BM == 0 && (TPR & (TPR - 1)) == 0 && TPR <= 64 && BK % (8 * TPR) == 0, "row-sum mapping");
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
    constexpr int LS = BK + LDS_PAD;
    // NBUF operand tile pairs in LDS: with two, the stores of tile k+1 overlap the MFMAs of tile k and
    // one barrier per tile suffices
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    constexpr int TILE = (BM + BN) * LS;
    uint16_t *As = smem, *Bs = smem + BM * LS;

    // Tile order.  Workgroups are dealt to the 8 XCDs round-robin and every XCD has its own L2, so the
    // launch index is first turned into (xcd, index within the xcd) and each XCD gets one contiguous
    // eighth of the tile sequence; within the sequence groups of 8 tile rows walk the columns together.
    // The workgroups that share an L2 then work on neighbouring tiles: the 8 A tiles of the group stay in
    // that L2 and every B tile is fetched into it once per group, instead of once per XCD per group.
    const int tid = threadIdx.x;
    const int total_tiles = tiles_m * tiles_n;
    const int xcd_chunk = (total_tiles + 7) / 8;
    const int bid = (int)(blockIdx.x % 8) * xcd_chunk + (int)(blockIdx.x / 8);
    if (bid >= total_tiles) return;          // padding workgroups of the last chunk (whole workgroup, before any barrier)
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int g = bid / per_group;
    const int gm0 = g * GROUP;
    const int gsz = tiles_m - gm0 < GROUP ? tiles_m - gm0 : GROUP;
    const int tm = gm0 + (bid % per_group) % gsz;
    const int tn = (bid % per_group) / gsz;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    Stage<BM, BK, NT, AKM> sa;
    Stage<BN, BK, NT, BKM> sb;
    // split-K: workgroup row blockIdx.y owns the contraction range [kbeg, kend) and writes an fp32
    // partial tile to the workspace; a second launch adds the partials in split order
    const int64_t kbeg = (int64_t)blockIdx.y * k_chunk;
    const int64_t kend = (ws != nullptr && kbeg + k_chunk < K) ? kbeg + k_chunk : K;
    const int nk = (int)((kend - kbeg + BK - 1) / BK);
    sa.load(A, lda, m0, M, kbeg, kend, tid);
    sb.load(B, ldb, n0, N, kbeg, kend, tid);
    sa.store(As, tid);
    sb.store(Bs, tid);
    __syncthreads();
    // optional fused row sums of A over the whole contraction (the bias gradient when A = dY^T):
    // done by the workgroups of the first tile column, TPR threads per row, in k order
    const bool do_rowsum = rowsum != nullptr && tn == 0;
    float rsum = 0.f;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) {
            sa.load(A, lda, m0, M, kbeg + (int64_t)(kt + 1) * BK, kend, tid);
            sb.load(B, ldb, n0, N, kbeg + (int64_t)(kt + 1) * BK, kend, tid);
        }
        if (NBUF == 2) { As = smem + (kt & 1) * TILE; Bs = As + BM * LS; }
        if (do_rowsum) {
            const uint16_t *row = As + (tid / TPR) * LS + (tid % TPR) * (BK / TPR);
#pragma unroll
            for (int c = 0; c < BK / TPR; c += 8) {
                const uint4 v = *reinterpret_cast<const uint4 *>(row + c);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) rsum += __uint_as_float(w[e] << 16) + __uint_as_float(w[e] & 0xffff0000u);
            }
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            Frag fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i].u = *reinterpret_cast<const uint4 *>(As + (wm * WM + i * 32 + l32) * LS + ks * 16 + lhi * 8);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j].u = *reinterpret_cast<const uint4 *>(Bs + (wn * WN + j * 32 + l32) * LS + ks * 16 + lhi * 8);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    // first operand indexes the accumulator's register dimension (n), second its lane dimension (m)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j].v, fa[i].v, acc[i][j], 0, 0, 0);
        }
        if (NBUF == 2) {
            if (kt + 1 < nk) {
                sa.store(smem + ((kt + 1) & 1) * TILE, tid);
                sb.store(smem + ((kt + 1) & 1) * TILE + BM * LS, tid);
            }
            __syncthreads();
        } else {
            __syncthreads();
            if (kt + 1 < nk) {
                sa.store(As, tid);
                sb.store(Bs, tid);
                __syncthreads();
            }
        }
    }

    if (do_rowsum) {
#pragma unroll
        for (int o = 1; o < TPR; o <<= 1) rsum += __shfl_xor(rsum, o, 64);
        const int64_t m = m0 + tid / TPR;
        if (tid % TPR == 0 && m < M) {
            if (ws) ws[(int64_t)gridDim.y * M * N + (int64_t)blockIdx.y * M + m] = rsum;
            else rowsum[m] = (uint16_t)f32_to_bf16_bits(rsum + (rowsum_acc ? bf16_bits_to_f32(rowsum[m]) : 0.f));
        }
    }
    // epilogue: lane holds C[m][n .. n+3] for 4 groups of columns per 32x32 tile
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t m = m0 + wm * WM + i * 32 + l32;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t n = n0 + wn * WN + j * 32 + q * 8 + lhi * 4;
                if (n >= N) continue;
                float v[4] = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
                if (ws) {          // N is a multiple of 4 in split mode
                    *reinterpret_cast<float4 *>(ws + ((int64_t)blockIdx.y * M + m) * N + n) = make_float4(v[0], v[1], v[2], v[3]);
                    continue;
                }
                if (n + 4 <= N) {
                    if (bias) {
                        const uint2 t = *reinterpret_cast<const uint2 *>(bias + n);
                        v[0] += __uint_as_float(t.x << 16); v[1] += __uint_as_float(t.x & 0xffff0000u);
                        v[2] += __uint_as_float(t.y << 16); v[3] += __uint_as_float(t.y & 0xffff0000u);
                    }
                    if (resid) {
                        const uint2 t = *reinterpret_cast<const uint2 *>(resid + m * ldr + n);
                        v[0] += __uint_as_float(t.x << 16); v[1] += __uint_as_float(t.x & 0xffff0000u);
                        v[2] += __uint_as_float(t.y << 16); v[3] += __uint_as_float(t.y & 0xffff0000u);
                    }
                    uint2 o;
                    o.x = pack_bf16x2(v[0], v[1]);
                    o.y = pack_bf16x2(v[2], v[3]);
                    *reinterpret_cast<uint2 *>(C + m * ldc + n) = o;
                } else {
                    for (int e = 0; e < 4 && n + e < N; ++e) {
                        float x = v[e];
                        if (bias) x += bf16_bits_to_f32(bias[n + e]);
                        if (resid) x += bf16_bits_to_f32(resid[m * ldr + n + e]);
                        C[m * ldc + n + e] = (uint16_t)f32_to_bf16_bits(x);
                    }
                }
            }
        }
    }
}

// adds the split-K partials in split order and rounds once; also finishes the fused row sums
__global__ void __launch_bounds__(256) splitk_reduce_k(const float *__restrict__ ws, uint16_t *__restrict__ C, int64_t ldc,
                                                       uint16_t *__restrict__ rowsum, int64_t M, int64_t N, int splits,
                                                       int accumulate) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t nq = N / 4, total = M * nq;
    if (idx < total) {
        const int64_t m = idx / nq, n = (idx % nq) * 4;
        float4 a = *reinterpret_cast<const float4 *>(ws + m * N + n);
        for (int sp = 1; sp < splits; ++sp) {
            const float4 b = *reinterpret_cast<const float4 *>(ws + ((int64_t)sp * M + m) * N + n);
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        }
        if (accumulate) {          // earlier micro-batches' sum is in C
            const uint2 t = *reinterpret_cast<const uint2 *>(C + m * ldc + n);
            a.x += __uint_as_float(t.x << 16); a.y += __uint_as_float(t.x & 0xffff0000u);
            a.z += __uint_as_float(t.y << 16); a.w += __uint_as_float(t.y & 0xffff0000u);
        }
        uint2 o;
        o.x = pack_bf16x2(a.x, a.y);
        o.y = pack_bf16x2(a.z, a.w);
        *reinterpret_cast<uint2 *>(C + m * ldc + n) = o;
    } else if (rowsum != nullptr && idx - total < M) {
        const int64_t m = idx - total;
        const float *r = ws + (int64_t)splits * M * N;
        float a = r[m];
        for (int sp = 1; sp < splits; ++sp) a += r[(int64_t)sp * M + m];
        if (accumulate) a += bf16_bits_to_f32(rowsum[m]);
        rowsum[m] = (uint16_t)f32_to_bf16_bits(a);
    }
}

// ---------------------------------------------------------------- fp32
template <bool AKM, bool BKM>
__global__ void __launch_bounds__(256) gemm_f32_k(const float *__restrict__ A, int64_t lda, const float *__restrict__ B,
                                                  int64_t ldb, const float *__restrict__ bias,
                                                  const float *__restrict__ resid, int64_t ldr, float *__restrict__ C,
                                                  int64_t ldc, int64_t M, int64_t N, int64_t K,
                                                  float *__restrict__ rowsum, int rowsum_acc) {
    constexpr int BT = 64, BKK = 16;
    __shared__ float As[BKK][BT + 1];
    __shared__ float Bs[BKK][BT + 1];
    const int tid = threadIdx.x;
    const int64_t m0 = (int64_t)blockIdx.y * BT, n0 = (int64_t)blockIdx.x * BT;
    const int ty = tid / 16, tx = tid % 16;             // thread computes rows ty*4.., cols tx*4..
    float acc[4][4] = {};
    float rsum = 0.f;                                     // fused row sums of A (first tile column, thread = row)
    const bool do_rowsum = rowsum != nullptr && blockIdx.x == 0 && tid < BT;
    for (int64_t k0 = 0; k0 < K; k0 += BKK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * 256;                 // 0..1023
            int r, kk;
            if (AKM) { r = e % BT; kk = e / BT; } else { kk = e % BKK; r = e / BKK; }
            const int64_t gm = m0 + r, gk = k0 + kk;
            As[kk][r] = (gm < M && gk < K) ? (AKM ? A[gk * lda + gm] : A[gm * lda + gk]) : 0.f;
            if (BKM) { r = e % BT; kk = e / BT; } else { kk = e % BKK; r = e / BKK; }
            const int64_t gn = n0 + r, gkb = k0 + kk;
            Bs[kk][r] = (gn < N && gkb < K) ? (BKM ? B[gkb * ldb + gn] : B[gn * ldb + gkb]) : 0.f;
        }
        __syncthreads();
        if (do_rowsum)
#pragma unroll
            for (int kk = 0; kk < BKK; ++kk) rsum += As[kk][tid];
#pragma unroll
        for (int kk = 0; kk < BKK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    if (do_rowsum && m0 + tid < M) rowsum[m0 + tid] = rsum + (rowsum_acc ? rowsum[m0 + tid] : 0.f);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float x = acc[i][j];
            if (bias) x += bias[n];
            if (resid) x += resid[m * ldr + n];
            C[m * ldc + n] = x;
        }
    }
}

}  // namespace

template <int BM, int BN, int BK, int WGM, int WGN, int NBUF>
static void launch_bf16(hipStream_t s, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                        const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr, void *C, int64_t ldc,
                        void *rowsum, void *workspace, int splits, bool accumulate) {
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    float *ws = splits > 1 ? (float *)workspace : nullptr;
    const int64_t k_chunk = splits > 1 ? ((K + splits - 1) / splits + BK - 1) / BK * BK : K;
    const dim3 grid((unsigned)(8 * ((tiles_m * tiles_n + 7) / 8)), (unsigned)(splits > 1 ? splits : 1));
    const dim3 block(WGM * WGN * 64);
    constexpr size_t lds = (size_t)NBUF * (BM + BN) * (BK + LDS_PAD) * 2;
    static bool attr_done = false;           // tiles above 64 KiB of LDS need the limit raised once per kernel
    if (!attr_done) {
        (void)hipFuncSetAttribute((const void *)gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_done = true;
    }
#define TIO_GEMM_ARGS (const uint16_t *)A, lda, (const uint16_t *)B, ldb, (const uint16_t *)bias, (const uint16_t *)resid, ldr, \
                      (uint16_t *)C, ldc, M, N, K, tiles_m, tiles_n, (uint16_t *)rowsum, ws, k_chunk, (int)accumulate
    if (!a_km && !b_km) gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, false, false><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else if (!a_km && b_km) gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, false, true><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else if (a_km && b_km) gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, true, true><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else gemm_bf16_k<BM, BN, BK, WGM, WGN, NBUF, true, false><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
#undef TIO_GEMM_ARGS
    if (ws) {
        const int64_t n = M * (N / 4) + (rowsum ? M : 0);
        splitk_reduce_k<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(ws, (uint16_t *)C, ldc, (uint16_t *)rowsum, M, N, splits, (int)accumulate);
    }
}

static int gemm_cfg_override() {
    static int v = -2;
    if (v == -2) { const char *e = getenv("TIO_GEMM_CFG"); v = e ? atoi(e) : -1; }
    return v;
}

static bool gemm_direct_enabled() {
    static int v = -1;
    if (v < 0) { const char *e = getenv("TIO_GEMM_DIRECT"); v = e ? (atoi(e) != 0) : 1; }
    return v != 0;
}

void gemm(hipStream_t s, int dtype, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
          const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr, void *C, int64_t ldc,
          void *rowsum, void *workspace, int splits, bool accumulate) {
    if (M <= 0 || N <= 0 || K <= 0) return;
    // split-K needs the fp32 workspace, no epilogue operands and whole float4 rows
    if (dtype != TIO_PREC_BF16 || !workspace || bias || resid || (N % 4) || splits < 2) splits = 1;
    // accumulate: C += A.B^T and rowsum += row sums (gradient accumulation over micro-batches).  In a single
    // pass the old C is the residual operand (every element is read and then written by the same lane); with
    // split-K the reduction launch adds it.
    if (accumulate && splits == 1) {
        if (resid) throw std::invalid_argument("gemm: accumulate cannot be combined with a residual operand");
        resid = C;
        ldr = ldc;
    }
    if (dtype == TIO_PREC_BF16) {
        // The pipelined kernel is the default.  Its 256x256 tiles (eight wavefronts, 128x64 each: fewer LDS
        // bytes per MFMA) run one per CU, its 128x128 tiles two per CU at about 0.8 of the large tile's rate
        // (measured on 768- to 5120-wide products); the choice goes to the one that loses less to the last,
        // partly filled round over the 256 CUs.  TIO_GEMM_CFG forces a choice: 0 plain kernel, 1 pipelined 128x128,
        // 2 pipelined 256x256.
        const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
        const int64_t small_tiles = ((M + 127) / 128) * ((N + 127) / 128) * (splits > 1 ? splits : 1);
        auto fill = [](int64_t tiles, int64_t slots) { return (double)tiles / (double)((tiles + slots - 1) / slots * slots); };
        const bool large = splits <= 1 && fill(big_tiles, 256) >= 0.8 * fill(small_tiles, 512);
        const int ov = gemm_cfg_override();
        const int pipe_cfg = ov == 1 ? 0 : ov == 2 ? 1 : (large ? 1 : 0);
        // first choice: operand tiles straight from global memory into LDS; the kernel that stages them through
        // registers takes the products it refuses (K not a multiple of 8); TIO_GEMM_DIRECT=0 switches the first one off
        float *const wsp = splits > 1 ? (float *)workspace : nullptr;
        if (ov != 0 && ((gemm_direct_enabled() && gemm_bf16_direct(s, pipe_cfg, a_km, b_km, M, N, K, A, lda, B, ldb, bias, resid, ldr, C,
                                                                   ldc, rowsum, wsp, splits, accumulate)) ||
                        gemm_bf16_pipelined(s, pipe_cfg, a_km, b_km, M, N, K, A, lda, B, ldb, bias, resid, ldr, C, ldc, rowsum, wsp,
                                            splits, accumulate))) {
            if (splits > 1) {
                const int64_t n = M * (N / 4) + (rowsum ? M : 0);
                splitk_reduce_k<<<(unsigned)((n + 255) / 256), 256, 0, s>>>((const float *)workspace, (uint16_t *)C, ldc, (uint16_t *)rowsum, M, N, splits, (int)accumulate);
            }
            return;
        }
        // operands too large for 32-bit buffer offsets: plain kernel with 64-bit addressing
        launch_bf16<128, 128, 64, 2, 2, 1>(s, a_km, b_km, M, N, K, A, lda, B, ldb, bias, resid, ldr, C, ldc, rowsum, workspace, splits, accumulate);
    } else {
        const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
#define TIO_GEMM_ARGS (const float *)A, lda, (const float *)B, ldb, (const float *)bias, (const float *)resid, ldr, (float *)C, ldc, M, N, K, (float *)rowsum, (int)accumulate
        if (!a_km && !b_km) gemm_f32_k<false, false><<<grid, 256, 0, s>>>(TIO_GEMM_ARGS);
        else if (!a_km && b_km) gemm_f32_k<false, true><<<grid, 256, 0, s>>>(TIO_GEMM_ARGS);
        else if (a_km && b_km) gemm_f32_k<true, true><<<grid, 256, 0, s>>>(TIO_GEMM_ARGS);
        else gemm_f32_k<true, false><<<grid, 256, 0, s>>>(TIO_GEMM_ARGS);
#undef TIO_GEMM_ARGS
    }
}

}  // namespace k
}  // namespace tio
