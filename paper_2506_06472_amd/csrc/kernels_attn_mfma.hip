// Causal self-attention on the matrix cores (bf16, head dimension 64 or 128), forward and backward,
// on the packed [S, 3d] q|k|v layout.
//
// Each wavefront owns 32 query rows (forward, dQ) or 32 key rows (dK/dV) and keeps their operand
// fragments in registers for the whole kernel; the other side streams through LDS in tiles of 64 rows.
// Scores are produced transposed (keys x queries in the forward and dQ kernels, queries x keys in the
// dK/dV kernel) so that in the accumulator layout of v_mfma_f32_32x32x16_bf16 the row owned by the
// wavefront is the lane index: the softmax statistics of a row live in one lane (plus one exchange with
// lane+32), and the probabilities can be fed to the second product straight from registers as its B
// operand.  The operand whose contraction index is the sequence position (V in P.V, K in dS.K, Q and dO
// in the dK/dV products) is staged into LDS transposed (8x8 register transposes), and its fragments are
// read with the slot order the accumulator registers dictate.  Statistics are fp32, exp2 with the
// 1/sqrt(dh) scale folded into the exponent; the backward pass recomputes P from the saved
// log-sum-exp; dQ and dK/dV are separate launches, so every sum has a fixed order and no atomics.
#include "../../include/teraio.h"
#include "device_common.h"
#include "kernels.h"
#include "mfma_tiles.h"

namespace tio {
namespace k {

namespace {

constexpr int NT = 256;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int PT = 64 + LDS_PAD;          // row pitch (elements) of the transposed tiles: 64 sequence positions

__device__ __forceinline__ uint32_t pack2(float a, float b) { return f32_to_bf16_bits(a) | (f32_to_bf16_bits(b) << 16); }

// B operand of a 16-deep product from accumulator registers R0..R0+7 (the contraction index is the
// accumulator's row index: slots 0..3 = rows base+4*lhi+0..3, slots 4..7 = rows base+8+4*lhi+0..3)
template <int R0> __device__ __forceinline__ bf16x8 pack8(const floatx16 &v) {
    Frag f;
    f.u = make_uint4(pack2(v[R0], v[R0 + 1]), pack2(v[R0 + 2], v[R0 + 3]), pack2(v[R0 + 4], v[R0 + 5]), pack2(v[R0 + 6], v[R0 + 7]));
    return f.v;
}
// A operand from a row-major LDS tile: row, 8 consecutive elements
__device__ __forceinline__ bf16x8 row_frag(const uint16_t *lds, int pitch, int row, int col) {
    Frag f;
    f.u = *reinterpret_cast<const uint4 *>(lds + row * pitch + col);
    return f.v;
}
// A operand from a transposed LDS tile with the slot order of pack8
__device__ __forceinline__ bf16x8 t_frag(const uint16_t *lds, int row, int colbase, int lhi) {
    const uint2 a = *reinterpret_cast<const uint2 *>(lds + row * PT + colbase + 4 * lhi);
    const uint2 b = *reinterpret_cast<const uint2 *>(lds + row * PT + colbase + 8 + 4 * lhi);
    Frag f;
    f.u = make_uint4(a.x, a.y, b.x, b.y);
    return f.v;
}
__device__ __forceinline__ floatx16 zero16() {
    floatx16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}
__device__ __forceinline__ bf16x8 global_frag(const uint16_t *p, bool ok) {
    Frag f;
    f.u = ok ? *reinterpret_cast<const uint4 *>(p) : make_uint4(0, 0, 0, 0);
    return f.v;
}
// row index inside a 32x32 accumulator tile of register r for lane half lhi
__device__ __forceinline__ int acc_row(int r, int lhi) { return 8 * (r >> 2) + 4 * lhi + (r & 3); }

// ------------------------------------------------------------------------------------------ forward
template <int DH>
__global__ void __launch_bounds__(NT) attn_fwd_mfma_k(const uint16_t *__restrict__ qkv, uint16_t *__restrict__ o,
                                                      float *__restrict__ lse, int64_t Tn, int64_t H, float scale) {
    constexpr int KS = DH / 16, DT = DH / 32, PK = DH + LDS_PAD;
    __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * PK];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[DH * PT];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int64_t d = H * DH, ld = 3 * d;
    const int64_t bh = blockIdx.y, b = bh / H, h = bh % H;
    const int64_t q0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * 128;      // longest rows first
    const int64_t q0w = q0 + wave * 32, q = q0w + l32;
    const uint16_t *qb = qkv + b * Tn * ld + h * DH, *kb = qb + d, *vb = qb + 2 * d;
    const float c = scale * LOG2E;

    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = global_frag(qb + q * ld + ks * 16 + lhi * 8, q < Tn);
    floatx16 oacc[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) oacc[i] = zero16();
    float m = -INFINITY, l = 0.f;
    const int64_t kv_end = q0 + 128 < Tn ? q0 + 128 : Tn;
    for (int64_t j0 = 0; j0 < kv_end; j0 += 64) {
        Stage<64, DH, NT, false> sk;
        Stage<DH, 64, NT, true> sv;
        sk.load(kb, ld, j0, Tn, 0, DH, tid);
        sv.load(vb, ld, 0, DH, j0, Tn, tid);
        __syncthreads();
        sk.store(Ks, tid);
        sv.store(Vt, tid);
        __syncthreads();
        if (j0 <= q0w + 31) {
            floatx16 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                s[kt] = zero16();
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(Ks, PK, kt * 32 + l32, ks * 16 + lhi * 8), qf[ks], s[kt], 0, 0, 0);
            }
            float tmax = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t kv = j0 + kt * 32 + acc_row(r, lhi);
                    const float x = kv <= q ? s[kt][r] * c : -INFINITY;
                    s[kt][r] = x;
                    tmax = fmaxf(tmax, x);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float mn = fmaxf(m, tmax);
            const bool dead = mn == -INFINITY;                 // nothing visible to this row yet
            const float corr = dead ? 1.0f : __builtin_amdgcn_exp2f(m - mn);
            l *= corr;
#pragma unroll
            for (int i = 0; i < DT; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = dead ? 0.0f : __builtin_amdgcn_exp2f(s[kt][r] - mn);
                    l += p;
                    s[kt][r] = p;
                }
            m = mn;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16x8 p0 = pack8<0>(s[kt]), p1 = pack8<8>(s[kt]);
#pragma unroll
                for (int i = 0; i < DT; ++i) {
                    oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Vt, i * 32 + l32, kt * 32, lhi), p0, oacc[i], 0, 0, 0);
                    oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Vt, i * 32 + l32, kt * 32 + 16, lhi), p1, oacc[i], 0, 0, 0);
                }
            }
        }
    }
    l += __shfl_xor(l, 32, 64);
    if (q < Tn) {
        const float inv = 1.0f / l;
        uint16_t *orow = o + (b * Tn + q) * d + h * DH;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                w.x = pack2(oacc[i][4 * g] * inv, oacc[i][4 * g + 1] * inv);
                w.y = pack2(oacc[i][4 * g + 2] * inv, oacc[i][4 * g + 3] * inv);
                *reinterpret_cast<uint2 *>(orow + i * 32 + 8 * g + 4 * lhi) = w;
            }
        if (lhi == 0) lse[bh * Tn + q] = (m + log2f(l)) * LN2;
    }
}

// ------------------------------------------------------------------------------------------ dQ
template <int DH>
__global__ void __launch_bounds__(NT) attn_bwd_dq_mfma_k(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ qkv,
                                                         const float *__restrict__ lse, const float *__restrict__ delta,
                                                         uint16_t *__restrict__ dqkv, int64_t Tn, int64_t H, float scale) {
    constexpr int KS = DH / 16, DT = DH / 32, PK = DH + LDS_PAD;
    __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * PK];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[64 * PK];
    __shared__ __attribute__((aligned(16))) uint16_t Kt[DH * PT];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int64_t d = H * DH, ld = 3 * d;
    const int64_t bh = blockIdx.y, b = bh / H, h = bh % H;
    const int64_t q0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * 128;
    const int64_t q0w = q0 + wave * 32, q = q0w + l32;
    const uint16_t *qb = qkv + b * Tn * ld + h * DH, *kb = qb + d, *vb = qb + 2 * d;
    const uint16_t *gb = dO + b * Tn * d + h * DH;
    const float c = scale * LOG2E;
    const bool live = q < Tn;

    bf16x8 qf[KS], gf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qf[ks] = global_frag(qb + q * ld + ks * 16 + lhi * 8, live);
        gf[ks] = global_frag(gb + q * d + ks * 16 + lhi * 8, live);
    }
    const float lse2 = live ? lse[bh * Tn + q] * LOG2E : 0.f;
    const float dl = live ? delta[bh * Tn + q] : 0.f;
    floatx16 dq[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) dq[i] = zero16();
    const int64_t kv_end = q0 + 128 < Tn ? q0 + 128 : Tn;
    for (int64_t j0 = 0; j0 < kv_end; j0 += 64) {
        __syncthreads();
        {
            Stage<64, DH, NT, false> sk, sv;
            sk.load(kb, ld, j0, Tn, 0, DH, tid);
            sv.load(vb, ld, j0, Tn, 0, DH, tid);
            sk.store(Ks, tid);
            sv.store(Vs, tid);
        }
        {
            Stage<DH, 64, NT, true> st;
            st.load(kb, ld, 0, DH, j0, Tn, tid);
            st.store(Kt, tid);
        }
        __syncthreads();
        if (j0 <= q0w + 31) {
            floatx16 s[2], dp[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                s[kt] = zero16(); dp[kt] = zero16();
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(Ks, PK, kt * 32 + l32, ks * 16 + lhi * 8), qf[ks], s[kt], 0, 0, 0);
                    dp[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(Vs, PK, kt * 32 + l32, ks * 16 + lhi * 8), gf[ks], dp[kt], 0, 0, 0);
                }
            }
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t kv = j0 + kt * 32 + acc_row(r, lhi);
                    const float p = kv <= q ? __builtin_amdgcn_exp2f(s[kt][r] * c - lse2) : 0.0f;
                    s[kt][r] = p * (dp[kt][r] - dl) * scale;
                }
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16x8 d0 = pack8<0>(s[kt]), d1 = pack8<8>(s[kt]);
#pragma unroll
                for (int i = 0; i < DT; ++i) {
                    dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Kt, i * 32 + l32, kt * 32, lhi), d0, dq[i], 0, 0, 0);
                    dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Kt, i * 32 + l32, kt * 32 + 16, lhi), d1, dq[i], 0, 0, 0);
                }
            }
        }
    }
    if (live) {
        uint16_t *orow = dqkv + (b * Tn + q) * ld + h * DH;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                w.x = pack2(dq[i][4 * g], dq[i][4 * g + 1]);
                w.y = pack2(dq[i][4 * g + 2], dq[i][4 * g + 3]);
                *reinterpret_cast<uint2 *>(orow + i * 32 + 8 * g + 4 * lhi) = w;
            }
    }
}

// ------------------------------------------------------------------------------------------ dK, dV
template <int DH>
__global__ void __launch_bounds__(NT) attn_bwd_dkv_mfma_k(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ qkv,
                                                          const float *__restrict__ lse, const float *__restrict__ delta,
                                                          uint16_t *__restrict__ dqkv, int64_t Tn, int64_t H, float scale) {
    constexpr int KS = DH / 16, DT = DH / 32, PK = DH + LDS_PAD;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *Qs = smem, *Gs = Qs + 64 * PK, *Qt = Gs + 64 * PK, *Gt = Qt + DH * PT;
    float *L2s = reinterpret_cast<float *>(Gt + DH * PT), *Ds = L2s + 64;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int64_t d = H * DH, ld = 3 * d;
    const int64_t bh = blockIdx.y, b = bh / H, h = bh % H;
    const int64_t kv0 = (int64_t)blockIdx.x * 128;                        // earliest keys see the most queries: first
    const int64_t kv0w = kv0 + wave * 32, kv = kv0w + l32;
    const uint16_t *qb = qkv + b * Tn * ld + h * DH, *kb = qb + d, *vb = qb + 2 * d;
    const uint16_t *gb = dO + b * Tn * d + h * DH;
    const float c = scale * LOG2E;
    const bool live = kv < Tn;

    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        kf[ks] = global_frag(kb + kv * ld + ks * 16 + lhi * 8, live);
        vf[ks] = global_frag(vb + kv * ld + ks * 16 + lhi * 8, live);
    }
    floatx16 dk[DT], dv[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) { dk[i] = zero16(); dv[i] = zero16(); }
    for (int64_t i0 = kv0; i0 < Tn; i0 += 64) {
        __syncthreads();
        {
            Stage<64, DH, NT, false> sq, sg;
            sq.load(qb, ld, i0, Tn, 0, DH, tid);
            sg.load(gb, d, i0, Tn, 0, DH, tid);
            sq.store(Qs, tid);
            sg.store(Gs, tid);
        }
        {
            Stage<DH, 64, NT, true> st;                       // the two transposed tiles use different waves
            st.load(qb, ld, 0, DH, i0, Tn, tid);
            st.store(Qt, tid);
            const int tid2 = (tid + 128) & 255;
            st.load(gb, d, 0, DH, i0, Tn, tid2);
            st.store(Gt, tid2);
        }
        if (tid < 64) {
            const bool ok = i0 + tid < Tn;
            L2s[tid] = ok ? lse[bh * Tn + i0 + tid] * LOG2E : 0.f;
            Ds[tid] = ok ? delta[bh * Tn + i0 + tid] : 0.f;
        }
        __syncthreads();
        if (i0 + 63 >= kv0w) {
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                floatx16 s = zero16(), dp = zero16();
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(Qs, PK, qt * 32 + l32, ks * 16 + lhi * 8), kf[ks], s, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(Gs, PK, qt * 32 + l32, ks * 16 + lhi * 8), vf[ks], dp, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ql = qt * 32 + acc_row(r, lhi);
                    const int64_t qi = i0 + ql;
                    const float p = (qi >= kv && qi < Tn) ? __builtin_amdgcn_exp2f(s[r] * c - L2s[ql]) : 0.0f;
                    dp[r] = p * (dp[r] - Ds[ql]) * scale;
                    s[r] = p;
                }
                const bf16x8 p0 = pack8<0>(s), p1 = pack8<8>(s), d0 = pack8<0>(dp), d1 = pack8<8>(dp);
#pragma unroll
                for (int i = 0; i < DT; ++i) {
                    dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Gt, i * 32 + l32, qt * 32, lhi), p0, dv[i], 0, 0, 0);
                    dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Gt, i * 32 + l32, qt * 32 + 16, lhi), p1, dv[i], 0, 0, 0);
                    dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Qt, i * 32 + l32, qt * 32, lhi), d0, dk[i], 0, 0, 0);
                    dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(t_frag(Qt, i * 32 + l32, qt * 32 + 16, lhi), d1, dk[i], 0, 0, 0);
                }
            }
        }
    }
    if (live) {
        uint16_t *krow = dqkv + (b * Tn + kv) * ld + d + h * DH, *vrow = krow + d;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                w.x = pack2(dk[i][4 * g], dk[i][4 * g + 1]);
                w.y = pack2(dk[i][4 * g + 2], dk[i][4 * g + 3]);
                *reinterpret_cast<uint2 *>(krow + i * 32 + 8 * g + 4 * lhi) = w;
                w.x = pack2(dv[i][4 * g], dv[i][4 * g + 1]);
                w.y = pack2(dv[i][4 * g + 2], dv[i][4 * g + 3]);
                *reinterpret_cast<uint2 *>(vrow + i * 32 + 8 * g + 4 * lhi) = w;
            }
    }
}

template <int DH> constexpr size_t dkv_smem() { return (size_t)(2 * 64 * (DH + LDS_PAD) + 2 * DH * PT) * 2 + 128 * 4; }

}  // namespace

bool attn_mfma_supported(int dtype, int64_t dh) { return dtype == TIO_PREC_BF16 && (dh == 64 || dh == 128); }

void attn_fwd_mfma(hipStream_t s, const void *qkv, void *o, float *lse, int64_t B, int64_t Tn, int64_t H, int64_t dh) {
    const dim3 grid((unsigned)((Tn + 127) / 128), (unsigned)(B * H));
    const float scale = 1.0f / sqrtf((float)dh);
    if (dh == 64) attn_fwd_mfma_k<64><<<grid, NT, 0, s>>>((const uint16_t *)qkv, (uint16_t *)o, lse, Tn, H, scale);
    else attn_fwd_mfma_k<128><<<grid, NT, 0, s>>>((const uint16_t *)qkv, (uint16_t *)o, lse, Tn, H, scale);
}

void attn_bwd_mfma(hipStream_t s, const void *dO, const void *qkv, const float *lse, const float *delta, void *dqkv,
                   int64_t B, int64_t Tn, int64_t H, int64_t dh) {
    const dim3 grid((unsigned)((Tn + 127) / 128), (unsigned)(B * H));
    const float scale = 1.0f / sqrtf((float)dh);
    static bool attr_set = false;
    if (!attr_set) {       // the dK/dV kernel for head dimension 128 needs more than the default 64 KiB of LDS
        (void)hipFuncSetAttribute((const void *)attn_bwd_dkv_mfma_k<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dkv_smem<64>());
        (void)hipFuncSetAttribute((const void *)attn_bwd_dkv_mfma_k<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dkv_smem<128>());
        attr_set = true;
    }
    if (dh == 64) {
        attn_bwd_dq_mfma_k<64><<<grid, NT, 0, s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, Tn, H, scale);
        attn_bwd_dkv_mfma_k<64><<<grid, NT, dkv_smem<64>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, Tn, H, scale);
    } else {
        attn_bwd_dq_mfma_k<128><<<grid, NT, 0, s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, Tn, H, scale);
        attn_bwd_dkv_mfma_k<128><<<grid, NT, dkv_smem<128>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, Tn, H, scale);
    }
}

}  // namespace k
}  // namespace tio
