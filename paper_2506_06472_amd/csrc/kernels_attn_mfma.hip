// Causal self-attention on the matrix cores (bf16, head dimension 64 or 128), forward and backward,
// on the packed [S, 3d] q|k|v layout.
//
// Each wavefront owns 32 query rows (forward, dQ) or 32 key rows (dK/dV) and keeps their operand
// fragments in registers for the whole kernel; the other side streams through LDS in row-major tiles of
// 64 rows.  Scores are produced transposed (keys x queries in the forward and dQ kernels, queries x keys
// in the dK/dV kernel) so that in the accumulator layout of v_mfma_f32_32x32x16_bf16 the row owned by the
// wavefront is the lane index: the softmax statistics of a row live in one lane (plus one exchange with
// lane+32), and the probabilities can be fed to the second product straight from registers as its B
// operand.  The operand whose contraction index is the sequence position (V in P.V, K in dS.K, Q and dO
// in the dK/dV products) is read from the same row-major tile with the transposing LDS read
// (ds_read_b64_tr_b16), in the slot order the accumulator registers dictate: no transposed copies.
// Tiles go from global memory straight into the other half of a double LDS buffer one tile ahead (buffer
// loads with the LDS bit; rows past the end of the sequence arrive as zeros), so a tile costs one barrier and
// neither staging registers nor LDS store instructions.  The tiles are unpadded; a permutation of the 16-byte
// chunks of every row, applied through the choice of the chunk each lane fetches, keeps both kinds of
// fragment reads free of bank conflicts.  The fragments of the first products of a tile run through a small
// ring of registers a few fragments ahead of the products that use them.
// Statistics are fp32, exp2 with the 1/sqrt(dh) scale folded into the exponent; the causal mask is
// applied only on tiles that cross the diagonal; the backward pass recomputes P from the saved
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

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2(float a, float b) {
    union { bf16x2 h; uint32_t u; } c;
    c.h = __builtin_convertvector((f32x2){a, b}, bf16x2);
    return c.u;
}

// B operand of a 16-deep product from accumulator registers R0..R0+7 (the contraction index is the
// accumulator's row index: slots 0..3 = rows base+4*lhi+0..3, slots 4..7 = rows base+8+4*lhi+0..3)
template <int R0> __device__ __forceinline__ bf16x8 pack8(const floatx16 &v) {
    Frag f;
    f.u = make_uint4(pack2(v[R0], v[R0 + 1]), pack2(v[R0 + 2], v[R0 + 3]), pack2(v[R0 + 4], v[R0 + 5]), pack2(v[R0 + 6], v[R0 + 7]));
    return f.v;
}
__device__ __forceinline__ floatx16 zero16() {
    floatx16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}
// a value combined over the two halves of the wavefront (lanes i and i + 32), the same in both: v_permlane32_swap hands
// every lane the value of both halves without a trip through the LDS queue, behind which a cross-lane read would wait
__device__ __forceinline__ float max_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// row index inside a 32x32 accumulator tile of register r for lane half lhi
__device__ __forceinline__ int acc_row(int r, int lhi) { return 8 * (r >> 2) + 4 * lhi + (r & 3); }

__device__ __forceinline__ u32x4 buf_load(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
}
// descriptor over rows [0, Tn) of one head's slice: rows at or past Tn read as zero
__device__ __forceinline__ __amdgpu_buffer_rsrc_t head_rsrc(const uint16_t *base, int64_t Tn, int64_t ld, int dh) {
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)(((Tn - 1) * ld + dh) * 2), 0x00020000);
}
__device__ __forceinline__ bf16x8 buf_frag(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
    union { u32x4 u; bf16x8 v; } f;
    f.u = buf_load(rsrc, off);
    return f.v;
}

// Workgroup index -> (batch*head, block of 128 rows).  Workgroups are dealt to the 8 XCDs round-robin and
// each XCD has its own L2, so all row blocks of one head are given to one XCD (head = 8*i + xcd): the K and
// V rows of a head are then fetched into one L2 only, and reused there by the head's other row blocks.
// Returns false for the padding workgroups when the head count is not a multiple of 8.
__device__ __forceinline__ bool head_and_block(int64_t n_heads, int n_blocks, int64_t &bh, int &blk) {
    const int id = (int)blockIdx.x, xcd = id & 7, slot = id >> 3;
    bh = (int64_t)(slot / n_blocks) * 8 + xcd;
    blk = slot % n_blocks;
    return bh < n_heads;
}

// ------------------------------------------------------------------------------------------ forward
// LDS tiles of the forward kernel: [64 rows][DH] bf16 without padding, filled straight from global memory (no
// staging registers, no LDS store instructions); the 16-byte chunk c of row r sits at chunk c ^ swz(r).  K is read
// row-wise (16-byte fragments of 16 consecutive rows at one logical chunk) and V through transposing reads (32 lanes
// take 64 bytes, an aligned quad of chunks, of each of four consecutive rows); the permutation keeps both free of bank
// conflicts (the banks span 256 bytes): over the rows that share banks swz takes 16 (DH 128) or 8 (DH 64, two rows per
// 256 bytes) different values, and the quads of four consecutive rows land on different quads (DH 128:
// swz = (r%4)*4 + (r/4)%4) or on two quads in each half of the banks (DH 64: swz = ((r/2)%2)*4 + (r/4)%4).
template <int DH> __device__ __forceinline__ int swz(int r) {
    return DH == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}
// per-lane parts of the fragment addresses (element offsets into a tile), computed once per kernel: the XOR makes
// them non-additive in the contraction step, so each step has its own
template <int DH> struct TileLanes {
    static constexpr int CPR = DH / 8, KS = DH / 16, DT = DH / 32;
    int roff[KS];          // row-wise fragment of contraction step ks: row lane%32, chunk 2 ks + lane/32
    int troff[DT][2];      // transposing fragment of column block i: rows 4 (lane/32) + (lane%16)/4 (+ 8), columns by lane
    __device__ __forceinline__ TileLanes(int lane) {
        const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) roff[ks] = (l32 * CPR + ((ks * 2 + lhi) ^ swz<DH>(l32 & 15))) * 8;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int rl = 4 * lhi + ((lane & 15) >> 2) + 8 * h;
                const int chunk = 4 * i + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
                troff[i][h] = (rl * CPR + (chunk ^ swz<DH>(rl))) * 8 + 4 * (lane & 1);
            }
    }
    // A operand, rows row0 + lane%32 (row0 a multiple of 16), contraction step ks
    __device__ __forceinline__ bf16x8 row(const uint16_t *lds, int row0, int ks) const {
        Frag f;
        f.u = *reinterpret_cast<const uint4 *>(lds + row0 * DH + roff[ks]);
        return f.v;
    }
    // A operand "column 32 i + lane%32, contraction over rows r0 .. r0+15 in the slot order of pack8" (r0 a multiple of 16)
    __device__ __forceinline__ bf16x8 tr(const uint16_t *lds, int r0, int i) const {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        union { s16x4 h[2]; bf16x8 v; } f;
        f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds + r0 * DH + troff[i][0]));
        f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds + r0 * DH + troff[i][1]));
        return f.v;
    }
};
// A [64][DH] tile on its way from global memory into LDS: a wavefront-wide load fills 1 KiB of consecutive LDS bytes
// (lane i writes bytes 16 i ..), so which chunk a lane fetches decides where it lands: lane i of block b fetches, for
// row b*RPB + i/CPR, the logical chunk (i%CPR) ^ swz(row).  Rows past the sequence lie outside the descriptor and
// arrive as zeros.
template <int DH> struct DmaTile {
    static constexpr int CPR = DH / 8, RPB = 64 / CPR, BLOCKS = 64 * DH * 2 / 1024, PER = BLOCKS / (NT / 64);
    static_assert(BLOCKS % (NT / 64) == 0, "blocks divide over the wavefronts");
    static_assert(((NT / 64) * RPB) % 16 == 0, "the permutation repeats from one load of a wavefront to its next");
    uint32_t voff, step;           // byte offset of this lane's chunk in the wavefront's first block; bytes between its blocks (uniform)
    __device__ __forceinline__ DmaTile(uint32_t ld_bytes, int wave, int lane) {
        const int row = wave * RPB + lane / CPR;
        voff = (uint32_t)row * ld_bytes + (uint32_t)(((lane % CPR) ^ swz<DH>(row & 15)) * 16);
        step = __builtin_amdgcn_readfirstlane((uint32_t)((NT / 64) * RPB) * ld_bytes);
    }
    // load i of the PER that make up this wavefront's share of a tile (soff = row0 * ld_bytes, uniform): rows
    // i * (NT / 64) * RPB further down, which only moves the uniform part of the address (the scalar offset takes part
    // in the descriptor's range check like the per-lane one: checked on the hardware)
    __device__ __forceinline__ void load_one(int i, i32x4 rsrc, uint32_t soff, uint32_t lds_addr, int wave) const {
        load_to_lds_b128(rsrc, lds_addr + (uint32_t)(i * (NT / 64) + wave) * 1024u, voff, soff + (uint32_t)i * step);
    }
    // rows row0 .. row0+63 of the head behind rsrc to the tile at LDS address lds_addr
    __device__ __forceinline__ void load(i32x4 rsrc, uint32_t row0, uint32_t ld_bytes, uint32_t lds_addr, int wave) const {
        const uint32_t soff = __builtin_amdgcn_readfirstlane(row0 * ld_bytes);
#pragma unroll
        for (int i = 0; i < PER; ++i) load_one(i, rsrc, soff, lds_addr, wave);
    }
};

// Scores are produced transposed (keys x queries); a 64-key tile is handled as two groups of 32 keys.  The K
// fragments run through a ring of registers RING fragments ahead of their products: left to itself the compiler reads
// every fragment into the same registers right before its product and waits for it, sixteen exposed LDS latencies per
// tile.  Both score products are issued first; the softmax arithmetic of the first group then runs on the vector ALU
// while the matrix cores are still busy with the second group's scores, and that of the second group while they
// accumulate the first group's P.V.
template <int DH>
__global__ void __launch_bounds__(NT, 2) attn_fwd_mfma_k(const uint16_t *__restrict__ qkv, uint16_t *__restrict__ o,
                                                      float *__restrict__ lse, int64_t Bn, int64_t Tn, int64_t H, float scale) {
    constexpr int KS = DH / 16, DT = DH / 32, TE = 64 * DH, RING = 4;
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];    // [2 buffers][K tile | V tile]
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int64_t d = H * DH, ld = 3 * d;
    const uint32_t ldb = (uint32_t)(ld * 2);
    const int nblk = (int)((Tn + 127) / 128);
    int64_t bh;
    int blk;
    if (!head_and_block(Bn * H, nblk, bh, blk)) return;
    const int64_t b = bh / H, h = bh % H;
    const int q0 = (nblk - 1 - blk) * 128;                               // longest rows first
    const int q0w = q0 + wave * 32, q = q0w + l32;
    const uint16_t *qb = qkv + b * Tn * ld + h * DH;
    const __amdgpu_buffer_rsrc_t rsQ = head_rsrc(qb, Tn, ld, DH);
    const uint32_t head_bytes = (uint32_t)(((Tn - 1) * ld + DH) * 2);
    const i32x4 rsK = make_rsrc(qb + d, head_bytes), rsV = make_rsrc(qb + 2 * d, head_bytes);
    const float c = scale * LOG2E;
    const TileLanes<DH> L(lane);
    const DmaTile<DH> dma(ldb, wave, lane);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));

    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = buf_frag(rsQ, (uint32_t)q * ldb + (ks * 16 + lhi * 8) * 2);
    floatx16 oacc[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) oacc[i] = zero16();
    float m = -INFINITY, l = 0.f;                       // reference exponent (log2 domain, scaled) and sum
    const int kv_end = q0 + 128 < (int)Tn ? q0 + 128 : (int)Tn;
    const int ntiles = (kv_end + 63) / 64;

    dma.load(rsK, 0, ldb, lds0, wave);
    dma.load(rsV, 0, ldb, lds0 + TE * 2, wave);
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this wavefront's part of tile 0 has landed
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int j0 = t * 64;
        const uint16_t *Ks = smem + (t & 1) * 2 * TE, *Vs = Ks + TE;
        // Tile t+1 goes to the other buffer, free since the barrier that ended tile t-1.  Its loads are issued one at a
        // time between the score products: issued together right after the barrier, the loads of all eight wavefronts
        // of a compute unit queue up behind one another and every wavefront stalls in the issue.
        const bool more = t + 1 < ntiles;
        const uint32_t nx = lds0 + (uint32_t)((t + 1) & 1) * 2 * TE * 2;
        const uint32_t nsoff = __builtin_amdgcn_readfirstlane(((uint32_t)j0 + 64) * ldb);
        constexpr int NL = 2 * DmaTile<DH>::PER;           // K loads, then V loads
        auto next_load = [&](int i) {
            if (i < DmaTile<DH>::PER) dma.load_one(i, rsK, nsoff, nx, wave);
            else dma.load_one(i - DmaTile<DH>::PER, rsV, nsoff, nx + TE * 2, wave);
        };
        if (more && j0 > q0w + 31) {                    // this wavefront has no products here: it still loads its share
#pragma unroll
            for (int i = 0; i < NL; ++i) next_load(i);
        }
        if (j0 <= q0w + 31) {
            floatx16 s[2];
            {
                constexpr int N = 2 * KS;
                bf16x8 ring[RING];
#pragma unroll
                for (int i = 0; i < RING; ++i) ring[i] = L.row(Ks, (i / KS) * 32, i % KS);
                s[0] = zero16();
                s[1] = zero16();
#pragma unroll
                for (int idx = 0; idx < N; ++idx) {
                    s[idx / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[idx % RING], qf[idx % KS], s[idx / KS], 0, 0, 0);
                    if (idx + RING < N) ring[idx % RING] = L.row(Ks, ((idx + RING) / KS) * 32, (idx + RING) % KS);
                    if (more) {
#pragma unroll
                        for (int i = idx * NL / N; i < (idx + 1) * NL / N; ++i) next_load(i);
                    }
                }
                // pin the order: RING reads, then one product and one read in turn, then the last products
                __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
                for (int idx = 0; idx < N - RING; ++idx) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, RING, 0);
            }
            const bool diag = j0 + 63 > q0w;           // the tile crosses the diagonal of some row of this wavefront
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                if (diag) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (j0 + kt * 32 + acc_row(r, lhi) > q) s[kt][r] = -INFINITY;
                }
                // The reference exponent m only has to keep exp2(x - m) in range, it need not be the running maximum.  The
                // probabilities are first taken with the m at hand, and their sum tells whether that was good enough: only
                // when some lane's sum reaches 2^16 (or is not a number: m is still -inf in the first group of a row,
                // where key 0 is visible to every row) is the row maximum of the group computed, m raised to it, everything
                // accumulated so far rescaled and the group redone.  After the first keys that is rare, and the common
                // path has no maximum, no exchange between the lane halves and no rescale in it.
                float pr[16], psum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    pr[r] = __builtin_amdgcn_exp2f(fmaf(s[kt][r], c, -m));
                    psum += pr[r];
                }
                if (__any(!(psum < 65536.0f))) {
                    float tmax = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kt][r]);
                    tmax = max_halves(tmax) * c;
                    const float mn = fmaxf(m, tmax);
                    const float corr = __builtin_amdgcn_exp2f(m - mn);
                    l *= corr;
                    m = mn;
#pragma unroll
                    for (int i = 0; i < DT; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
                    psum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        pr[r] = __builtin_amdgcn_exp2f(fmaf(s[kt][r], c, -m));
                        psum += pr[r];
                    }
                }
                l += psum;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kt][r] = pr[r];
                const bf16x8 pk[2] = {pack8<0>(s[kt]), pack8<8>(s[kt])};
                // V fragment f of the group: keys 16 (f / DT) .. + 15, columns 32 (f % DT) .. + 31; like the K fragments
                // they run through a ring of register sets, VR products ahead
                constexpr int NPV = 2 * DT, VR = 4;
                bf16x8 vf[VR];
#pragma unroll
                for (int f = 0; f < VR; ++f) vf[f] = L.tr(Vs, kt * 32 + 16 * (f / DT), f % DT);
#pragma unroll
                for (int f = 0; f < NPV; ++f) {
                    oacc[f % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[f % VR], pk[f / DT], oacc[f % DT], 0, 0, 0);
                    if (f + VR < NPV) vf[f % VR] = L.tr(Vs, kt * 32 + 16 * ((f + VR) / DT), (f + VR) % DT);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * VR, 0);
#pragma unroll
                for (int f = 0; f < NPV - VR; ++f) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, VR, 0);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this wavefront's part of tile t+1 has landed
        __syncthreads();
    }
    l = sum_halves(l);
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
__global__ void __launch_bounds__(NT, 2) attn_bwd_dq_mfma_k(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ qkv,
                                                         const float *__restrict__ lse, const float *__restrict__ delta,
                                                         uint16_t *__restrict__ dqkv, int64_t Bn, int64_t Tn, int64_t H, float scale) {
    constexpr int KS = DH / 16, DT = DH / 32, TE = 64 * DH, RING = 4;
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];    // [2 buffers][K tile | V tile], filled as in the forward kernel
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int64_t d = H * DH, ld = 3 * d;
    const uint32_t ldb = (uint32_t)(ld * 2);
    const int nblk = (int)((Tn + 127) / 128);
    int64_t bh;
    int blk;
    if (!head_and_block(Bn * H, nblk, bh, blk)) return;
    const int64_t b = bh / H, h = bh % H;
    const int q0 = (nblk - 1 - blk) * 128;
    const int q0w = q0 + wave * 32, q = q0w + l32;
    const uint16_t *qb = qkv + b * Tn * ld + h * DH;
    const __amdgpu_buffer_rsrc_t rsQ = head_rsrc(qb, Tn, ld, DH);
    const uint32_t head_bytes = (uint32_t)(((Tn - 1) * ld + DH) * 2);
    const i32x4 rsK = make_rsrc(qb + d, head_bytes), rsV = make_rsrc(qb + 2 * d, head_bytes);
    const __amdgpu_buffer_rsrc_t rsG = head_rsrc(dO + b * Tn * d + h * DH, Tn, d, DH);
    const float c = scale * LOG2E;
    const bool live = q < Tn;
    const TileLanes<DH> L(lane);
    const DmaTile<DH> dma(ldb, wave, lane);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));

    bf16x8 qf[KS], gf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qf[ks] = buf_frag(rsQ, (uint32_t)q * ldb + (ks * 16 + lhi * 8) * 2);
        gf[ks] = buf_frag(rsG, (uint32_t)q * (uint32_t)(d * 2) + (ks * 16 + lhi * 8) * 2);
    }
    const float lse2 = live ? lse[bh * Tn + q] * LOG2E : 0.f;
    const float dl = live ? delta[bh * Tn + q] : 0.f;
    floatx16 dq[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) dq[i] = zero16();
    const int kv_end = q0 + 128 < (int)Tn ? q0 + 128 : (int)Tn;
    const int ntiles = (kv_end + 63) / 64;

    dma.load(rsK, 0, ldb, lds0, wave);
    dma.load(rsV, 0, ldb, lds0 + TE * 2, wave);
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this wavefront's part of tile 0 has landed
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int j0 = t * 64;
        const uint16_t *Ks = smem + (t & 1) * 2 * TE, *Vs = Ks + TE;
        if (t + 1 < ntiles) {                           // the other buffer is free since the barrier that ended tile t-1
            const uint32_t nx = lds0 + (uint32_t)((t + 1) & 1) * 2 * TE * 2;
            dma.load(rsK, (uint32_t)j0 + 64, ldb, nx, wave);
            dma.load(rsV, (uint32_t)j0 + 64, ldb, nx + TE * 2, wave);
        }
        if (j0 <= q0w + 31) {
            floatx16 s[2], dp[2];
            {
                // S = K.Q^T and dP = V.dO^T for both key groups; the K and V fragments run RING ahead of their products
                constexpr int N = 4 * KS;
                bf16x8 ring[RING];
                auto frag = [&](int idx) { return L.row((idx & 1) ? Vs : Ks, (idx / (2 * KS)) * 32, (idx / 2) % KS); };
#pragma unroll
                for (int i = 0; i < RING; ++i) ring[i] = frag(i);
                s[0] = zero16(); s[1] = zero16(); dp[0] = zero16(); dp[1] = zero16();
#pragma unroll
                for (int idx = 0; idx < N; ++idx) {
                    const int kt = idx / (2 * KS), ks = (idx / 2) % KS;
                    if (idx & 1) dp[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[idx % RING], gf[ks], dp[kt], 0, 0, 0);
                    else s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[idx % RING], qf[ks], s[kt], 0, 0, 0);
                    if (idx + RING < N) ring[idx % RING] = frag(idx + RING);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
                for (int idx = 0; idx < N - RING; ++idx) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, RING, 0);
            }
            const bool diag = j0 + 63 > q0w;
            // per group of 32 keys: the element-wise part of one group overlaps the other group's products
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = __builtin_amdgcn_exp2f(fmaf(s[kt][r], c, -lse2));
                    if (diag && j0 + kt * 32 + acc_row(r, lhi) > q) p = 0.0f;
                    s[kt][r] = p * (dp[kt][r] - dl);          // the 1/sqrt(dh) factor is applied once, to the sums
                }
                const bf16x8 d0 = pack8<0>(s[kt]), d1 = pack8<8>(s[kt]);
#pragma unroll
                for (int i = 0; i < DT; ++i) {
                    dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L.tr(Ks, kt * 32, i), d0, dq[i], 0, 0, 0);
                    dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L.tr(Ks, kt * 32 + 16, i), d1, dq[i], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this wavefront's part of tile t+1 has landed
        __syncthreads();
    }
    if (live) {
        uint16_t *orow = dqkv + (b * Tn + q) * ld + h * DH;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                w.x = pack2(dq[i][4 * g] * scale, dq[i][4 * g + 1] * scale);
                w.y = pack2(dq[i][4 * g + 2] * scale, dq[i][4 * g + 3] * scale);
                *reinterpret_cast<uint2 *>(orow + i * 32 + 8 * g + 4 * lhi) = w;
            }
    }
}

// ------------------------------------------------------------------------------------------ dK, dV
// MODE 0 produces both gradients in one pass.  With head dimension 128 the two accumulators, the K and V
// fragments and the prefetch registers do not fit the 256 registers that two wavefronts per SIMD allow, so
// there the work is split: MODE 1 computes dV only (needs S), MODE 2 dK only (needs S and dP).
template <int DH, int MODE>
__global__ void __launch_bounds__(NT, 2) attn_bwd_dkv_mfma_k(const uint16_t *__restrict__ dO, const uint16_t *__restrict__ qkv,
                                                          const float *__restrict__ lse, const float *__restrict__ delta,
                                                          uint16_t *__restrict__ dqkv, int64_t Bn, int64_t Tn, int64_t H, float scale) {
    constexpr int KS = DH / 16, DT = DH / 32, TE = 64 * DH, RING = 4;
    constexpr int BUF = 2 * TE;                                          // Q tile | dO tile, filled as in the forward kernel
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];    // [2 buffers][Q | dO], then [2][64 lse | 64 delta] floats
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int64_t d = H * DH, ld = 3 * d;
    const uint32_t ldb = (uint32_t)(ld * 2), ldg = (uint32_t)(d * 2);
    int64_t bh;
    int blk;
    if (!head_and_block(Bn * H, (int)((Tn + 127) / 128), bh, blk)) return;
    const int64_t b = bh / H, h = bh % H;
    const int kv0 = blk * 128;                                            // earliest keys see the most queries: first
    const int kv0w = kv0 + wave * 32, kv = kv0w + l32;
    const uint16_t *qb = qkv + b * Tn * ld + h * DH;
    const __amdgpu_buffer_rsrc_t rsK = head_rsrc(qb + d, Tn, ld, DH), rsV = head_rsrc(qb + 2 * d, Tn, ld, DH);
    const i32x4 rsQ = make_rsrc(qb, (uint32_t)(((Tn - 1) * ld + DH) * 2));
    const i32x4 rsG = make_rsrc(dO + b * Tn * d + h * DH, (uint32_t)(((Tn - 1) * d + DH) * 2));
    const float c = scale * LOG2E;
    const bool live = kv < Tn;
    const TileLanes<DH> L(lane);
    const DmaTile<DH> dmaQ(ldb, wave, lane), dmaG(ldg, wave, lane);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    constexpr bool DO_DV = MODE != 2, DO_DK = MODE != 1;
    constexpr int NDK = DO_DK ? DT : 1, NDV = DO_DV ? DT : 1, NVF = DO_DK ? KS : 1;

    bf16x8 kf[KS], vf[NVF];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        kf[ks] = buf_frag(rsK, (uint32_t)kv * ldb + (ks * 16 + lhi * 8) * 2);
        if (DO_DK) vf[ks] = buf_frag(rsV, (uint32_t)kv * ldb + (ks * 16 + lhi * 8) * 2);
    }
    floatx16 dk[NDK], dv[NDV];
#pragma unroll
    for (int i = 0; i < NDK; ++i) dk[i] = zero16();
#pragma unroll
    for (int i = 0; i < NDV; ++i) dv[i] = zero16();
    const int ntiles = ((int)Tn - kv0 + 63) / 64;

    float st_l = 0.f, st_d = 0.f;                       // statistics of row i0 + tid (threads 0..63), one tile ahead
    float *stats = reinterpret_cast<float *>(smem + 2 * BUF);
    auto load_stats = [&](int i0) {
        if (tid < 64) {
            const bool ok = i0 + tid < Tn;
            st_l = ok ? lse[bh * Tn + i0 + tid] * LOG2E : 0.f;
            st_d = ok ? delta[bh * Tn + i0 + tid] : 0.f;
        }
    };
    auto store_stats = [&](int buf) {
        if (tid < 64) {
            stats[buf * 128 + tid] = st_l;
            stats[buf * 128 + 64 + tid] = st_d;
        }
    };
    auto load_tile = [&](int i0, int buf) {
        const uint32_t at = lds0 + (uint32_t)buf * BUF * 2;
        dmaQ.load(rsQ, (uint32_t)i0, ldb, at, wave);
        dmaG.load(rsG, (uint32_t)i0, ldg, at + TE * 2, wave);
    };
    load_tile(kv0, 0);
    load_stats(kv0);
    store_stats(0);
    if (ntiles > 1) load_stats(kv0 + 64);
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this wavefront's part of tile 0 has landed
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int i0 = kv0 + t * 64;
        const uint16_t *Qs = smem + (t & 1) * BUF, *Gs = Qs + TE;
        const float *L2s = stats + (t & 1) * 128, *Ds = L2s + 64;
        if (t + 1 < ntiles) {                           // the other buffer is free since the barrier that ended tile t-1
            // The statistics fetched a tile ago go to LDS before the tile loads are issued: the write waits for every
            // outstanding vector memory operation of the wavefront, and behind the tile loads that would be their
            // whole latency, at the start of every tile.
            store_stats((t + 1) & 1);
            load_tile(i0 + 64, (t + 1) & 1);
            if (t + 2 < ntiles) load_stats(i0 + 128);
        }
        if (i0 + 63 >= kv0w) {
            // masking is needed where some query of the tile precedes some key of this wavefront, and for
            // rows past the end of the sequence (zero Q and dO, but a zero statistic too)
            const bool edge = i0 < kv0w + 31 || i0 + 64 > (int)Tn;
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                floatx16 s = zero16(), dp = zero16();
                {
                    // S^T = Q.K^T (and dP^T = dO.V^T); the Q and dO fragments run RING ahead of their products
                    constexpr int PERK = DO_DK ? 2 : 1, N = PERK * KS;
                    bf16x8 ring[RING];
                    auto frag = [&](int idx) { return L.row((PERK == 2 && (idx & 1)) ? Gs : Qs, qt * 32, idx / PERK); };
#pragma unroll
                    for (int i = 0; i < RING; ++i) ring[i] = frag(i);
#pragma unroll
                    for (int idx = 0; idx < N; ++idx) {
                        const int ks = idx / PERK;
                        if (PERK == 2 && (idx & 1)) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[idx % RING], vf[ks % NVF], dp, 0, 0, 0);
                        else s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[idx % RING], kf[ks], s, 0, 0, 0);
                        if (idx + RING < N) ring[idx % RING] = frag(idx + RING);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x100, RING, 0);
#pragma unroll
                    for (int idx = 0; idx < N - RING; ++idx) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, RING, 0);
                }
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    // rows 8*r4 + 4*lhi + 0..3 of this 32-row group: their statistics are 16 contiguous bytes
                    const int ql = qt * 32 + 8 * r4 + 4 * lhi;
                    const float4 l4 = *reinterpret_cast<const float4 *>(L2s + ql);
                    const float4 d4 = DO_DK ? *reinterpret_cast<const float4 *>(Ds + ql) : make_float4(0.f, 0.f, 0.f, 0.f);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * r4 + e;
                        float p = __builtin_amdgcn_exp2f(fmaf(s[r], c, -lv[e]));
                        if (edge && (i0 + ql + e < kv || i0 + ql + e >= (int)Tn)) p = 0.0f;
                        if (DO_DK) dp[r] = p * (dp[r] - dvv[e]);     // the 1/sqrt(dh) factor is applied once, to the sums
                        s[r] = p;
                    }
                }
                if (DO_DV) {
                    const bf16x8 p0 = pack8<0>(s), p1 = pack8<8>(s);
#pragma unroll
                    for (int i = 0; i < NDV; ++i) {
                        dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L.tr(Gs, qt * 32, i), p0, dv[i], 0, 0, 0);
                        dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L.tr(Gs, qt * 32 + 16, i), p1, dv[i], 0, 0, 0);
                    }
                }
                if (DO_DK) {
                    const bf16x8 d0 = pack8<0>(dp), d1 = pack8<8>(dp);
#pragma unroll
                    for (int i = 0; i < NDK; ++i) {
                        dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L.tr(Qs, qt * 32, i), d0, dk[i], 0, 0, 0);
                        dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(L.tr(Qs, qt * 32 + 16, i), d1, dk[i], 0, 0, 0);
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this wavefront's part of tile t+1 has landed
        __syncthreads();
    }
    if (live) {
        uint16_t *krow = dqkv + (b * Tn + kv) * ld + d + h * DH, *vrow = krow + d;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w;
                if (DO_DK) {
                    w.x = pack2(dk[i % NDK][4 * g] * scale, dk[i % NDK][4 * g + 1] * scale);
                    w.y = pack2(dk[i % NDK][4 * g + 2] * scale, dk[i % NDK][4 * g + 3] * scale);
                    *reinterpret_cast<uint2 *>(krow + i * 32 + 8 * g + 4 * lhi) = w;
                }
                if (DO_DV) {
                    w.x = pack2(dv[i % NDV][4 * g], dv[i % NDV][4 * g + 1]);
                    w.y = pack2(dv[i % NDV][4 * g + 2], dv[i % NDV][4 * g + 3]);
                    *reinterpret_cast<uint2 *>(vrow + i * 32 + 8 * g + 4 * lhi) = w;
                }
            }
    }
}

template <int DH> constexpr size_t kv_smem() { return (size_t)2 * 2 * 64 * DH * 2; }       // two buffers of two tiles
template <int DH> constexpr size_t dkv_smem() { return (size_t)2 * 2 * 64 * DH * 2 + 2 * 128 * 4; }      // tiles, then statistics

// 32-bit buffer offsets: one head's rows must span less than 2 GiB
bool fits(int64_t Tn, int64_t H, int64_t dh) { return (Tn + 192) * 3 * H * dh * 2 < ((int64_t)1 << 31); }

}  // namespace

bool attn_mfma_supported(int dtype, int64_t Tn, int64_t H, int64_t dh) {
    return dtype == TIO_PREC_BF16 && (dh == 64 || dh == 128) && fits(Tn, H, dh);
}

void attn_fwd_mfma(hipStream_t s, const void *qkv, void *o, float *lse, int64_t B, int64_t Tn, int64_t H, int64_t dh) {
    const dim3 grid((unsigned)(((Tn + 127) / 128) * ((B * H + 7) / 8) * 8));
    const float scale = 1.0f / sqrtf((float)dh);
    static bool attr_set = false;
    if (!attr_set) {       // head dimension 128 needs more than the default 64 KiB of LDS
        (void)hipFuncSetAttribute((const void *)attn_fwd_mfma_k<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kv_smem<128>());
        attr_set = true;
    }
    if (dh == 64) attn_fwd_mfma_k<64><<<grid, NT, kv_smem<64>(), s>>>((const uint16_t *)qkv, (uint16_t *)o, lse, B, Tn, H, scale);
    else attn_fwd_mfma_k<128><<<grid, NT, kv_smem<128>(), s>>>((const uint16_t *)qkv, (uint16_t *)o, lse, B, Tn, H, scale);
}

void attn_bwd_mfma(hipStream_t s, const void *dO, const void *qkv, const float *lse, const float *delta, void *dqkv,
                   int64_t B, int64_t Tn, int64_t H, int64_t dh) {
    const dim3 grid((unsigned)(((Tn + 127) / 128) * ((B * H + 7) / 8) * 8));
    const float scale = 1.0f / sqrtf((float)dh);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)attn_bwd_dq_mfma_k<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kv_smem<128>());
        (void)hipFuncSetAttribute((const void *)attn_bwd_dkv_mfma_k<128, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dkv_smem<128>());
        (void)hipFuncSetAttribute((const void *)attn_bwd_dkv_mfma_k<128, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dkv_smem<128>());
        attr_set = true;
    }
    if (dh == 64) {
        attn_bwd_dq_mfma_k<64><<<grid, NT, kv_smem<64>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, B, Tn, H, scale);
        attn_bwd_dkv_mfma_k<64, 0><<<grid, NT, dkv_smem<64>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, B, Tn, H, scale);
    } else {
        attn_bwd_dq_mfma_k<128><<<grid, NT, kv_smem<128>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, B, Tn, H, scale);
        attn_bwd_dkv_mfma_k<128, 1><<<grid, NT, dkv_smem<128>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, B, Tn, H, scale);
        attn_bwd_dkv_mfma_k<128, 2><<<grid, NT, dkv_smem<128>(), s>>>((const uint16_t *)dO, (const uint16_t *)qkv, lse, delta, (uint16_t *)dqkv, B, Tn, H, scale);
    }
}

}  // namespace k
}  // namespace tio
