// bf16 MFMA GEMM for gfx950 whose operand tiles go from global memory straight into LDS
// (buffer loads with the LDS bit): C[M,N] = A . B^T (+bias) (+residual), fp32 accumulate.
//
//  * no staging registers and no LDS store instructions: a wavefront-wide load instruction fills 1 KiB of
//    consecutive LDS bytes (lane i writes bytes 16 i .. 16 i + 15); which 16-byte chunk of the operand a lane
//    fetches is chosen so that the LDS image is the bank-swizzled tile the fragment reads expect;
//  * an operand tile is ROWS x 64 bf16 = ROWS * 128 bytes without padding.
//      contraction index contiguous ("k-contig"): LDS row r holds the eight chunks of operand row r, chunk c at
//      slot c ^ ((r >> 1) & 7): the sixteen rows read together by a quarter wavefront fall into sixteen
//      different 16-byte bank groups;
//      contraction index slow ("k-major"): LDS row k holds ROWS elements, chunk c at slot c ^ ((k & 3) << 2):
//      the four k-rows a transposing read touches together fall into different 64-byte bank groups, and
//      the 32 consecutive bytes four lanes read stay consecutive;
//  * two stages in LDS; the loads of tile t+2 are issued right after the barrier that retires tile t, so they have
//    a whole tile of MFMAs to land; MFMA fragments are double-buffered in registers across contraction steps and
//    across the barrier.
#include "../../include/teraio.h"
#include "device_common.h"
#include "kernels.h"
#include "mfma_tiles.h"

namespace tio {
namespace k {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int ROWS, int BK, int NT, bool KM> struct DlOperand;

// ---- contraction index contiguous
template <int ROWS, int BK, int NT> struct DlOperand<ROWS, BK, NT, false> {
    static_assert(BK == 64, "one LDS row is eight 16-byte chunks");
    static constexpr int BYTES = ROWS * 128;
    static constexpr int BLOCKS = BYTES / 1024, NW = NT / 64, PER = BLOCKS / NW;     // 1 KiB blocks per wavefront
    static_assert(BLOCKS % NW == 0, "blocks divide over the wavefronts");
    uint32_t voff[PER];
    __device__ __forceinline__ void init(int64_t ld, int rows_valid, int kvalid, int wave, int lane) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int b = i * NW + wave, r = b * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
            voff[i] = (r < rows_valid && c * 8 < kvalid) ? (uint32_t)(((int64_t)r * ld + c * 8) * 2) : DL_OOB;
        }
    }
    static __device__ __forceinline__ uint32_t tile_step(int64_t) { return BK * 2; }
    __device__ __forceinline__ void load(i32x4 rsrc, uint32_t kb, uint32_t stage, int wave) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) load_to_lds_b128(rsrc, stage + (i * NW + wave) * 1024, voff[i], kb);
    }
    __device__ __forceinline__ void load_one(int i, i32x4 rsrc, uint32_t kb, uint32_t stage, int wave) const {
        load_to_lds_b128(rsrc, stage + (i * NW + wave) * 1024, voff[i], kb);
    }
    // fragments: lane (l32, lhi) reads chunk 2 ks + lhi of row row0 + sub*32 + l32 (row0 a multiple of 32)
    uint32_t foff[BK / 16];
    __device__ __forceinline__ void init_frag(int row0, int lane) {
        const int l32 = lane & 31, lhi = lane >> 5, x = (l32 >> 1) & 7;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) foff[ks] = (uint32_t)((row0 + l32) * 128 + (((ks * 2 + lhi) ^ x) << 4));
    }
    __device__ __forceinline__ bf16x8 frag(const unsigned char *stage, int sub, int ks) const {
        Frag f;
        f.u = *reinterpret_cast<const uint4 *>(stage + foff[ks] + sub * 4096);
        return f.v;
    }
    template <int TPR> static __device__ __forceinline__ float row_partial(const unsigned char *stage, int row, int part) {
        float s = 0.f;
        const int x = (row >> 1) & 7;
#pragma unroll
        for (int c = 0; c < 8 / TPR; ++c) {
            const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * 128 + (((part * (8 / TPR) + c) ^ x) << 4));
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) s += __uint_as_float(w[e] << 16) + __uint_as_float(w[e] & 0xffff0000u);
        }
        return s;
    }
};

// ---- contraction index slow: LDS row k = ROWS elements
template <int ROWS, int BK, int NT> struct DlOperand<ROWS, BK, NT, true> {
    static constexpr int BYTES = ROWS * BK * 2;
    static constexpr int CPK = ROWS / 8;                        // chunks per k-row
    static constexpr int KPB = 64 / CPK;                        // k-rows per 1 KiB block
    static constexpr int BLOCKS = BYTES / 1024, NW = NT / 64, PER = BLOCKS / NW;
    static_assert(BLOCKS % NW == 0 && CPK >= 16 && 64 % CPK == 0, "blocks divide over the wavefronts");
    uint32_t voff[PER];
    __device__ __forceinline__ void init(int64_t ld, int rows_valid, int kvalid, int wave, int lane) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int b = i * NW + wave, kk = b * KPB + lane / CPK, c = (lane % CPK) ^ ((kk & 3) << 2);
            voff[i] = (c * 8 < rows_valid && kk < kvalid) ? (uint32_t)(((int64_t)kk * ld + c * 8) * 2) : DL_OOB;
        }
    }
    static __device__ __forceinline__ uint32_t tile_step(int64_t ld) { return (uint32_t)(BK * ld * 2); }
    __device__ __forceinline__ void load(i32x4 rsrc, uint32_t kb, uint32_t stage, int wave) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) load_to_lds_b128(rsrc, stage + (i * NW + wave) * 1024, voff[i], kb);
    }
    __device__ __forceinline__ void load_one(int i, i32x4 rsrc, uint32_t kb, uint32_t stage, int wave) const {
        load_to_lds_b128(rsrc, stage + (i * NW + wave) * 1024, voff[i], kb);
    }
    // transposing read: within 16 lanes, lanes 4j..4j+3 address k-row j (32 consecutive bytes); lane i receives
    // column i of four consecutive k
    static constexpr int SUBS = ROWS / 32 > 4 ? 4 : ROWS / 32;
    uint32_t foff[4];                                           // per 32-row group of the wavefront's tile
    __device__ __forceinline__ void init_frag(int row0, int lane) {
        const int kk = (lane >> 5) * 8 + ((lane & 15) >> 2);
#pragma unroll
        for (int sub = 0; sub < 4; ++sub) {
            const int col = row0 + sub * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
            const int c = (col >> 3) ^ ((kk & 3) << 2);
            foff[sub] = (uint32_t)(kk * (ROWS * 2) + c * 16 + (col & 7) * 2);
        }
    }
    __device__ __forceinline__ bf16x8 frag(const unsigned char *stage, int sub, int ks) const {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const unsigned char *p = stage + foff[sub] + ks * 16 * (ROWS * 2);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * (ROWS * 2)));
        union { s16x4 h[2]; bf16x8 v; } f;
        f.h[0] = lo;
        f.h[1] = hi;
        return f.v;
    }
    template <int TPR> static __device__ __forceinline__ float row_partial(const unsigned char *stage, int row, int part) {
        float s = 0.f;
#pragma unroll 8
        for (int j = 0; j < BK / TPR; ++j) {
            const int kk = part * (BK / TPR) + j;
            const int c = (row >> 3) ^ ((kk & 3) << 2);
            s += bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(stage + kk * (ROWS * 2) + c * 16 + (row & 7) * 2));
        }
        return s;
    }
};

template <int BM, int BN, int BK, int WGM, int WGN, bool AKM, bool BKM>
__global__ void __launch_bounds__(WGM *WGN * 64)
    gemm_bf16_dl_k(const uint16_t *__restrict__ A, int64_t lda, const uint16_t *__restrict__ B, int64_t ldb,
                   const uint16_t *__restrict__ bias, const uint16_t *__restrict__ resid, int64_t ldr,
                   uint16_t *__restrict__ C, int64_t ldc, int64_t M, int64_t N, int64_t K, int tiles_m, int tiles_n,
                   uint16_t *__restrict__ rowsum, float *__restrict__ ws, int64_t k_chunk, int rowsum_acc, int xsplits) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int TPR = NT / BM;
    static_assert(NT % BM == 0 && (TPR & (TPR - 1)) == 0 && TPR <= 8, "row-sum mapping");
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32, KS = BK / 16;
    static_assert(KS % 2 == 0 && TM <= 4 && TN <= 4, "fragment double buffering needs an even number of contraction steps");
    constexpr int NREADS = TM * (AKM ? 2 : 1) + TN * (BKM ? 2 : 1);     // LDS read instructions per contraction step
    using OpA = DlOperand<BM, BK, NT, AKM>;
    using OpB = DlOperand<BN, BK, NT, BKM>;
    constexpr int STAGE = OpA::BYTES + OpB::BYTES;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_dl[];

    const int tid = threadIdx.x;
    const int total_tiles = tiles_m * tiles_n;
    int split, nsplit, bid;
    if (xsplits) {
        const int x = (int)(blockIdx.x % 8), i = (int)(blockIdx.x / 8);
        const int parts = 8 / xsplits, chunk = (total_tiles + parts - 1) / parts;
        nsplit = xsplits;
        split = x % xsplits;
        if (i >= chunk) return;
        bid = (x / xsplits) * chunk + i;
    } else {
        nsplit = (int)gridDim.y;
        split = (int)blockIdx.y;
        bid = (int)(blockIdx.x % 8) * ((total_tiles + 7) / 8) + (int)(blockIdx.x / 8);
    }
    if (bid >= total_tiles) return;
    // consecutive workgroups walk down GROUP tile rows before moving to the next tile column; products with very many tile
    // rows (weight gradients of the wide layers) do better with the narrower band (measured: +3..5 % there, -2 % elsewhere)
    const int GROUP = tiles_m > 64 ? 4 : 8;
    const int per_group = GROUP * tiles_n;
    const int g = bid / per_group;
    const int gm0 = g * GROUP;
    const int gsz = tiles_m - gm0 < GROUP ? tiles_m - gm0 : GROUP;
    const int tm = gm0 + (bid % per_group) % gsz;
    const int tn = (bid % per_group) / gsz;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;

    const int64_t kbeg = (int64_t)split * k_chunk;
    const int64_t kend = (ws != nullptr && kbeg + k_chunk < K) ? kbeg + k_chunk : K;
    const int kspan = kend > kbeg ? (int)(kend - kbeg) : 0;
    const int nkf = kspan / BK, rem = kspan % BK, nk = nkf + (rem ? 1 : 0);

    const int rows_a = (int)(M - m0 < BM ? M - m0 : BM), rows_b = (int)(N - n0 < BN ? N - n0 : BN);
    const uint16_t *baseA = AKM ? A + kbeg * lda + m0 : A + m0 * lda + kbeg;
    const uint16_t *baseB = BKM ? B + kbeg * ldb + n0 : B + n0 * ldb + kbeg;
    const int k8 = (kspan + 7) / 8 * 8;
    const int64_t recA = kspan == 0 ? 0 : AKM ? ((int64_t)(kspan - 1) * lda + (rows_a + 7) / 8 * 8) * 2 : ((int64_t)(rows_a - 1) * lda + k8) * 2;
    const int64_t recB = kspan == 0 ? 0 : BKM ? ((int64_t)(kspan - 1) * ldb + (rows_b + 7) / 8 * 8) * 2 : ((int64_t)(rows_b - 1) * ldb + k8) * 2;
    const i32x4 rsA = make_rsrc(baseA, (uint32_t)recA), rsB = make_rsrc(baseB, (uint32_t)recB);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem_dl));
    const uint32_t stepA = OpA::tile_step(lda), stepB = OpB::tile_step(ldb);

    OpA oa;
    OpB ob;
    oa.init(lda, rows_a, BK, wave, lane);
    ob.init(ldb, rows_b, BK, wave, lane);
    oa.init_frag(wm * WM, lane);
    ob.init_frag(wn * WN, lane);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    auto load_tile = [&](int kt, int buf) {          // kt < nk
        const uint32_t st = lds0 + buf * STAGE;
        if (kt < nkf) {
            oa.load(rsA, (uint32_t)kt * stepA, st, wave);
            ob.load(rsB, (uint32_t)kt * stepB, st + OpA::BYTES, wave);
        } else {                                     // the last, partial tile: chunks beyond the contraction read as zero
            OpA ta;
            OpB tb;
            ta.init(lda, rows_a, rem, wave, lane);
            tb.init(ldb, rows_b, rem, wave, lane);
            ta.load(rsA, (uint32_t)kt * stepA, st, wave);
            tb.load(rsB, (uint32_t)kt * stepB, st + OpA::BYTES, wave);
        }
    };

    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int set, int buf, int ks) {
        const unsigned char *As = smem_dl + buf * STAGE, *Bs = As + OpA::BYTES;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[set][i] = oa.frag(As, i, ks);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[set][j] = ob.frag(Bs, j, ks);
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
    };

    const bool do_rowsum = rowsum != nullptr && tn == 0;
    float rsum = 0.f;

    // prologue: tiles 0 and 1 on their way, tile 0 landed, fragments of its step 0 in registers
    if (nk > 0) load_tile(0, 0);
    if (nk > 1) load_tile(1, 1);
    if (nk > 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (OpA::PER + OpB::PER));      // vmcnt: tile 1's loads may be outstanding
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_s_barrier();
    if (nk > 0) read_frags(0, 0, 0);

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1, nxt = cur ^ 1;
        if (do_rowsum) rsum += OpA::template row_partial<TPR>(smem_dl + cur * STAGE, tid / TPR, tid % TPR);
#pragma unroll
        for (int ks = 0; ks + 1 < KS; ++ks) {
            read_frags((ks + 1) & 1, cur, ks + 1);
            mfmas(ks & 1);
            // one MFMA, two reads, one MFMA, ...: the reads of the next step are issued under the first MFMAs of this one
#pragma unroll
            for (int q = 0; q < NREADS / 2; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - NREADS / 2, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // tile kt+1 (issued a tile ago) has landed for this wavefront; after the barrier it has landed for all, and
        // nobody reads stage `cur` any more
        __builtin_amdgcn_s_waitcnt(0x0070);          // vmcnt(0) lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        if (kt + 1 < nk) read_frags(0, nxt, 0);
        // the loads of tile kt+2 go out one by one between the MFMAs of the last step
        const bool full = kt + 2 < nkf;
        if (!full && kt + 2 < nk) load_tile(kt + 2, cur);
        {
            const uint32_t st = lds0 + cur * STAGE;
            const uint32_t kbA = full ? (uint32_t)(kt + 2) * stepA : DL_OOB, kbB = full ? (uint32_t)(kt + 2) * stepB : DL_OOB;
#pragma unroll
            for (int q = 0; q < TM * TN; ++q) {
                const int i = q / TN, j = q % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[(KS - 1) & 1][j], fa[(KS - 1) & 1][i], acc[i][j], 0, 0, 0);
                constexpr int NL = OpA::PER + OpB::PER;
                if (full) {
#pragma unroll
                    for (int l = q * NL / (TM * TN); l < (q + 1) * NL / (TM * TN); ++l) {
                        if (l < OpA::PER) oa.load_one(l, rsA, kbA, st, wave);
                        else ob.load_one(l - OpA::PER, rsB, kbB, st + OpA::BYTES, wave);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    if (do_rowsum) {
#pragma unroll
        for (int o = 1; o < TPR; o <<= 1) rsum += __shfl_xor(rsum, o, 64);
        const int64_t m = m0 + tid / TPR;
        if (tid % TPR == 0 && m < M) {
            if (ws) ws[(int64_t)nsplit * M * N + (int64_t)split * M + m] = rsum;
            else rowsum[m] = (uint16_t)f32_to_bf16_bits(rsum + (rowsum_acc ? bf16_bits_to_f32(rowsum[m]) : 0.f));
        }
    }
    // epilogue through LDS, 32 rows of a wavefront's tile at a time as fp32 (both stages are free: the last barrier of
    // the loop came after every fragment read)
    {
        constexpr int SPF = WN + 4, CPR = WN / 8, PASSES = 32 * CPR / 64;
        static_assert((32 * CPR) % 64 == 0, "a 32-row block is a whole number of wavefront passes");
        const bool wide = (ldc % 8 == 0) && (resid == nullptr || ldr % 8 == 0);
        static_assert((size_t)2 * STAGE >= (size_t)WGM * WGN * 32 * SPF * 4, "the staging blocks fit the two stages");
        float *stage = reinterpret_cast<float *>(smem_dl) + wave * (32 * SPF);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4 *>(stage + l32 * SPF + j * 32 + q * 8 + lhi * 4) =
                        make_float4(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int c = p * 64 + lane, row = c / CPR, ch = c % CPR;
                const float4 x0 = *reinterpret_cast<const float4 *>(stage + row * SPF + ch * 8);
                const float4 x1 = *reinterpret_cast<const float4 *>(stage + row * SPF + ch * 8 + 4);
                const int64_t m = m0 + wm * WM + i * 32 + row, n = n0 + wn * WN + ch * 8;
                if (m >= M || n >= N) continue;
                if (ws) {
                    float *dst = ws + ((int64_t)split * M + m) * N + n;
                    *reinterpret_cast<float4 *>(dst) = x0;
                    if (n + 4 < N) *reinterpret_cast<float4 *>(dst + 4) = x1;
                    continue;
                }
                float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                if (n + 8 <= N && wide) {
                    if (bias) {
                        const uint4 t = *reinterpret_cast<const uint4 *>(bias + n);
                        const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(u[e] << 16); v[2 * e + 1] += __uint_as_float(u[e] & 0xffff0000u); }
                    }
                    if (resid) {
                        const uint4 t = *reinterpret_cast<const uint4 *>(resid + m * ldr + n);
                        const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(u[e] << 16); v[2 * e + 1] += __uint_as_float(u[e] & 0xffff0000u); }
                    }
                    uint4 o;
                    o.x = pack_bf16x2(v[0], v[1]);
                    o.y = pack_bf16x2(v[2], v[3]);
                    o.z = pack_bf16x2(v[4], v[5]);
                    o.w = pack_bf16x2(v[6], v[7]);
                    *reinterpret_cast<uint4 *>(C + m * ldc + n) = o;
                } else {
                    for (int e = 0; e < 8 && n + e < N; ++e) {
                        float x = v[e];
                        if (bias) x += bf16_bits_to_f32(bias[n + e]);
                        if (resid) x += bf16_bits_to_f32(resid[m * ldr + n + e]);
                        C[m * ldc + n + e] = (uint16_t)f32_to_bf16_bits(x);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

#define TIO_DL_INSTANCE(BM, BN, WGM, WGN, AKM, BKM)                                                                         \
    template __global__ void gemm_bf16_dl_k<BM, BN, 64, WGM, WGN, AKM, BKM>(                                                \
        const uint16_t *, int64_t, const uint16_t *, int64_t, const uint16_t *, const uint16_t *, int64_t, uint16_t *, int64_t, \
        int64_t, int64_t, int64_t, int, int, uint16_t *, float *, int64_t, int, int);
TIO_DL_INSTANCE(256, 256, 2, 4, false, false) TIO_DL_INSTANCE(256, 256, 2, 4, false, true)
TIO_DL_INSTANCE(256, 256, 2, 4, true, true) TIO_DL_INSTANCE(256, 256, 2, 4, true, false)
TIO_DL_INSTANCE(128, 128, 2, 2, false, false) TIO_DL_INSTANCE(128, 128, 2, 2, false, true)
TIO_DL_INSTANCE(128, 128, 2, 2, true, true) TIO_DL_INSTANCE(128, 128, 2, 2, true, false)
#undef TIO_DL_INSTANCE

template <int BM, int BN, int BK, int WGM, int WGN>
bool launch_dl(hipStream_t s, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
               const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr, void *C, int64_t ldc,
               void *rowsum, float *ws, int splits, bool rowsum_acc) {
    if (K % 8) return false;                 // a partly valid 16-byte chunk cannot be masked on its way into LDS
    const int64_t k_chunk = splits > 1 ? ((K + splits - 1) / splits + BK - 1) / BK * BK : K;
    const int64_t kspan = splits > 1 ? k_chunk : K;
    const int64_t spanA = a_km ? (kspan + 3 * BK) * lda * 2 : ((int64_t)BM * lda + kspan + 3 * BK) * 2;
    const int64_t spanB = b_km ? (kspan + 3 * BK) * ldb * 2 : ((int64_t)BN * ldb + kspan + 3 * BK) * 2;
    constexpr int64_t LIMIT = (int64_t)1 << 30;
    if (spanA >= LIMIT || spanB >= LIMIT) return false;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    const int tiles = tiles_m * tiles_n;
    const int xsplits = (splits == 2 || splits == 4 || splits == 8) ? splits : 0;
    const dim3 grid = xsplits ? dim3((unsigned)(8 * ((tiles + 8 / xsplits - 1) / (8 / xsplits))))
                              : dim3((unsigned)(8 * ((tiles + 7) / 8)), (unsigned)(splits > 1 ? splits : 1));
    const dim3 block(WGM * WGN * 64);
    constexpr size_t lds = (size_t)2 * (BM + BN) * BK * 2;
    static bool attr_done = false;
    if (!attr_done) {
        (void)hipFuncSetAttribute((const void *)gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        (void)hipFuncSetAttribute((const void *)gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_done = true;
    }
#define TIO_GEMM_ARGS (const uint16_t *)A, lda, (const uint16_t *)B, ldb, (const uint16_t *)bias, (const uint16_t *)resid, ldr, \
                      (uint16_t *)C, ldc, M, N, K, tiles_m, tiles_n, (uint16_t *)rowsum, ws, k_chunk, (int)rowsum_acc, xsplits
    if (!a_km && !b_km) gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, false, false><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else if (!a_km && b_km) gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, false, true><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else if (a_km && b_km) gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, true, true><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
    else gemm_bf16_dl_k<BM, BN, BK, WGM, WGN, true, false><<<grid, block, lds, s>>>(TIO_GEMM_ARGS);
#undef TIO_GEMM_ARGS
    return true;
}

}  // namespace

bool gemm_bf16_direct(hipStream_t s, int cfg, bool a_km, bool b_km, int64_t M, int64_t N, int64_t K, const void *A,
                      int64_t lda, const void *B, int64_t ldb, const void *bias, const void *resid, int64_t ldr,
                      void *C, int64_t ldc, void *rowsum, float *ws, int splits, bool rowsum_accumulate) {
#define TIO_P(BM, BN, BK, WGM, WGN) launch_dl<BM, BN, BK, WGM, WGN>(s, a_km, b_km, M, N, K, A, lda, B, ldb, bias, resid, ldr, C, ldc, rowsum, ws, splits, rowsum_accumulate)
    if (cfg == 1) return TIO_P(256, 256, 64, 2, 4);
    return TIO_P(128, 128, 64, 2, 2);
#undef TIO_P
}

}  // namespace k
}  // namespace tio
