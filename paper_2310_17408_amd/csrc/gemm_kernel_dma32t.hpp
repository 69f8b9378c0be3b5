// fp32 workgroup-tile GEMM kernel with global -> LDS transfers for transposed operands (gemm_ex): A with K
// contiguous (A_KC) and / or B with N contiguous (B_NC).  As in the canonical kernel the transfers are the
// packing step (Pack A / Pack B of the paper's Fig. "Pseudo-code of the BLIS base GEMM algorithm") and the
// MFMA chain on fragments read from LDS is its micro-kernel (Sec. "Micro-kernel Generation").  The canonical orientation is served by
// gemm_kernel_dma32.hpp, whose tile geometry (Dma32Tile), transfers and stage layout this kernel shares.
//
// An fp32 MFMA fragment is one float per lane, so no operand ever needs a transpose: each one is staged as
// it lies in memory and only the index map of the fragment reads changes.
//   * an operand whose rows (m or n) are contiguous (the canonical A; B when B_NC) is staged k-row by k-row
//     (tile row k, BM or BN floats); a lane reads, for one k, the TM (TN) consecutive rows it owns with one
//     LDS read, so the wave tile is interleaved in that dimension: block b is the rows {T*l + b};
//   * an operand with K contiguous (the canonical B; A when A_KC) is staged row by row (tile row m or n,
//     4*BK bytes of K, 16-byte chunks XOR-swizzled by the row) and a lane reads 4 consecutive k of its row,
//     which feed 4 MFMAs; block b is the rows {32*b + l}.
// Transfers move 16 bytes per lane; tiles that cannot be moved inside the matrix, a partial last K step and
// operands whose rows are not 16-byte aligned go through guarded loads and registers into the same layout.
#pragma once
#include "gemm_kernel_dma32.hpp"

namespace mig {

template <class T, bool A_KC, bool B_NC>
struct Dma32MicroT {
    static constexpr int TM = T::TM, TN = T::TN, KSTEPS = T::KSTEPS;
    static constexpr int AK_ROWB = T::B_ROWB;          // a K-contiguous tile row: BK floats
    static constexpr int AM_ROWB = T::BM * 4, BN_ROWB = T::BN * 4;   // a k-row of an operand with contiguous rows
    struct aset { float v[4][TM]; };
    struct bset { float v[4][TN]; };
    uint32_t aoff[A_KC ? KSTEPS : 1], boff[B_NC ? 1 : KSTEPS];

    __device__ __forceinline__ void init(int lane, int wm0, int wn0)
    {
        const int frow = lane & 31, fgrp = lane >> 5;
        const int x = (frow / T::B_RP256) % T::B_CPR;          // chunk swizzle of a K-contiguous row (period 16 rows)
        if constexpr (A_KC) {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) aoff[s] = (wm0 + frow) * AK_ROWB + (((2 * s + fgrp) ^ x) << 4);
        } else {
            aoff[0] = (4 * fgrp) * AM_ROWB + (wm0 + TM * frow) * 4;
        }
        if constexpr (B_NC) {
            boff[0] = T::A_BYTES + (4 * fgrp) * BN_ROWB + (wn0 + TN * frow) * 4;
        } else {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) boff[s] = T::A_BYTES + (wn0 + frow) * AK_ROWB + (((2 * s + fgrp) ^ x) << 4);
        }
    }

    // `count` consecutive floats (1, 2 or 4) at q into dst[0 .. count-1]
    template <int COUNT>
    static __device__ __forceinline__ void read_run(const unsigned char *q, float *dst)
    {
        if constexpr (COUNT == 1) {
            dst[0] = *(const float *)q;
        } else if constexpr (COUNT == 2) {
            const v2f v = *(const v2f *)q;
            dst[0] = v[0]; dst[1] = v[1];
        } else {
            const v4f v = *(const v4f *)q;
            dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
        }
    }

    // fragments of step s (8 consecutive k: this lane's 4 are k = 8 s + 4 (lane / 32) + t)
    __device__ __forceinline__ void load(const unsigned char *stage, int s, aset &xa, bset &xb) const
    {
        if constexpr (A_KC) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const v4f v = *(const v4f *)(stage + aoff[s] + i * 32 * AK_ROWB);
#pragma unroll
                for (int t = 0; t < 4; ++t) xa.v[t][i] = v[t];
            }
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) read_run<TM>(stage + aoff[0] + (8 * s + t) * AM_ROWB, xa.v[t]);
        }
        if constexpr (B_NC) {
#pragma unroll
            for (int t = 0; t < 4; ++t) read_run<TN>(stage + boff[0] + (8 * s + t) * BN_ROWB, xb.v[t]);
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const v4f v = *(const v4f *)(stage + boff[s] + j * 32 * AK_ROWB);
#pragma unroll
                for (int t = 0; t < 4; ++t) xb.v[t][j] = v[t];
            }
        }
    }

    static __device__ __forceinline__ void mma(aset &xa, bset &xb, v16f (&acc)[TM][TN])
    {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.v[t][j], xa.v[t][i], acc[i][j], 0, 0, 0);
    }
};

template <class T, bool A_KC, bool B_NC>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel_dma32t(const Params p)
{
    static_assert(A_KC || B_NC, "the canonical orientation has its own kernel");
    typedef F32 DT;
    typedef Dma32MicroT<T, A_KC, B_NC> Micro;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NW = T::NW, NS = T::NSTAGE;
    constexpr int TM = T::TM, TN = T::TN;
    // 1 KiB transfer blocks: of an operand with contiguous rows `RP` k-rows each, of a K-contiguous one B_R4 rows
    constexpr int AM_RP = 1024 / (BM * 4), BN_RP = 1024 / (BN * 4);
    constexpr int A_BLK = T::A_BYTES / 1024, B_BLK = T::B_BYTES / 1024;
    constexpr int A_J = (A_BLK + NW - 1) / NW, B_J = (B_BLK + NW - 1) / NW;
    static_assert(1024 % (BN * 4) == 0 && 1024 % (BM * 4) == 0, "k-rows must tile 1 KiB blocks");
    static_assert(T::B_R4 % T::B_RP256 == 0 && (NW * T::B_R4 / T::B_RP256) % T::B_CPR == 0, "swizzle must repeat every NW blocks");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(MIG_LDS unsigned char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % T::WAVES_M) * T::WM;
    const int wn0 = (wave / T::WAVES_M) * T::WN;

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    // a tile that sticks out of C is moved back to end at the edge (when the matrix is at least one tile wide)
    const int m_own = tm * BM, n_own = tn * BN;
    const int m0 = (m_own + BM > p.M && p.M >= BM) ? p.M - BM : m_own;
    const int n0 = (n_own + BN > p.N && p.N >= BN) ? p.N - BN : n_own;

    const int z = blockIdx.y;
    const int kt_begin = z * p.ktiles_per_split;
    int kt_end = kt_begin + p.ktiles_per_split;
    if (kt_end > p.ktiles) kt_end = p.ktiles;
    const int nkt = kt_end - kt_begin;

    const float *__restrict__ A = (const float *)p.A;
    const float *__restrict__ B = (const float *)p.B;
    // an operand's tile goes by transfers when its rows lie inside the matrix, are 16-byte aligned (a tile with
    // contiguous rows that was moved may start at any row) and lane offsets fit 32 bits
    const bool fast_a = p.vecA != 0 && (m0 + BM <= p.M) && (p.lda < (1 << 26)) && (A_KC || m0 % 4 == 0);
    const bool fast_b = p.vecB != 0 && (n0 + BN <= p.N) && (p.ldb < (1 << 26)) && (!B_NC || n0 % 4 == 0);

    // ---- which 16 bytes of a 1 KiB block this lane moves: (tile row inside the block, chunk)
    // contiguous rows: AM_RP / BN_RP k-rows per block, no swizzle; K contiguous: B_R4 rows per block, the lane's
    // physical chunk holds the logical chunk that undoes the row's swizzle (the same for blocks NW apart)
    const int a_row_in = A_KC ? lane / T::B_CPR : lane / (BM / 4);
    const int a_ch = A_KC ? (lane % T::B_CPR) ^ (((wave * T::B_R4 + a_row_in) / T::B_RP256) % T::B_CPR) : lane % (BM / 4);
    const int b_row_in = B_NC ? lane / (BN / 4) : lane / T::B_CPR;
    const int b_ch = B_NC ? lane % (BN / 4) : (lane % T::B_CPR) ^ (((wave * T::B_R4 + b_row_in) / T::B_RP256) % T::B_CPR);
    constexpr int A_RPB = A_KC ? T::B_R4 : AM_RP, B_RPB = B_NC ? BN_RP : T::B_R4;      // tile rows per block
    const uint32_t a_off = (uint32_t)(((int64_t)a_row_in * p.lda + a_ch * 4) * 4);
    const uint32_t b_off = (uint32_t)(((int64_t)b_row_in * p.ldb + b_ch * 4) * 4);

    int my_blocks = 0;                  // transfers this wave issues per stage that goes by transfers alone
#pragma unroll
    for (int j = 0; j < A_J; ++j) my_blocks += (wave + NW * j < A_BLK) ? 1 : 0;
#pragma unroll
    for (int j = 0; j < B_J; ++j) my_blocks += (wave + NW * j < B_BLK) ? 1 : 0;
    my_blocks = __builtin_amdgcn_readfirstlane(my_blocks);

    auto stage_tiles = [&](int kt, int buf) {
        const int k0 = kt * BK;
        const bool kfull = (k0 + BK <= p.K);
#pragma unroll
        for (int j = 0; j < A_J; ++j) {
            const int blk = wave + NW * j;
            if (A_BLK % NW != 0 && blk >= A_BLK) break;
            const uint32_t loff = buf * T::STAGE + blk * 1024;
            const int row = blk * A_RPB + a_row_in;             // tile row of this lane: m (A_KC) or k
            if (fast_a && kfull) {
                const float *src = A_KC ? A + (int64_t)(m0 + blk * A_RPB) * p.lda + k0 : A + (int64_t)(k0 + blk * A_RPB) * p.lda + m0;
                lds_dma16(src, a_off, lds_base + loff);
            } else if constexpr (A_KC) {
                const int k = k0 + a_ch * 4;
                int valid = (m0 + row < p.M) ? (p.K - k) : 0;
                valid = valid > 4 ? 4 : valid;
                *(v4i *)(smem + loff + lane * 16) = guarded_chunk<DT>(A + (int64_t)(m0 + row) * p.lda + k, valid);
            } else {
                const int m = m0 + a_ch * 4;
                int valid = (k0 + row < p.K) ? (p.M - m) : 0;
                valid = valid > 4 ? 4 : valid;
                *(v4i *)(smem + loff + lane * 16) = guarded_chunk<DT>(A + (int64_t)(k0 + row) * p.lda + m, valid);
            }
        }
#pragma unroll
        for (int j = 0; j < B_J; ++j) {
            const int blk = wave + NW * j;
            if (B_BLK % NW != 0 && blk >= B_BLK) break;
            const uint32_t loff = buf * T::STAGE + T::A_BYTES + blk * 1024;
            const int row = blk * B_RPB + b_row_in;             // tile row of this lane: k (B_NC) or n
            if (fast_b && kfull) {
                const float *src = B_NC ? B + (int64_t)(k0 + blk * B_RPB) * p.ldb + n0 : B + (int64_t)(n0 + blk * B_RPB) * p.ldb + k0;
                lds_dma16(src, b_off, lds_base + loff);
            } else if constexpr (B_NC) {
                const int n = n0 + b_ch * 4;
                int valid = (k0 + row < p.K) ? (p.N - n) : 0;
                valid = valid > 4 ? 4 : valid;
                *(v4i *)(smem + loff + lane * 16) = guarded_chunk<DT>(B + (int64_t)(k0 + row) * p.ldb + n, valid);
            } else {
                const int k = k0 + b_ch * 4;
                int valid = (n0 + row < p.N) ? (p.K - k) : 0;
                valid = valid > 4 ? 4 : valid;
                *(v4i *)(smem + loff + lane * 16) = guarded_chunk<DT>(B + (int64_t)(n0 + row) * p.ldb + k, valid);
            }
        }
    };

    const int frow = lane & 31, fgrp = lane >> 5;
    Micro micro;
    micro.init(lane, wm0, wn0);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // ---- the micro-kernel, fragments double buffered in registers; the K loop rotates NS stages: the barrier
    // that ends step i sits between the LDS reads and the MFMAs of its last fragment step
    typename Micro::aset fa[2];
    typename Micro::bset fb[2];
    auto steps_but_last = [&](int buf) {
#pragma unroll
        for (int s = 0; s + 1 < T::KSTEPS; ++s) {
            micro.load(smem + buf * T::STAGE, s + 1, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            Micro::mma(fa[s & 1], fb[s & 1], acc);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    constexpr int LAST = (T::KSTEPS - 1) & 1;
    int nfast = 0;                      // leading steps of this workgroup that are transfers only
    if (fast_a && fast_b) {
        nfast = p.K / BK - kt_begin;
        nfast = nfast < 0 ? 0 : (nfast > nkt ? nkt : nfast);
    }
    // A full K step that goes by transfers alone, with all a wave needs precomputed: base pointers of its first
    // block that advance by a constant per step, a constant distance between its blocks, lane offsets that never change
    const unsigned char *a_wave = (const unsigned char *)(A_KC ? A + (int64_t)(m0 + wave * A_RPB) * p.lda : A + (int64_t)(wave * A_RPB) * p.lda + m0);
    const unsigned char *b_wave = (const unsigned char *)(B_NC ? B + (int64_t)(wave * B_RPB) * p.ldb + n0 : B + (int64_t)(n0 + wave * B_RPB) * p.ldb);
    const int64_t a_step = A_KC ? (int64_t)BK * 4 : (int64_t)BK * p.lda * 4;
    const int64_t b_step = B_NC ? (int64_t)BK * p.ldb * 4 : (int64_t)BK * 4;
    const int64_t a_blk = (int64_t)NW * A_RPB * p.lda * 4, b_blk = (int64_t)NW * B_RPB * p.ldb * 4;
    auto stage_direct = [&](int kt, int buf) {
        const unsigned char *ab = a_wave + (int64_t)kt * a_step;
        const unsigned char *bb = b_wave + (int64_t)kt * b_step;
        const uint32_t la = lds_base + buf * T::STAGE + wave * 1024;
#pragma unroll
        for (int j = 0; j < A_J; ++j) {
            if (A_BLK % NW != 0 && wave + NW * j >= A_BLK) break;
            lds_dma16(ab + j * a_blk, a_off, la + j * NW * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_J; ++j) {
            if (B_BLK % NW != 0 && wave + NW * j >= B_BLK) break;
            lds_dma16(bb + j * b_blk, b_off, la + T::A_BYTES + j * NW * 1024);
        }
    };

    if (nkt > 0) {
#pragma unroll
        for (int t = 0; t < NS; ++t)
            if (t < nkt) stage_tiles(kt_begin + t, t);
        {
            const int staged = nkt < NS ? nkt : NS;
            wait_transfers_upto(staged <= nfast ? (staged - 1) * my_blocks : 0);
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        micro.load(smem, 0, fa[0], fb[0]);
        int buf = 0, i = 0;
        // hot loop: runs while the step it stages (i + NS) and all steps in flight go by transfers alone
        for (; i + NS < nfast; ++i) {
            const int nxt = (buf + 1 == NS) ? 0 : buf + 1;
            steps_but_last(buf);
            wait_transfers_upto((NS - 2) * my_blocks);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            stage_direct(kt_begin + i + NS, buf);
            micro.load(smem + nxt * T::STAGE, 0, fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            Micro::mma(fa[LAST], fb[LAST], acc);
            buf = nxt;
        }
        for (; i < nkt; ++i) {
            const int nxt = (buf + 1 == NS) ? 0 : buf + 1;
            steps_but_last(buf);
            if (i + 1 < nkt) {
                // steps i+1 .. min(i+NS-1, nkt-1) are staged; step i+1 has landed when only the later ones are
                // outstanding (transfers complete in order), if all of them go by transfers alone
                int last = i + NS - 1;
                last = last < nkt - 1 ? last : nkt - 1;
                wait_transfers_upto(last < nfast ? (last - (i + 1)) * my_blocks : 0);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (i + NS < nkt) stage_tiles(kt_begin + i + NS, buf);
                micro.load(smem + nxt * T::STAGE, 0, fa[0], fb[0]);
                __builtin_amdgcn_sched_barrier(0);
            }
            Micro::mma(fa[LAST], fb[LAST], acc);
            buf = nxt;
        }
    }

    // ---- epilogue.  In a 32 x 32 block lane l holds the column of the block that its A-operand row (l % 32)
    // gives and, in register v, the row 8 (v / 4) + 4 (l / 32) + v % 4 that the B-operand gives; rows and columns
    // of C follow from the two index maps of the fragment reads.
    {
        const bool interior = (m0 + BM <= p.M) && (n0 + BN <= p.N) && m0 == m_own && n0 == n_own;
        const float alpha = __builtin_bit_cast(float, p.alpha_bits);
        const float beta = __builtin_bit_cast(float, p.beta_bits);
        const bool use_beta = p.use_beta != 0;
        // with contiguous rows of A a lane owns TM consecutive m of every column: one vector store where C allows
        const int mrow = m0 + wm0 + TM * frow;
        const bool vec_c = !A_KC && (TM > 1) && interior && ((p.ldc % TM) == 0) && (((uintptr_t)p.C % (TM * 4)) == 0) &&
                           p.split <= 1;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rho = 8 * (v >> 2) + 4 * fgrp + (v & 3);
                const int n = n0 + wn0 + (B_NC ? TN * rho + j : 32 * j + rho);
                if (vec_c) {
                    float *c = (float *)p.C + (int64_t)n * p.ldc + mrow;
                    if constexpr (TM == 2) {
                        v2f r = {alpha * acc[0][j][v], alpha * acc[1][j][v]};
                        if (use_beta) { v2f o = *(const v2f *)c; r[0] += beta * o[0]; r[1] += beta * o[1]; }
                        *(v2f *)c = r;
                    } else if constexpr (TM == 4) {
                        v4f r = {alpha * acc[0][j][v], alpha * acc[1][j][v], alpha * acc[2][j][v], alpha * acc[3][j][v]};
                        if (use_beta) {
                            v4f o = *(const v4f *)c;
                            r[0] += beta * o[0]; r[1] += beta * o[1]; r[2] += beta * o[2]; r[3] += beta * o[3];
                        }
                        *(v4f *)c = r;
                    }
                    continue;
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int m = m0 + wm0 + (A_KC ? 32 * i + frow : TM * frow + i);
                    if (!(interior || (m >= m_own && m < p.M && n >= n_own && n < p.N))) continue;
                    if (p.split > 1) {
                        ((float *)p.ws)[((int64_t)z * p.N + n) * p.M + m] = acc[i][j][v];
                    } else {
                        float *c = (float *)p.C + (int64_t)n * p.ldc + m;
                        float r = alpha * acc[i][j][v];
                        if (use_beta) r += beta * (*c);
                        *c = r;
                    }
                }
            }
        }
    }
}

}  // namespace mig
