// Workgroup-tile GEMM kernel for gfx950 whose packing step (Pack A / Pack B of
// the paper's Fig. "Pseudo-code of the BLIS base GEMM algorithm") is done by
// the memory system: operand tiles go from global memory straight into LDS
// (16 bytes per lane, no registers in between), several stages deep, and the
// micro-kernel reads MFMA fragments from them:
//   * the K-contiguous operand B is staged row by row (tile row n, 128 bytes of
//     K) and read with 16-byte LDS reads;
//   * the M-contiguous operand A is staged as it lies in memory (tile row k, BM
//     elements of M) and read with the transposing LDS reads of gfx950, which
//     hand each lane consecutive K for its own m.  This replaces the register
//     transposes of the staged kernel in gemm_kernel.hpp.
// A 16-byte chunk is stored at a position XOR-ed with low bits of its tile row,
// so that the lanes of one LDS read hit distinct banks; the writer applies the
// same permutation by choosing which global chunk each lane fetches.
// Edge tiles, a partial last K step and operands that are not 16-byte aligned
// are staged by guarded loads through registers into the same layout.
//
// Canonical problem and epilogue are those of gemm_kernel.hpp.
#pragma once
#include "gemm_kernel.hpp"

namespace mig {

typedef short v4s __attribute__((ext_vector_type(4)));
#define MIG_LDS __attribute__((address_space(3)))

template <class DT_, int BM_, int BN_, int WAVES_M_, int WAVES_N_, int KSTEPS_, int NSTAGE_, int MINB_>
struct DmaTile {
    typedef DT_ DT;
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, MINB = MINB_;
    static constexpr int KSTEPS = KSTEPS_;              // fragment steps (2 chunks of K each) per stage
    static constexpr int NSTAGE = NSTAGE_;              // LDS stages: one being multiplied, the others in flight
    static constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int ES = DT::ES, KCH = DT::KCH;
    static constexpr int BK = 2 * KCH * KSTEPS;         // K elements per stage
    static constexpr int B_ROWB = 32 * KSTEPS;          // bytes of one row of the B tile
    static constexpr int B_CPR = 2 * KSTEPS;            // 16-byte chunks per B row
    static constexpr int B_RP256 = 16 / B_CPR;          // B rows per 256 bytes (one pass over the LDS banks)
    // Chunk swizzle of a K-contiguous tile row: chunk c of row n is stored at c ^ b_swz(n), so that the 16-byte
    // fragment reads of a wave (lane l: row l%16, chunk l/16 of a K step) meet no bank twice.  Rows of 128 bytes:
    // the row pair takes the 3 chunk bits; rows of 64 bytes (4 chunks, 4 rows per pass over the banks): the
    // second of two groups of 4 rows swaps its chunk pairs (found by measuring all linear maps of the row
    // index with SQ_LDS_BANK_CONFLICT: (n / 4) % 4, the analogue of the wider rows, conflicts two-way).
    static __host__ __device__ constexpr int b_swz(int n)
    {
        return B_CPR == 8 ? ((n / 2) % 8) : (((n >> 2) & 1) << 1);
    }
    static constexpr int B_SWZ_PERIOD = 16;             // b_swz(n + 16) == b_swz(n)
    static constexpr int A_ROWB = BM * ES;              // bytes of one k-row of the A tile
    static constexpr int A_CPR = A_ROWB / 16;           // 16-byte chunks per k-row
    static constexpr int A_BYTES = BK * A_ROWB;
    static constexpr int B_BYTES = BN * B_ROWB;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE;
    static constexpr int A_INST = A_BYTES / 1024 / NW;  // 1 KiB transfers per wave and stage
    static constexpr int B_INST = B_BYTES / 1024 / NW;
    static constexpr int A_ROWS_PER_INST = 1024 / A_ROWB;
    static constexpr int B_ROWS_PER_INST = 1024 / B_ROWB;
    static constexpr int INST = A_INST + B_INST;
    // transposing read: a group of 16 lanes reads KH k-rows x 16 m; LPR lanes share a row
    static constexpr int LPR = 2 * ES;                  // 4 (16-bit) or 2 (8-bit)
    static constexpr int KH = 16 / LPR;                 // k-rows per transposing read: 4 or 8
    // A chunk swizzle: the chunk index of k-row k is XORed with a_swz(k), so that one pass of the
    // transposing reads (32 lanes: KH consecutive k-rows of two neighbouring k groups, LPR 8-byte pieces
    // each) touches every LDS bank once.  With k-rows of 256 bytes or more the KH rows take the upper
    // chunk bits and the parity of the k group the bit below them; with 128-byte k-rows (int8, BM = 128)
    // the parity of k is an address bit already and the row pairs take the swizzle.
    static constexpr int SWZ_SHIFT = (ES == 2) ? 2 : 1;
    static constexpr int SWZ_MASK_FULL = KH - 1;
    static constexpr int SWZ_MASK = ((SWZ_MASK_FULL << SWZ_SHIFT) < A_CPR) ? SWZ_MASK_FULL : (SWZ_MASK_FULL >> 1);
    static constexpr int SWZ_PERIOD = 2 * KCH;          // a_swz(k + SWZ_PERIOD) == a_swz(k)
    static __host__ __device__ constexpr int a_swz(int k)
    {
        return A_CPR >= 16 ? (((k & SWZ_MASK_FULL) << SWZ_SHIFT) ^ (((k / KCH) & 1) << (SWZ_SHIFT - 1)))
                           : ((((k >> 1) & 3) << 1) ^ ((k / KCH) & 1));
    }
    static_assert(KSTEPS == 2 || KSTEPS == 4, "a B row holds 4 or 8 chunks");
    static_assert(NSTAGE >= 2 && (NSTAGE - 2) * INST <= 63, "transfers in flight must fit the counter");
    static_assert(ES == 1 || ES == 2, "transposing LDS reads exist for 8- and 16-bit elements");
    static_assert(A_ROWB <= 1024 && 1024 % A_ROWB == 0, "a 1 KiB transfer must cover whole k-rows of A");
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tiles must split evenly over the waves");
    static_assert(A_CPR >= 16 || (A_CPR == 8 && ES == 1), "k-rows of at least 256 bytes, or 128 bytes of int8");
    static_assert(A_CPR >= 16 ? ((SWZ_MASK_FULL << SWZ_SHIFT) | (1 << (SWZ_SHIFT - 1))) < A_CPR : true,
                  "swizzle must stay inside a row");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tiles are made of 32x32 blocks");
};

// One 1 KiB global -> LDS transfer by the calling wave: lane l writes LDS bytes
// [lds_addr + 16*l, +16) with the 16 bytes at base + lane_off (base is uniform,
// lane_off a 32-bit byte offset of the lane).
__device__ __forceinline__ void lds_dma16(const void *base, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_off), "s"(base)
                 : "memory");
}

// Wait until at most N of this wave's vector-memory operations (the transfers above complete in
// order) and none of its LDS operations are outstanding.  s_waitcnt immediate of gfx9:
// vmcnt = bits 3:0 and 15:14, expcnt = bits 6:4 (7 = no wait), lgkmcnt = bits 11:8.
template <int N>
__device__ __forceinline__ void wait_transfers()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
    asm volatile("" ::: "memory");
}

// 16 bytes along the contiguous dimension with the first `valid` elements taken
// from memory and the rest zero (edge tiles, K tail, unaligned operands).
template <class DT>
__device__ __forceinline__ v4i guarded_chunk(const typename DT::elt *src, int valid)
{
    constexpr int ES = DT::ES;
    if (valid >= 16 / ES) return *(const v4i_u *)src;     // the whole chunk exists: one load at any alignment
    v4i v;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t word = 0;
#pragma unroll
        for (int e = 0; e < 4 / ES; ++e) {
            const int idx = w * (4 / ES) + e;
            uint32_t bits = 0;
            if (idx < valid) {
                if constexpr (ES == 4) bits = __builtin_bit_cast(uint32_t, src[idx]);
                else if constexpr (ES == 2) bits = (uint16_t)src[idx];
                else bits = (uint8_t)src[idx];
            }
            word |= bits << (8 * ES * e);
        }
        v[w] = (int)word;
    }
    return v;
}

// The micro-kernel of the direct kernels (loop L6 and the fragment reads that feed it), shared by
// the GEMM kernel and by the solo-mode benchmark.  A stage holds the A tile (k-rows of BM elements,
// chunks swizzled by k) followed by the B tile (rows of B_ROWB bytes, chunks swizzled by row).
template <class T>
struct DmaMicro {
    typedef typename T::DT DT;
    typedef typename DT::accv accv;
    static constexpr int TM = T::TM, TN = T::TN, ES = T::ES, KCH = T::KCH, A_ROWB = T::A_ROWB, KH = T::KH;
    static constexpr int STEPS = T::KSTEPS;          // fragment steps per stage (an even number)
    static constexpr int ACC = 16;
    // the fragments of one step, double buffered: per block row / column 16 bytes = KCH consecutive k
    v4i fa[2][TM], fb[2][TN];
    uint32_t aoff[TM], boff[T::KSTEPS];

    // fragment addresses of this lane inside a stage, for the wave whose tile starts at (wm0, wn0)
    __device__ __forceinline__ void init(int lane, int wm0, int wn0)
    {
        const int frow = lane & 31, fgrp = lane >> 5;
        // B: row wn0 + 32*j + frow, logical chunk 2*s + fgrp; wn0 and 32*j are multiples of 16,
        // so the swizzle of the row depends on frow only
        const int x = (frow / T::B_RP256) % T::B_CPR;
#pragma unroll
        for (int s = 0; s < T::KSTEPS; ++s)
            boff[s] = T::A_BYTES + (wn0 + frow) * T::B_ROWB + (((2 * s + fgrp) ^ x) << 4);
        // A: the 16-lane group q = lane/16 serves m-half q%2 of the block for k-group q/2 (= fgrp);
        // inside it, lane t addresses k-row t/LPR and the (t%LPR)-th 8-byte piece of 16 m.
        const int t = lane & 15, mh = (lane >> 4) & 1;
        const int kr = t / T::LPR, ml = t % T::LPR;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mbyte = (wm0 + 32 * i + 16 * mh) * ES + 8 * ml;
            const int ch = (mbyte >> 4) ^ T::a_swz(KCH * fgrp + kr);
            aoff[i] = (KCH * fgrp + kr) * A_ROWB + (ch << 4) + (mbyte & 15);
        }
    }

    // two transposing reads give a lane KCH consecutive k of its m
    static __device__ __forceinline__ v4i read_a(const unsigned char *q0)
    {
        const unsigned char *q1 = q0 + KH * A_ROWB;
        if constexpr (ES == 2) {
            v2i lo = __builtin_bit_cast(v2i, __builtin_amdgcn_ds_read_tr16_b64_v4i16((MIG_LDS v4s *)q0));
            v2i hi = __builtin_bit_cast(v2i, __builtin_amdgcn_ds_read_tr16_b64_v4i16((MIG_LDS v4s *)q1));
            return v4i{lo[0], lo[1], hi[0], hi[1]};
        } else {
            v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((MIG_LDS v2i *)q0);
            v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((MIG_LDS v2i *)q1);
            return v4i{lo[0], lo[1], hi[0], hi[1]};
        }
    }

    // LDS reads of fragment step s (2*KCH consecutive k) of the stage at `stage` into set s%2
    __device__ __forceinline__ void load(const unsigned char *stage, int s)
    {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[s & 1][i] = read_a(stage + aoff[i] + (2 * KCH * s) * A_ROWB);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[s & 1][j] = *(const v4i *)(stage + boff[s] + j * 32 * T::B_ROWB);
    }

    // the MFMAs of fragment step s
    __device__ __forceinline__ void mma(int s, accv (&acc)[TM][TN])
    {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) Mma<DT>::run(fb[s & 1][j], fa[s & 1][i], acc[i][j]);
    }

    static __device__ __forceinline__ void store(accv (&acc)[TM][TN], const Params &p, int m0, int n0, int wm0, int wn0,
                                                 int lane, int z, int m_own, int n_own)
    {
        store_tile<DT, TM, TN>(acc, p, m0, n0, T::BM, T::BN, wm0, wn0, lane, z, m_own, n_own);
    }
};

// The same wave tile cut into 16 x 16 blocks for the MFMA shapes with the deepest K per
// instruction (16x16x32 for 16-bit inputs, 16x16x64 for int8).  They update a quarter of the
// accumulators per multiply-add of the 32 x 32 shapes; on random operands the chip, which lowers
// its clock under the power these instructions draw, sustains 18-25 % more with them (register-only
// loops: fp16 1.83 against 1.55 PFLOP/s, bf16 2.02 against 1.71, int8 4.13 against 3.31 POP/s).
// A lane holds row (or column) lane%16 and the k group lane/16 of 4: KCH consecutive k per fragment.
// A fragment step covers 4*KCH k; it is taken in two halves of the wave tile's rows so that the
// fragments in flight stay at 16 + 16 registers per set: sub-step s = (k step s/2, row half s%2);
// the B fragments are read with the first half and kept for the second.
template <class DT> struct Mma16;
template <> struct Mma16<F16> {
    typedef v4f accv;
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v4f &c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, rowop), __builtin_bit_cast(v8h, colop), c, 0, 0, 0);
    }
};
template <> struct Mma16<BF16> {
    typedef v4f accv;
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v4f &c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, rowop), __builtin_bit_cast(v8bf, colop), c, 0, 0, 0);
    }
};
template <> struct Mma16<I8> {
    typedef v4i accv;
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v4i &c) {
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(rowop, colop, c, 0, 0, 0);
    }
};

// A_KC: the operand A has K contiguous as well (a transposed A: op(A) = A^T of a column-major problem,
// or the weight matrix of x W^T in row-major terms).  Its tile is then staged exactly like B's (tile
// rows of K, chunks swizzled by row) and its fragments are plain 16-byte reads; no transposing reads.
// B_NC: the operand B has N contiguous (a transposed B); its tile is then staged exactly like the
// canonical A's (k-rows of BN elements, the same swizzle) and read with the transposing reads.
// Square tiles only, so that both operands share the constants of that layout.
template <class T, bool A_KC = false, bool B_NC = false>
struct DmaMicro16 {
    typedef typename T::DT DT;
    typedef typename Mma16<DT>::accv accv;
    static constexpr int TM = T::WM / 16, TN = T::WN / 16, HM = TM / 2;
    static constexpr int ES = T::ES, KCH = T::KCH, A_ROWB = T::A_ROWB, KH = T::KH;
    static constexpr int STEPS = T::KSTEPS;          // sub-steps per stage: KSTEPS/2 k steps x 2 row halves
    static constexpr int ACC = 4;
    static_assert(T::KSTEPS % 2 == 0 && TM % 2 == 0, "k steps of 4 chunks, two row halves");
    v4i fa[2][HM], fb[2][TN];
    uint32_t aoff[A_KC ? T::KSTEPS / 2 : TM], boff[B_NC ? TN : T::KSTEPS / 2];
    static_assert(!B_NC || T::BM == T::BN, "a transposed B needs a square tile");

    __device__ __forceinline__ void init(int lane, int wm0, int wn0)
    {
        const int r = lane & 15, g = lane >> 4;
        // B: row wn0 + 16*j + r, logical chunk 4*ks + g; the swizzle of the row depends on r only
        const int x = (r / T::B_RP256) % T::B_CPR;
        if constexpr (B_NC) {
            // B staged like the canonical A: k group g of the 16 columns n of a block
            const int kr = r / T::LPR, ml = r % T::LPR;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nbyte = (wn0 + 16 * j) * ES + 8 * ml;
                const int ch = (nbyte >> 4) ^ T::a_swz(KCH * g + kr);
                boff[j] = T::A_BYTES + (KCH * g + kr) * A_ROWB + (ch << 4) + (nbyte & 15);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < T::KSTEPS / 2; ++ks)
                boff[ks] = T::A_BYTES + (wn0 + r) * T::B_ROWB + (((4 * ks + g) ^ x) << 4);
        }
        if constexpr (A_KC) {
            // A staged like B: row wm0 + 16*i + r of the A region, same chunk and swizzle
#pragma unroll
            for (int ks = 0; ks < T::KSTEPS / 2; ++ks)
                aoff[ks] = (wm0 + r) * T::B_ROWB + (((4 * ks + g) ^ x) << 4);
            return;
        }
        // A: the 16-lane group g reads k group g of the 16 rows of a block; inside it, lane r
        // addresses k-row r/LPR and the (r%LPR)-th 8-byte piece of the 16 m
        const int kr = r / T::LPR, ml = r % T::LPR;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mbyte = (wm0 + 16 * i) * ES + 8 * ml;
            const int ch = (mbyte >> 4) ^ T::a_swz(KCH * g + kr);
            aoff[i] = (KCH * g + kr) * A_ROWB + (ch << 4) + (mbyte & 15);
        }
    }

    __device__ __forceinline__ void load(const unsigned char *stage, int s)
    {
        const int ks = s >> 1, mh = s & 1;
#pragma unroll
        for (int i = 0; i < HM; ++i) {
            if constexpr (A_KC) fa[s & 1][i] = *(const v4i *)(stage + aoff[ks] + (mh * HM + i) * 16 * T::B_ROWB);
            else fa[s & 1][i] = DmaMicro<T>::read_a(stage + aoff[mh * HM + i] + (4 * KCH * ks) * A_ROWB);
        }
        if (mh == 0) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (B_NC) fb[ks & 1][j] = DmaMicro<T>::read_a(stage + boff[j] + (4 * KCH * ks) * A_ROWB);
                else fb[ks & 1][j] = *(const v4i *)(stage + boff[ks] + j * 16 * T::B_ROWB);
            }
        }
    }

    __device__ __forceinline__ void mma(int s, accv (&acc)[TM][TN])
    {
        const int ks = s >> 1, mh = s & 1;
#pragma unroll
        for (int i = 0; i < HM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) Mma16<DT>::run(fb[ks & 1][j], fa[s & 1][i], acc[mh * HM + i][j]);
    }

    // In a 16 x 16 block a lane holds row m = lane%16 and the columns n = 4*(lane/16) + v.
    static __device__ __forceinline__ void store(accv (&acc)[TM][TN], const Params &p, int m0, int n0, int wm0, int wn0,
                                                 int lane, int z, int m_own, int n_own)
    {
        typedef typename DT::acc_t acc_t;
        const int r = lane & 15, g = lane >> 4;
        const bool interior = (m0 + T::BM <= p.M) && (n0 + T::BN <= p.N) && m0 == m_own && n0 == n_own;
        const acc_t alpha = __builtin_bit_cast(acc_t, p.alpha_bits);
        const acc_t beta = __builtin_bit_cast(acc_t, p.beta_bits);
        const bool use_beta = p.use_beta != 0;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + wm0 + 16 * i + r;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int n = n0 + wn0 + 16 * j + 4 * g + v;
                    if (interior || (m >= m_own && m < p.M && n >= n_own && n < p.N)) {
                        const acc_t a = acc[i][j][v];
                        if (p.split > 1) {
                            ((acc_t *)p.ws)[((int64_t)z * p.N + n) * p.M + m] = a;
                        } else {
                            acc_t *c = (acc_t *)p.C + (int64_t)n * p.ldc + m;
                            if constexpr (DT::ES == 1) {
                                uint32_t o = (uint32_t)alpha * (uint32_t)a;
                                if (use_beta) o += (uint32_t)beta * (uint32_t)(*c);
                                *c = (int)o;
                            } else {
                                update_c(p, (int64_t)n * p.ldc + m, a, alpha, beta, use_beta);
                            }
                        }
                    }
                }
            }
        }
    }
};

template <class T, class Micro = DmaMicro<T>, bool A_KC = false, bool B_NC = false>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel_dma(const Params p)
{
    static_assert(!B_NC || T::BM == T::BN, "a transposed B needs a square tile");
    typedef typename T::DT DT;
    typedef typename DT::elt elt;
    typedef typename Micro::accv accv;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NW = T::NW, ES = T::ES, KCH = T::KCH;
    constexpr int TM = Micro::TM, TN = Micro::TN, A_CPR = T::A_CPR;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(MIG_LDS unsigned char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % T::WAVES_M) * T::WM;
    const int wn0 = (wave / T::WAVES_M) * T::WN;

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    // A tile that sticks out of C is moved back so that it ends at the edge, when the matrix is at
    // least one tile wide and the moved tile keeps the 16-byte alignment of its rows: it then takes
    // the direct transfers of an interior tile and stores only the part no other tile owns.
    const int m_own = tm * BM, n_own = tn * BN;
    // (A_KC: rows of A are lda apart, so a moved tile is as aligned as any other)
    const int m0 = (m_own + BM > p.M && p.M >= BM && (A_KC || (p.M * ES) % 16 == 0)) ? p.M - BM : m_own;
    const int n0 = (n_own + BN > p.N && p.N >= BN && (!B_NC || (p.N * ES) % 16 == 0)) ? p.N - BN : n_own;

    const int z = blockIdx.y;
    const int kt_begin = z * p.ktiles_per_split;
    int kt_end = kt_begin + p.ktiles_per_split;
    if (kt_end > p.ktiles) kt_end = p.ktiles;
    const int nkt = kt_end - kt_begin;

    const elt *__restrict__ A = (const elt *)p.A;
    const elt *__restrict__ B = (const elt *)p.B;
    const bool tile_fast_a = p.vecA && (m0 + BM <= p.M);
    const bool tile_fast_b = p.vecB && (n0 + BN <= p.N);

    // ---- staging: which chunk of the A and B tiles this lane moves in transfer j
    // A: transfer block b = wave + NW*j covers k-rows b*A_ROWS_PER_INST ...; lane -> (row, physical chunk)
    // (A_KC: like B, transfer block b covers B_ROWS_PER_INST tile rows m)
    const int a_row_in = A_KC ? lane / T::B_CPR : lane / A_CPR, a_pch = A_KC ? lane % T::B_CPR : lane % A_CPR;
    // B: transfer block b covers B_ROWS_PER_INST tile rows; lane -> (row, physical chunk)
    // (B_NC: like the canonical A, transfer block b covers A_ROWS_PER_INST k-rows)
    const int b_row_in = B_NC ? lane / A_CPR : lane / T::B_CPR, b_pch = B_NC ? lane % A_CPR : lane % T::B_CPR;
    // The swizzle term of a lane's row does not depend on j (NW transfers apart the row pattern
    // repeats), so a lane's byte offset from the block's first element is the same in every transfer.
    static_assert((NW * T::A_ROWS_PER_INST) % T::SWZ_PERIOD == 0, "A swizzle must repeat every NW blocks");
    static_assert((NW * T::B_ROWS_PER_INST) % (T::B_RP256 * T::B_CPR) == 0, "B swizzle must repeat every NW blocks");
    const int a_ch = A_KC ? a_pch ^ (((wave * T::B_ROWS_PER_INST + a_row_in) / T::B_RP256) % T::B_CPR)
                          : a_pch ^ T::a_swz(wave * T::A_ROWS_PER_INST + a_row_in);
    const int b_ch = B_NC ? b_pch ^ T::a_swz(wave * T::A_ROWS_PER_INST + b_row_in)
                          : b_pch ^ (((wave * T::B_ROWS_PER_INST + b_row_in) / T::B_RP256) % T::B_CPR);
    const uint32_t a_lane_off = (uint32_t)(((int64_t)a_row_in * p.lda + a_ch * (16 / ES)) * ES);   // 16/ES == KCH
    const uint32_t b_lane_off = (uint32_t)(((int64_t)b_row_in * p.ldb + b_ch * KCH) * ES);
    constexpr int A_RPI = A_KC ? T::B_ROWS_PER_INST : T::A_ROWS_PER_INST;          // tile rows (m or k) per transfer
    const int64_t a_blk_stride = (int64_t)NW * A_RPI * p.lda * ES;                 // bytes between transfers j, j+1
    constexpr int B_RPI = B_NC ? T::A_ROWS_PER_INST : T::B_ROWS_PER_INST;         // tile rows (k or n) per transfer
    const int64_t b_blk_stride = (int64_t)NW * B_RPI * p.ldb * ES;
    const int64_t b_step = B_NC ? (int64_t)BK * p.ldb * ES : (int64_t)BK * ES;
    const int64_t a_step = A_KC ? (int64_t)BK * ES : (int64_t)BK * p.lda * ES;      // bytes from one K step to the next
    const unsigned char *a_wave = A_KC ? (const unsigned char *)A + ((int64_t)(m0 + wave * A_RPI) * p.lda) * ES
                                       : (const unsigned char *)A + ((int64_t)wave * A_RPI * p.lda + m0) * ES;
    const unsigned char *b_wave = B_NC ? (const unsigned char *)B + ((int64_t)wave * B_RPI * p.ldb + n0) * ES
                                       : (const unsigned char *)B + ((int64_t)(n0 + wave * B_RPI) * p.ldb) * ES;

    // all transfers of one K step, operands fully inside the matrices and 16-byte aligned
    auto stage_dma = [&](int kt, int buf) {
        const unsigned char *ab = a_wave + (int64_t)kt * a_step;
        const unsigned char *bb = b_wave + (int64_t)kt * b_step;
        const uint32_t la = lds_base + buf * T::STAGE + wave * 1024;
#pragma unroll
        for (int j = 0; j < T::A_INST; ++j) lds_dma16(ab + j * a_blk_stride, a_lane_off, la + j * NW * 1024);
#pragma unroll
        for (int j = 0; j < T::B_INST; ++j)
            lds_dma16(bb + j * b_blk_stride, b_lane_off, la + T::A_BYTES + j * NW * 1024);
    };

    // the same chunks through registers, with zero fill: edge tiles, partial K step, unaligned operands
    auto stage_guarded = [&](int kt, int buf, bool dma_a, bool dma_b) {
        const int k0 = kt * BK;
        const uint32_t sbase = buf * T::STAGE;
        if (dma_a) {
            const unsigned char *ab = a_wave + (int64_t)kt * a_step;
#pragma unroll
            for (int j = 0; j < T::A_INST; ++j)
                lds_dma16(ab + j * a_blk_stride, a_lane_off, lds_base + sbase + (wave + NW * j) * 1024);
        } else {
#pragma unroll
            for (int j = 0; j < T::A_INST; ++j) {
                const int blk = wave + NW * j;
                if constexpr (A_KC) {
                    const int r = blk * A_RPI + a_row_in;                      // tile row m
                    const int k = k0 + a_ch * KCH;
                    const elt *src = A + (int64_t)(m0 + r) * p.lda + k;
                    int valid = (m0 + r < p.M) ? (p.K - k) : 0;
                    valid = valid > KCH ? KCH : valid;
                    *(v4i *)(smem + sbase + blk * 1024 + lane * 16) = guarded_chunk<DT>(src, valid);
                    continue;
                }
                const int k = blk * T::A_ROWS_PER_INST + a_row_in;             // tile-local k-row
                const int m = m0 + a_ch * (16 / ES);
                const elt *src = A + (int64_t)(k0 + k) * p.lda + m;
                int valid = (k0 + k < p.K) ? (p.M - m) : 0;
                valid = valid > 16 / ES ? 16 / ES : valid;
                *(v4i *)(smem + sbase + blk * 1024 + lane * 16) = guarded_chunk<DT>(src, valid);
            }
        }
        if (dma_b) {
            const unsigned char *bb = b_wave + (int64_t)kt * b_step;
#pragma unroll
            for (int j = 0; j < T::B_INST; ++j)
                lds_dma16(bb + j * b_blk_stride, b_lane_off, lds_base + sbase + T::A_BYTES + (wave + NW * j) * 1024);
        } else {
#pragma unroll
            for (int j = 0; j < T::B_INST; ++j) {
                const int blk = wave + NW * j;
                if constexpr (B_NC) {
                    const int k = blk * B_RPI + b_row_in;                      // tile-local k-row
                    const int n = n0 + b_ch * (16 / ES);
                    const elt *src = B + (int64_t)(k0 + k) * p.ldb + n;
                    int valid = (k0 + k < p.K) ? (p.N - n) : 0;
                    valid = valid > 16 / ES ? 16 / ES : valid;
                    *(v4i *)(smem + sbase + T::A_BYTES + blk * 1024 + lane * 16) = guarded_chunk<DT>(src, valid);
                    continue;
                }
                const int r = blk * T::B_ROWS_PER_INST + b_row_in;              // tile row n
                const int k = k0 + b_ch * KCH;
                const elt *src = B + (int64_t)(n0 + r) * p.ldb + k;
                int valid = (n0 + r < p.N) ? (p.K - k) : 0;
                valid = valid > KCH ? KCH : valid;
                *(v4i *)(smem + sbase + T::A_BYTES + blk * 1024 + lane * 16) = guarded_chunk<DT>(src, valid);
            }
        }
    };
    auto stage_tiles = [&](int kt, int buf) {
        const bool kfull = ((kt + 1) * BK <= p.K);
        stage_guarded(kt, buf, tile_fast_a && kfull, tile_fast_b && kfull);
    };

    Micro micro;
    micro.init(lane, wm0, wn0);

    accv acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < Micro::ACC; ++v) acc[i][j][v] = 0;

    // ---- the micro-kernel: Micro::STEPS fragment steps per stage.  Fragments are double buffered in
    // registers (inside `micro`): while the MFMAs of one step run, the LDS reads of the next are in
    // flight, also across the barrier that ends a K step.
    auto load_frags = [&](int buf, int s) { micro.load(smem + buf * T::STAGE, s); };
    auto mma_step = [&](int s) { micro.mma(s, acc); };
    // all but the last step of the stage `buf`; on entry the fragments of its step 0 have been read
    auto steps_but_last = [&](int buf) {
#pragma unroll
        for (int s = 0; s + 1 < Micro::STEPS; ++s) {
            load_frags(buf, s + 1);
            mma_step(s);
            __builtin_amdgcn_sched_barrier(0);   // keep each step's reads and MFMAs together
        }
    };
    constexpr int LAST = Micro::STEPS - 1;       // the last step of a stage

    // ---- K loop over NSTAGE LDS stages.  When the LDS reads of step i's last fragments have been
    // issued, the wave waits for its transfers of step i+1, meets the others at the barrier (now
    // step i+1 is visible to all, and nobody reads the stage of step i any more), refills that stage
    // with step i+NSTAGE, starts reading step i+1 and only then issues the last MFMAs of step i,
    // which cover the latency of those reads.  The first `nfast` steps of this workgroup are direct
    // transfers only; the hot loop runs while every step in flight is one of them.
    constexpr int NS = T::NSTAGE;
    int nfast = 0;
    if (tile_fast_a && tile_fast_b) {
        nfast = p.K / BK - kt_begin;
        nfast = nfast < 0 ? 0 : (nfast > nkt ? nkt : nfast);
    }
    if (nkt > 0) {
#pragma unroll
        for (int t = 0; t < NS; ++t)
            if (t < nkt) stage_tiles(kt_begin + t, t);
        wait_transfers<0>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        load_frags(0, 0);
        int buf = 0;
        int i = 0;
        for (; i + NS < nfast; ++i) {
            const int nxt = (buf + 1 == NS) ? 0 : buf + 1;
            steps_but_last(buf);
            // transfers complete in order: step i+1 is done when at most those of the NS-2 later
            // steps are outstanding; lgkmcnt(0): this wave's reads of stage `buf` have returned
            wait_transfers<(NS - 2) * T::INST>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            stage_dma(kt_begin + i + NS, buf);
            load_frags(nxt, 0);
            __builtin_amdgcn_sched_barrier(0);
            mma_step(LAST);
            buf = nxt;
        }
        for (; i < nkt; ++i) {
            const int nxt = (buf + 1 == NS) ? 0 : buf + 1;
            steps_but_last(buf);
            if (i + 1 < nkt) {
                wait_transfers<0>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (i + NS < nkt) stage_tiles(kt_begin + i + NS, buf);
                load_frags(nxt, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            mma_step(LAST);
            buf = nxt;
        }
    }

    Micro::store(acc, p, m0, n0, wm0, wn0, lane, z, m_own, n_own);
}

}  // namespace mig
