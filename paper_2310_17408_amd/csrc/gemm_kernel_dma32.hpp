// fp32 workgroup-tile GEMM kernel for gfx950 with global -> LDS transfers as the
// packing step (Pack A / Pack B of the paper's Fig. "Pseudo-code of the BLIS
// base GEMM algorithm") and several K steps in flight.
//
// An fp32 MFMA fragment is one float per lane, so the M-contiguous operand A
// needs no transpose: it is staged as it lies in memory (tile row k, BM floats
// of M) and a lane reads, for one k, the TM consecutive m it owns in one LDS
// read.  The wave tile is therefore interleaved in M: lane l of the 32 owns
// m = TM*l .. TM*l+TM-1, block bm of the wave tile is {TM*l + bm}, and in the
// epilogue a lane stores TM consecutive floats of a column of C.
// The K-contiguous operand B is staged row by row (tile row n, 4*BK bytes of
// K, chunks XOR-swizzled as in gemm_kernel_dma.hpp) and read 16 bytes (4
// consecutive k) at a time; those 4 k feed 4 MFMA instructions.
//
// Operands whose rows are 16-byte aligned move 16 bytes per lane and transfer;
// fp32 rows with any other leading dimension are still 4-byte aligned and move
// 4 bytes per lane, so that also the im2row shapes with odd K (K-contiguous
// rows of 147 floats) are staged without registers.  Edge tiles and a partial
// last K step go through guarded loads and registers into the same layout.
//
// IM2ROW: the K-contiguous operand B is the im2row matrix of a channels-last image (paper Sec.
// "Rectangular Matrices"), staged from the image in place.  Cin is a multiple of the K step, so a
// step lies inside one filter tap and a tile row (an output pixel) is one 16-byte-aligned run of the
// image.  Every lane always issues its transfer (the counting of outstanding transfers relies on
// it): a lane whose tap falls outside the image reads the nearest pixel inside instead and, once
// its transfer has landed, overwrites those 16 bytes of LDS with zeros before the barrier that
// publishes the stage.
//
// With NSTAGE stages, NSTAGE-1 K steps are in flight while one is multiplied;
// a short K loop (the im2row GEMMs with K of a few hundred) is fetched whole
// before the first MFMA.
#pragma once
#include "gemm_kernel_dma.hpp"
#include <type_traits>

namespace mig {

typedef float v2f __attribute__((ext_vector_type(2)));

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int KSTEPS_, int NSTAGE_, int MINB_>
struct Dma32Tile {
    typedef F32 DT;
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, MINB = MINB_;
    static constexpr int KSTEPS = KSTEPS_, NSTAGE = NSTAGE_;
    static constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int BK = 8 * KSTEPS;              // floats of K per stage
    static constexpr int A_ROWB = BM * 4, A_BYTES = BK * A_ROWB;
    static constexpr int B_ROWB = BK * 4, B_BYTES = BN * B_ROWB;
    static constexpr int B_CPR = 2 * KSTEPS;           // 16-byte chunks per B row
    static constexpr int B_RP256 = 16 / B_CPR;         // B rows per 256 bytes
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NSTAGE * STAGE;
    static constexpr int A_BLK = A_BYTES / 1024, B_BLK = B_BYTES / 1024;   // 1 KiB transfer blocks per stage
    static constexpr int A_J = (A_BLK + NW - 1) / NW, B_J = (B_BLK + NW - 1) / NW;
    static constexpr int A_CPR = A_ROWB / 16;          // 16-byte chunks per k-row of A
    static constexpr int A_R4 = 1024 / A_ROWB;         // k-rows per 1 KiB block
    static constexpr int B_R4 = 1024 / B_ROWB;         // B rows per 1 KiB block
    static_assert(KSTEPS == 2 || KSTEPS == 4, "a B row holds 4 or 8 chunks");
    static_assert(TM == 1 || TM == 2 || TM == 4, "a lane reads 1, 2 or 4 consecutive m");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tiles are made of 32x32 blocks");
    static_assert(A_ROWB <= 1024 && 1024 % A_ROWB == 0 && A_ROWB % 256 == 0, "A rows must tile 1 KiB and 256 B blocks");
    static_assert(A_BYTES % 1024 == 0 && B_BYTES % 1024 == 0, "stages are made of 1 KiB blocks");
    static_assert(NW % 2 == 0, "the B swizzle of a lane must not depend on the block index");
    static_assert(NSTAGE >= 2, "at least one K step in flight");
};

// 256-byte global -> LDS transfer: lane l writes LDS bytes [lds_addr + 4*l, +4).
__device__ __forceinline__ void lds_dma4(const void *base, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_off), "s"(base)
                 : "memory");
}

// Wait until at most `allowed` vector-memory operations of this wave are outstanding (rounded
// down to a value the instruction can encode from a constant), and no LDS operations.
__device__ __forceinline__ void wait_transfers_upto(int allowed)
{
    if (allowed >= 48) wait_transfers<48>();
    else if (allowed >= 32) wait_transfers<32>();
    else if (allowed >= 24) wait_transfers<24>();
    else if (allowed >= 16) wait_transfers<16>();
    else if (allowed >= 12) wait_transfers<12>();
    else if (allowed >= 8) wait_transfers<8>();
    else if (allowed >= 6) wait_transfers<6>();
    else if (allowed >= 4) wait_transfers<4>();
    else if (allowed >= 3) wait_transfers<3>();
    else if (allowed >= 2) wait_transfers<2>();
    else if (allowed >= 1) wait_transfers<1>();
    else wait_transfers<0>();
}

// The fp32 micro-kernel of the direct kernels and the fragment reads that feed it, shared by the
// GEMM kernel and by the solo-mode benchmark.  A fragment step is 8 consecutive k = 4 MFMAs per block.
template <class T>
struct Dma32Micro {
    typedef v16f accv;
    static constexpr int TM = T::TM, TN = T::TN, A_ROWB = T::A_ROWB, B_ROWB = T::B_ROWB;
    // the fragments of one step: for each of 4 MFMAs the TM floats of m this lane owns, and per
    // block column 4 consecutive k of its row n
    struct aset { float v[4][TM]; };
    struct bset { v4f v[TN]; };
    uint32_t aoff, boff[T::KSTEPS];

    __device__ __forceinline__ void init(int lane, int wm0, int wn0)
    {
        const int frow = lane & 31, fgrp = lane >> 5;
        const int x = (frow / T::B_RP256) % T::B_CPR;
#pragma unroll
        for (int s = 0; s < T::KSTEPS; ++s)
            boff[s] = T::A_BYTES + (wn0 + frow) * B_ROWB + (((2 * s + fgrp) ^ x) << 4);
        // A: k-row 8*s + 4*fgrp + t, floats wm0 + TM*frow ... + TM-1
        aoff = (4 * fgrp) * A_ROWB + (wm0 + TM * frow) * 4;
    }

    __device__ __forceinline__ void load(const unsigned char *stage, int s, aset &xa, bset &xb) const
    {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const unsigned char *q = stage + aoff + (8 * s + t) * A_ROWB;
            if constexpr (TM == 1) {
                xa.v[t][0] = *(const float *)q;
            } else if constexpr (TM == 2) {
                v2f v = *(const v2f *)q;
                xa.v[t][0] = v[0]; xa.v[t][1] = v[1];
            } else {
                v4f v = *(const v4f *)q;
                xa.v[t][0] = v[0]; xa.v[t][1] = v[1]; xa.v[t][2] = v[2]; xa.v[t][3] = v[3];
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) xb.v[j] = *(const v4f *)(stage + boff[s] + j * 32 * B_ROWB);
    }

    static __device__ __forceinline__ void mma(aset &xa, bset &xb, accv (&acc)[TM][TN])
    {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(xb.v[j][t], xa.v[t][i], acc[i][j], 0, 0, 0);
    }
};

// Position in K of an im2row K step: filter tap (r, s) and first channel c, advanced one step at a time.
struct TapIter {
    int r, s, c;
    __device__ __forceinline__ void start(int k, const Im2row &g)
    {
        const int tap = k / g.Cin;
        c = k - tap * g.Cin;
        r = tap / g.kw;
        s = tap - r * g.kw;
    }
    __device__ __forceinline__ void advance(int bk, const Im2row &g)
    {
        c += bk;
        if (c == g.Cin) {
            c = 0;
            if (++s == g.kw) { s = 0; ++r; }
        }
    }
};

template <class T, bool IM2ROW = false>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel_dma32(const Params p)
{
    typedef F32 DT;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NW = T::NW, NS = T::NSTAGE;
    constexpr int TM = T::TM, TN = T::TN, A_ROWB = T::A_ROWB, B_ROWB = T::B_ROWB;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(MIG_LDS unsigned char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % T::WAVES_M) * T::WM;
    const int wn0 = (wave / T::WAVES_M) * T::WN;

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    // A tile that sticks out of C is moved back so that it ends at the edge (when the matrix is at
    // least one tile wide): it then reads only rows that exist, through the same transfers as an
    // interior tile, and stores only the part no other tile owns (from m_own, n_own on).
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
    // tile rows all inside the matrix, and a lane's 32-bit byte offset inside a block cannot overflow
    const bool in_a = (m0 + BM <= p.M) && (p.lda < (1 << 26));
    const bool in_b = IM2ROW || ((n0 + BN <= p.N) && (p.ldb < (1 << 26)));   // IM2ROW: rows beyond N read row N-1, as zeros
    // rows are 16-byte aligned (a moved tile of A may start at any m)
    const bool a16 = p.vecA != 0 && (m0 % 4 == 0), b16 = IM2ROW || p.vecB != 0;

    // ---- staging.  A stage is cut into 1 KiB blocks, block `blk` of an operand belongs to wave
    // blk % NW.  16-byte path: one transfer per block.  4-byte path: four 256-byte transfers.
    // A block: A_R4 k-rows; lane -> (row, 16-byte chunk), no swizzle.
    const int a_row_in = lane / T::A_CPR, a_ch = lane % T::A_CPR;
    const uint32_t a_off16 = (uint32_t)(((int64_t)a_row_in * p.lda + a_ch * 4) * 4);
    // B block: B_R4 rows; lane -> (row, physical chunk); the logical chunk undoes the row's swizzle,
    // which is the same for blocks wave, wave+NW, ... (NW even)
    const int b_row_in = lane / T::B_CPR, b_pch = lane % T::B_CPR;
    const int b_ch = b_pch ^ (((wave * T::B_R4 + b_row_in) / T::B_RP256) % T::B_CPR);
    const uint32_t b_off16 = (uint32_t)(((int64_t)b_row_in * p.ldb + b_ch * 4) * 4);
    static_assert(T::B_R4 % T::B_RP256 == 0 && (NW * T::B_R4 / T::B_RP256) % T::B_CPR == 0,
                  "B swizzle must repeat every NW blocks");

    // IM2ROW: the pixels this lane stages (one per transfer j): image row / column of the pixel's tap
    // (0, 0), its image (b*H, so that an image row index is one addition), whether the row exists
    constexpr int PJ = IM2ROW ? T::B_J : 1;
    int pix_ih0[PJ], pix_iw0[PJ], pix_bh[PJ];
    bool pix_ok[PJ];
    if constexpr (IM2ROW) {
        const int per_image = p.conv.Hout * p.conv.Wout;
#pragma unroll
        for (int j = 0; j < T::B_J; ++j) {
            int n = n0 + (wave + NW * j) * T::B_R4 + b_row_in;
            pix_ok[j] = n < p.N;
            n = n < p.N ? n : p.N - 1;
            const int b = n / per_image, rem = n - b * per_image;
            const int oh = rem / p.conv.Wout, ow = rem - oh * p.conv.Wout;
            pix_ih0[j] = oh * p.conv.stride_h - p.conv.pad_h;
            pix_iw0[j] = ow * p.conv.stride_w - p.conv.pad_w;
            pix_bh[j] = b * p.conv.H;
        }
    }
    TapIter tap_stage, tap_fix;                                 // next step to stage / to publish
    if constexpr (IM2ROW) {
        tap_stage.start(kt_begin * BK, p.conv);
        tap_fix = tap_stage;
    }
    // all B transfers of one K step: the lane's chunk of its pixel's tap, clamped into the image
    auto stage_b_im2row = [&](int buf) {
#pragma unroll
        for (int j = 0; j < T::B_J; ++j) {
            const int blk = wave + NW * j;
            if (T::B_BLK % NW != 0 && blk >= T::B_BLK) break;
            int ih = pix_ih0[j] + tap_stage.r, iw = pix_iw0[j] + tap_stage.s;
            ih = ih < 0 ? 0 : (ih >= p.conv.H ? p.conv.H - 1 : ih);
            iw = iw < 0 ? 0 : (iw >= p.conv.W ? p.conv.W - 1 : iw);
            const uint32_t off = (uint32_t)((((int64_t)(pix_bh[j] + ih) * p.conv.W + iw) * p.conv.Cin + tap_stage.c + b_ch * 4) * 4);
            lds_dma16(B, off, lds_base + buf * T::STAGE + T::A_BYTES + blk * 1024);
        }
        tap_stage.advance(BK, p.conv);
    };
    // after this wave's transfers of the step have landed: zeros where the tap is outside the image
    auto fix_b_im2row = [&](int buf) {
#pragma unroll
        for (int j = 0; j < T::B_J; ++j) {
            const int blk = wave + NW * j;
            if (T::B_BLK % NW != 0 && blk >= T::B_BLK) break;
            const bool inside = pix_ok[j] && (uint32_t)(pix_ih0[j] + tap_fix.r) < (uint32_t)p.conv.H &&
                                (uint32_t)(pix_iw0[j] + tap_fix.s) < (uint32_t)p.conv.W;
            if (!inside) *(v4i *)(smem + buf * T::STAGE + T::A_BYTES + blk * 1024 + lane * 16) = v4i{0, 0, 0, 0};
        }
        tap_fix.advance(BK, p.conv);
        __builtin_amdgcn_s_waitcnt(0xc07f);                     // lgkmcnt(0): the zeros are in LDS before the barrier
    };

    // number of transfer instructions this wave issues per fully direct stage (for the counter)
    int my_blocks = 0;
#pragma unroll
    for (int j = 0; j < T::A_J; ++j) my_blocks += (wave + NW * j < T::A_BLK) ? (a16 ? 1 : 4) : 0;
#pragma unroll
    for (int j = 0; j < T::B_J; ++j) my_blocks += (wave + NW * j < T::B_BLK) ? (b16 ? 1 : 4) : 0;
    my_blocks = __builtin_amdgcn_readfirstlane(my_blocks);

    auto stage_a = [&](int kt, int buf, bool direct) {
        const int k0 = kt * BK;
#pragma unroll
        for (int j = 0; j < T::A_J; ++j) {
            const int blk = wave + NW * j;
            if (T::A_BLK % NW != 0 && blk >= T::A_BLK) break;
            const uint32_t loff = buf * T::STAGE + blk * 1024;
            const int krow = blk * T::A_R4;                     // first tile-local k-row of the block
            if (direct && a16) {
                lds_dma16(A + (int64_t)(k0 + krow) * p.lda + m0, a_off16, lds_base + loff);
            } else if (direct) {
                // 4-byte transfers: quarter q of the block is 256 bytes = 64 floats of one k-row
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int byte = q * 256;                   // offset inside the block
                    const int r = krow + byte / A_ROWB, mofs = (byte % A_ROWB) / 4;
                    lds_dma4(A + (int64_t)(k0 + r) * p.lda + m0 + mofs, (uint32_t)lane * 4, lds_base + loff + byte);
                }
            } else {
                const int k = k0 + krow + a_row_in, m = m0 + a_ch * 4;
                int valid = (k < p.K) ? (p.M - m) : 0;
                valid = valid > 4 ? 4 : valid;
                *(v4i *)(smem + loff + lane * 16) = guarded_chunk<DT>(A + (int64_t)k * p.lda + m, valid);
            }
        }
    };
    auto stage_b = [&](int kt, int buf, bool direct) {
        const int k0 = kt * BK;
#pragma unroll
        for (int j = 0; j < T::B_J; ++j) {
            const int blk = wave + NW * j;
            if (T::B_BLK % NW != 0 && blk >= T::B_BLK) break;
            const uint32_t loff = buf * T::STAGE + T::A_BYTES + blk * 1024;
            const int row0 = blk * T::B_R4;                     // first tile row n of the block
            if (direct && b16) {
                lds_dma16(B + (int64_t)(n0 + row0) * p.ldb + k0, b_off16, lds_base + loff);
            } else if (direct) {
                // 4-byte transfers: lane l fills dword l of a 256-byte quarter = rows of B_ROWB bytes
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int dw = q * 64 + lane;               // dword inside the block
                    const int r = row0 + dw / (B_ROWB / 4), pos = dw % (B_ROWB / 4);
                    const int ch = (pos >> 2) ^ ((r / T::B_RP256) % T::B_CPR);
                    const uint32_t goff = (uint32_t)(((int64_t)(dw / (B_ROWB / 4)) * p.ldb + ch * 4 + (pos & 3)) * 4);
                    lds_dma4(B + (int64_t)(n0 + row0) * p.ldb + k0, goff, lds_base + loff + q * 256);
                }
            } else {
                const int n = n0 + row0 + b_row_in, k = k0 + b_ch * 4;
                int valid = (n < p.N) ? (p.K - k) : 0;
                valid = valid > 4 ? 4 : valid;
                *(v4i *)(smem + loff + lane * 16) = guarded_chunk<DT>(B + (int64_t)n * p.ldb + k, valid);
            }
        }
    };
    auto stage_tiles = [&](int kt, int buf) {
        const bool kfull = ((kt + 1) * BK <= p.K);
        stage_a(kt, buf, in_a && kfull);
        if constexpr (IM2ROW) stage_b_im2row(buf);              // steps are staged in order
        else stage_b(kt, buf, in_b && kfull);
    };

    const int frow = lane & 31, fgrp = lane >> 5;
    Dma32Micro<T> micro;
    micro.init(lane, wm0, wn0);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // ---- the micro-kernel, fragments double buffered in registers
    typename Dma32Micro<T>::aset fa[2];
    typename Dma32Micro<T>::bset fb[2];
    auto load_frags = [&](int buf, int s, typename Dma32Micro<T>::aset &xa, typename Dma32Micro<T>::bset &xb) {
        micro.load(smem + buf * T::STAGE, s, xa, xb);
    };
    auto mma_step = [&](typename Dma32Micro<T>::aset &xa, typename Dma32Micro<T>::bset &xb) {
        Dma32Micro<T>::mma(xa, xb, acc);
    };
    auto steps_but_last = [&](int buf) {
#pragma unroll
        for (int s = 0; s + 1 < T::KSTEPS; ++s) {
            load_frags(buf, s + 1, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            mma_step(fa[s & 1], fb[s & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    constexpr int LAST = (T::KSTEPS - 1) & 1;

    // ---- K loop (same rotation as in gemm_kernel_dma.hpp): the barrier that ends step i sits
    // between the LDS reads and the MFMAs of its last fragment step.
    int nfast = 0;                      // leading steps of this workgroup that are direct transfers only
    if (in_a && in_b) {
        nfast = p.K / BK - kt_begin;
        nfast = nfast < 0 ? 0 : (nfast > nkt ? nkt : nfast);
    }
    // Direct staging of one full K step with everything a lane or wave needs precomputed: per-wave
    // base pointers that advance by a constant per step, per-lane offsets that never change.  The
    // transfer width of each operand (16 or 4 bytes per lane) is a compile-time choice here, so the
    // hot loop below carries no branches.
    const unsigned char *a_wave = (const unsigned char *)(A + (int64_t)(wave * T::A_R4) * p.lda + m0);
    const unsigned char *b_wave = (const unsigned char *)(B + (int64_t)(n0 + wave * T::B_R4) * p.ldb);
    const int64_t a_step = (int64_t)BK * p.lda * 4, b_step = (int64_t)BK * 4;
    const int64_t a_blk = (int64_t)NW * T::A_R4 * p.lda * 4, b_blk = (int64_t)NW * T::B_R4 * p.ldb * 4;
    int64_t a_q[4];          // 4-byte path of A: quarter q of a block starts this many bytes after the block
    uint32_t b_q[4];         // 4-byte path of B: this lane's byte offset from the block's first row, quarter q
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a_q[q] = ((int64_t)((q * 256) / A_ROWB) * p.lda + ((q * 256) % A_ROWB) / 4) * 4;
        const int dw = q * 64 + lane;
        const int rin = dw / (B_ROWB / 4), pos = dw % (B_ROWB / 4);
        const int ch = (pos >> 2) ^ (((wave * T::B_R4 + rin) / T::B_RP256) % T::B_CPR);
        b_q[q] = (uint32_t)(((int64_t)rin * p.ldb + ch * 4 + (pos & 3)) * 4);
    }
    auto stage_direct = [&](auto a16c, auto b16c, int kt, int buf) {
        const unsigned char *ab = a_wave + (int64_t)kt * a_step;
        const unsigned char *bb = b_wave + (int64_t)kt * b_step;
        const uint32_t la = lds_base + buf * T::STAGE + wave * 1024;
#pragma unroll
        for (int j = 0; j < T::A_J; ++j) {
            if (T::A_BLK % NW != 0 && wave + NW * j >= T::A_BLK) break;
            if constexpr (decltype(a16c)::value) {
                lds_dma16(ab + j * a_blk, a_off16, la + j * NW * 1024);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    lds_dma4(ab + j * a_blk + a_q[q], (uint32_t)lane * 4, la + j * NW * 1024 + q * 256);
            }
        }
        if constexpr (IM2ROW) {
            stage_b_im2row(buf);
            return;
        }
#pragma unroll
        for (int j = 0; j < T::B_J; ++j) {
            if (T::B_BLK % NW != 0 && wave + NW * j >= T::B_BLK) break;
            if constexpr (decltype(b16c)::value) {
                lds_dma16(bb + j * b_blk, b_off16, la + T::A_BYTES + j * NW * 1024);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    lds_dma4(bb + j * b_blk, b_q[q], la + T::A_BYTES + j * NW * 1024 + q * 256);
            }
        }
    };

    int buf = 0, i = 0;
    // hot loop: runs while the step it stages (i + NS) and all steps in flight are direct
    auto hot_loop = [&](auto a16c, auto b16c) {
        for (; i + NS < nfast; ++i) {
            const int nxt = (buf + 1 == NS) ? 0 : buf + 1;
            steps_but_last(buf);
            wait_transfers_upto((NS - 2) * my_blocks);
            if constexpr (IM2ROW) fix_b_im2row(nxt);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            stage_direct(a16c, b16c, kt_begin + i + NS, buf);
            load_frags(nxt, 0, fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            mma_step(fa[LAST], fb[LAST]);
            buf = nxt;
        }
    };

    if (nkt > 0) {
#pragma unroll
        for (int t = 0; t < NS; ++t)
            if (t < nkt) stage_tiles(kt_begin + t, t);
        // step 0 is done when only the other staged steps are outstanding, if all of them are direct
        {
            const int staged = nkt < NS ? nkt : NS;
            wait_transfers_upto(staged <= nfast ? (staged - 1) * my_blocks : 0);
        }
        if constexpr (IM2ROW) fix_b_im2row(0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        load_frags(0, 0, fa[0], fb[0]);
        typedef std::integral_constant<bool, true> yes;
        typedef std::integral_constant<bool, false> no;
        if (a16 && b16) hot_loop(yes(), yes());
        else if (a16) hot_loop(yes(), no());
        else if (b16) hot_loop(no(), yes());
        else hot_loop(no(), no());
        for (; i < nkt; ++i) {
            const int nxt = (buf + 1 == NS) ? 0 : buf + 1;
            steps_but_last(buf);
            if (i + 1 < nkt) {
                // steps i+1 .. min(i+NS-1, nkt-1) are staged; step i+1 is done when only the later
                // ones are outstanding (transfers complete in order), if all of them are direct
                int last = i + NS - 1;
                last = last < nkt - 1 ? last : nkt - 1;
                wait_transfers_upto(last < nfast ? (last - (i + 1)) * my_blocks : 0);
                if constexpr (IM2ROW) fix_b_im2row(nxt);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (i + NS < nkt) stage_tiles(kt_begin + i + NS, buf);
                load_frags(nxt, 0, fa[0], fb[0]);
                __builtin_amdgcn_sched_barrier(0);
            }
            mma_step(fa[LAST], fb[LAST]);
            buf = nxt;
        }
    }

    // ---- epilogue: a lane holds, per block column n, the TM consecutive rows m it owns
    {
        const bool interior = (m0 + BM <= p.M) && (n0 + BN <= p.N) && m0 == m_own && n0 == n_own;
        const float alpha = __builtin_bit_cast(float, p.alpha_bits);
        const float beta = __builtin_bit_cast(float, p.beta_bits);
        const bool use_beta = p.use_beta != 0;
        const int mrow = m0 + wm0 + TM * frow;
        const bool vec_c = (TM > 1) && interior && ((p.ldc % TM) == 0) && (((uintptr_t)p.C % (TM * 4)) == 0) &&
                           p.split <= 1;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int n = n0 + wn0 + 32 * j + 8 * (v >> 2) + 4 * fgrp + (v & 3);
                if (p.split > 1) {
                    float *ws = (float *)p.ws + ((int64_t)z * p.N + n) * p.M + mrow;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (interior || (mrow + i >= m_own && mrow + i < p.M && n >= n_own && n < p.N)) ws[i] = acc[i][j][v];
                } else {
                    float *c = (float *)p.C + (int64_t)n * p.ldc + mrow;
                    if (vec_c) {
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
                    } else {
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            if (interior || (mrow + i >= m_own && mrow + i < p.M && n >= n_own && n < p.N)) {
                                float r = alpha * acc[i][j][v];
                                if (use_beta) r += beta * c[i];
                                c[i] = r;
                            }
                        }
                    }
                }
            }
        }
    }
}

}  // namespace mig
