// Workgroup-tile GEMM kernel for gfx950 (MI355X): the macro-kernel and the
// micro-kernel of the paper's Fig. "Pseudo-code of the BLIS base GEMM
// algorithm", re-mapped to the GPU.
//
//   loops L1 (jc) and L3 (ic)  -> the grid: one workgroup per BM x BN tile of C
//   loop  L2 (pc)              -> the K loop of a workgroup, in steps of BK
//                                 (one 128-byte row segment per step), and,
//                                 when asked for, split over blockIdx.y
//   Pack A / Pack B            -> staging of the operand tiles into LDS, both
//                                 stored row by row with K contiguous, so that
//                                 the micro-kernel reads its operands with unit
//                                 stride (the paper's reason for packing)
//   loops L4 (jr) and L5 (ir)  -> the waves of the workgroup and the 32 x 32
//                                 MFMA blocks of each wave tile
//   micro-kernel L6            -> a chain of MFMA instructions that keeps the
//                                 wave's block of C in registers over the whole
//                                 K loop, as C_reg does in the paper's Sec.
//                                 "Micro-kernel Generation"
//
// Canonical problem (the host swaps operands for row-major callers):
//   C is M x N column-major, element (m,n) at C[m + n*ldc];
//   A is M x K with M contiguous, element (m,k) at A[m + k*lda];
//   B is K x N with K contiguous, element (k,n) at B[k + n*ldb].
// Transposed operands (this kernel only): A with K contiguous, element (m,k) at A[k + m*lda], and
// B with N contiguous, element (k,n) at B[n + k*ldb].
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_table.h"

namespace mig {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
// the same vectors at element alignment only: gfx950 serves global loads at any alignment
// (the amdhsa target runs with unaligned access enabled), at the price of a second cache access
// when a load straddles a line
typedef int v4i_u __attribute__((ext_vector_type(4), aligned(1)));
typedef int v2i_u __attribute__((ext_vector_type(2), aligned(1)));
typedef int i32_u __attribute__((aligned(1)));

// ---------------------------------------------------------------- data types
struct F32 {
    typedef float elt;
    typedef float acc_t;
    typedef v16f accv;
    static constexpr int ES = 4;    // bytes per input element
    static constexpr int KCH = 4;   // K elements per 16-byte chunk
};
struct F16 {
    typedef uint16_t elt;
    typedef float acc_t;
    typedef v16f accv;
    static constexpr int ES = 2;
    static constexpr int KCH = 8;
};
struct BF16 {          // bfloat16 bit patterns in, fp32 accumulation; laid out like F16 everywhere
    typedef uint16_t elt;
    typedef float acc_t;
    typedef v16f accv;
    static constexpr int ES = 2;
    static constexpr int KCH = 8;
};
struct I8 {
    typedef int8_t elt;
    typedef int acc_t;
    typedef v16i accv;
    static constexpr int ES = 1;
    static constexpr int KCH = 16;
};

// One 16-byte fragment per lane and operand feeds 4 (fp32), 1 (fp16) or
// 1 (int8) MFMA instructions.  `rowop` is the operand whose tile rows become
// the rows of the 32 x 32 result block (held in registers), `colop` the one
// whose rows become its columns (one per lane).
template <class DT> struct Mma;
template <> struct Mma<F32> {
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v16f &c) {
        v4f a = __builtin_bit_cast(v4f, rowop), b = __builtin_bit_cast(v4f, colop);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], c, 0, 0, 0);
    }
};
template <> struct Mma<F16> {
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v16f &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, rowop),
                                                   __builtin_bit_cast(v8h, colop), c, 0, 0, 0);
    }
};
template <> struct Mma<BF16> {
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v16f &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, rowop),
                                                    __builtin_bit_cast(v8bf, colop), c, 0, 0, 0);
    }
};
template <> struct Mma<I8> {
    static __device__ __forceinline__ void run(const v4i &rowop, const v4i &colop, v16i &c) {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(rowop, colop, c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------- register transposes
// The A operand arrives with M contiguous: a lane loads KCH vectors, one per k,
// of MB consecutive m each, and turns them into MB chunks of KCH consecutive k.
// raw[kk][w] is 32-bit word w of the vector loaded for k offset kk.
template <class DT, int MB> struct Transpose;

template <int MB> struct Transpose<F32, MB> {     // MB = 2 or 4
    static __device__ __forceinline__ v4i chunk(const int (&raw)[4][MB], int c) {
        v4i o;
        o[0] = raw[0][c]; o[1] = raw[1][c]; o[2] = raw[2][c]; o[3] = raw[3][c];
        return o;
    }
};

template <int MB> struct Transpose<F16, MB> {     // MB = 2, 4 or 8
    static __device__ __forceinline__ v4i chunk(const int (&raw)[8][MB / 2], int c) {
        v4i o;
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {
            uint32_t x = (uint32_t)raw[2 * kp][c >> 1], y = (uint32_t)raw[2 * kp + 1][c >> 1];
            o[kp] = (c & 1) ? (int)((x >> 16) | (y & 0xffff0000u)) : (int)((x & 0xffffu) | (y << 16));
        }
        return o;
    }
};

template <int MB> struct Transpose<BF16, MB> : Transpose<F16, MB> {};   // 16-bit elements move alike

__device__ __forceinline__ uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);   // bytes 0-3 index lo, 4-7 index hi
}

template <int MB> struct Transpose<I8, MB> {     // MB = 4 or 8
    static constexpr int WORDS = MB / 4;
    // all MB chunks at once: out[c] holds k = 0..15 of row c
    static __device__ __forceinline__ void all(const int (&raw)[16][WORDS], v4i (&out)[MB]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int w = 0; w < WORDS; ++w) {
                uint32_t r0 = raw[4 * q][w], r1 = raw[4 * q + 1][w], r2 = raw[4 * q + 2][w], r3 = raw[4 * q + 3][w];
                uint32_t t0 = byte_perm(r1, r0, 0x05010400u);   // r0.b0 r1.b0 r0.b1 r1.b1
                uint32_t t1 = byte_perm(r1, r0, 0x07030602u);   // r0.b2 r1.b2 r0.b3 r1.b3
                uint32_t t2 = byte_perm(r3, r2, 0x05010400u);
                uint32_t t3 = byte_perm(r3, r2, 0x07030602u);
                out[4 * w + 0][q] = (int)byte_perm(t2, t0, 0x05040100u);
                out[4 * w + 1][q] = (int)byte_perm(t2, t0, 0x07060302u);
                out[4 * w + 2][q] = (int)byte_perm(t3, t1, 0x05040100u);
                out[4 * w + 3][q] = (int)byte_perm(t3, t1, 0x07060302u);
            }
        }
    }
};

// ---------------------------------------------------------------- the kernel
template <class DT_, int BM_, int BN_, int WAVES_M_, int WAVES_N_, int MB_, int MINB_>
struct Tile {
    typedef DT_ DT;
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, MB = MB_, MINB = MINB_;
    static constexpr int NT = WAVES_M * WAVES_N * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int BK = 128 / DT::ES;          // K elements per step
    static constexpr int ROWB = 128 + 16;            // LDS bytes per tile row (16 bytes of padding)
    static constexpr int STAGE = (BM + BN) * ROWB;   // one LDS buffer
    static constexpr int LDS_BYTES = 2 * STAGE;      // double buffered
    static constexpr int AW = MB * DT::ES / 4;       // 32-bit words per loaded A vector
    static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tiles are made of 32x32 blocks");
};

// Which tile of C a workgroup owns (loops L1 and L3).  Workgroups are dealt to
// the 8 XCDs round-robin, so each XCD is given a contiguous range of the tile
// order; within that order tiles run down columns of `group_m` tiles, so that
// workgroups resident together share A and B panels in their XCD's L2.
__device__ __forceinline__ void tile_coords(const Params &p, int bid, int &tm, int &tn)
{
    int pid = bid;
    const int ntiles = p.tiles_m * p.tiles_n;
    if (p.xcd_remap) {
        const int q = ntiles >> 3, r = ntiles & 7;
        const int xcd = pid & 7, idx = pid >> 3;
        pid = xcd * q + (xcd < r ? xcd : r) + idx;
    }
    const int group = p.group_m * p.tiles_n;
    const int gid = pid / group;
    const int first_m = gid * p.group_m;
    const int gm = (p.tiles_m - first_m) < p.group_m ? (p.tiles_m - first_m) : p.group_m;
    tm = first_m + (pid % group) % gm;
    tn = (pid % group) / gm;
}

// C kept in 16 bits (binary16 or bfloat16; paper Sec. "Data types": the storage type of an operand is a
// parameter of the micro-kernel): the update is evaluated in fp32 and rounded once, to nearest even.
__device__ __forceinline__ float narrow_load(int c_type, const void *C, int64_t idx)
{
    const uint16_t b = ((const uint16_t *)C)[idx];
    if (c_type == C_F16) return (float)__builtin_bit_cast(_Float16, b);
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
__device__ __forceinline__ void narrow_store(int c_type, void *C, int64_t idx, float v)
{
    uint16_t b;
    if (c_type == C_F16) {
        b = __builtin_bit_cast(uint16_t, (_Float16)v);
    } else {
        const uint32_t u = __builtin_bit_cast(uint32_t, v);
        b = (v != v) ? (uint16_t)((u >> 16) | 0x40u) : (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
    ((uint16_t *)C)[idx] = b;
}
// C(idx) <- alpha*a + beta*C(idx) for a float accumulator, C stored as p.c_type says
__device__ __forceinline__ void update_c(const Params &p, int64_t idx, float a, float alpha, float beta, bool use_beta)
{
    float o = alpha * a;
    if (p.c_type == C_WIDE) {
        float *c = (float *)p.C + idx;
        if (use_beta) o += beta * (*c);
        *c = o;
    } else {
        if (use_beta) o += beta * narrow_load(p.c_type, p.C, idx);
        narrow_store(p.c_type, p.C, idx, o);
    }
}

// Epilogue: C <- alpha*acc + beta*C, or the raw partial tile into the workspace
// when K is split.  In every 32 x 32 block a lane holds one row m and the 16
// columns n = 8*(v/4) + 4*(lane/32) + v%4, so the 32 lanes of a half-wave write
// 128 contiguous bytes of a column of C.
// A tile that was moved back to end at the edge of C (m0 < m_own or n0 < n_own) stores only the
// rows from m_own and the columns from n_own on; the rest belongs to its neighbours.
template <class DT, int TM, int TN>
__device__ __forceinline__ void store_tile(typename DT::accv (&acc)[TM][TN], const Params &p, int m0, int n0, int BM,
                                           int BN, int wm0, int wn0, int lane, int z, int m_own, int n_own)
{
    typedef typename DT::acc_t acc_t;
    const int frow = lane & 31, fgrp = lane >> 5;
    const bool interior = (m0 + BM <= p.M) && (n0 + BN <= p.N) && m0 == m_own && n0 == n_own;
    const acc_t alpha = __builtin_bit_cast(acc_t, p.alpha_bits);
    const acc_t beta = __builtin_bit_cast(acc_t, p.beta_bits);
    const bool use_beta = p.use_beta != 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm0 + 32 * i + frow;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int n = n0 + wn0 + 32 * j + 8 * (v >> 2) + 4 * fgrp + (v & 3);
                if (interior || (m >= m_own && m < p.M && n >= n_own && n < p.N)) {
                    const acc_t a = acc[i][j][v];
                    if (p.split > 1) {
                        acc_t *ws = (acc_t *)p.ws;
                        ws[((int64_t)z * p.N + n) * p.M + m] = a;
                    } else {
                        acc_t *c = (acc_t *)p.C + (int64_t)n * p.ldc + m;
                        if constexpr (DT::ES == 1) {
                            uint32_t r = (uint32_t)alpha * (uint32_t)a;
                            if (use_beta) r += (uint32_t)beta * (uint32_t)(*c);
                            *c = (int)r;
                        } else if constexpr (DT::ES == 2) {
                            update_c(p, (int64_t)n * p.ldc + m, a, alpha, beta, use_beta);
                        } else {
                            float r = alpha * a;
                            if (use_beta) r += beta * (*c);
                            *c = r;
                        }
                    }
                }
            }
        }
    }
}

// The micro-kernel (loop L6) on one staged K step: the wave at (wm0, wn0) of the
// workgroup tile reads its operand fragments from the LDS buffer `stage` (tile
// rows of ROWB bytes, A rows first, then B rows; K contiguous) and updates its
// TM x TN blocks of C held in registers.  Each of the 4 fragment steps covers
// two 16-byte chunks of K: lanes 0-31 take the even chunk, lanes 32-63 the odd.
template <class T>
__device__ __forceinline__ void micro_kernel(const unsigned char *stage, int wm0, int wn0, int lane,
                                             typename T::DT::accv (&acc)[T::TM][T::TN])
{
    constexpr int ROWB = T::ROWB, TM = T::TM, TN = T::TN;
    const int frow = lane & 31, fgrp = lane >> 5;
    const unsigned char *pa = stage + (wm0 + frow) * ROWB + fgrp * 16;
    const unsigned char *pb = stage + (T::BM + wn0 + frow) * ROWB + fgrp * 16;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        v4i fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const v4i *)(pa + i * 32 * ROWB + s * 32);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *(const v4i *)(pb + j * 32 * ROWB + s * 32);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) Mma<typename T::DT>::run(fb[j], fa[i], acc[i][j]);
    }
}

// One operand tile of the staged kernel on its way global -> registers -> LDS: ROWS tile rows (m for
// A, n for B) of BK elements of K.  In memory the operand has either K contiguous (element (r, k) at
// src[r*ld + k]: the canonical B, or a transposed A) or its rows contiguous (element (r, k) at
// src[k*ld + r]: the canonical A, or a transposed B); in LDS it always ends up row by row with K
// contiguous (the packing step), the second kind through the register transposes above.
template <class T, int ROWS, bool K_CONTIGUOUS>
struct StagedOperand {
    typedef typename T::DT DT;
    typedef typename DT::elt elt;
    static constexpr int NT = T::NT, ROWB = T::ROWB, BK = T::BK, MB = T::MB, KCH = DT::KCH, ES = DT::ES;
    static constexpr int AW = T::AW;
    static constexpr int RBLKS = ROWS / MB;                         // blocks of MB rows
    static constexpr int BLOCKS = RBLKS * 8, CHUNKS = ROWS * 8;     // MB x KCH blocks / 16-byte chunks per tile
    static constexpr int IT = K_CONTIGUOUS ? (CHUNKS + NT - 1) / NT : (BLOCKS + NT - 1) / NT;
    int raw[IT][K_CONTIGUOUS ? 1 : KCH][K_CONTIGUOUS ? 4 : AW];

    static __device__ __forceinline__ uint32_t bits_of(const elt *src, int i)
    {
        if constexpr (ES == 4) return __builtin_bit_cast(uint32_t, src[i]);
        else if constexpr (ES == 2) return (uint16_t)src[i];
        else return (uint8_t)src[i];
    }

    // global -> registers for the K step that starts at k0; `r0` is the first row of the tile, `nrows`
    // and `K` bound the operand; `inside`: every row of the tile exists and the step is a full one
    __device__ __forceinline__ void load(const elt *__restrict__ src, int64_t ld, int r0, int k0, int nrows, int K,
                                         bool inside, int tid)
    {
        if constexpr (K_CONTIGUOUS) {
            // 16-byte chunks along k; 8 consecutive lanes cover one 128-byte row segment
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int cid = tid + it * NT;
                if (CHUNKS % NT != 0 && cid >= CHUNKS) continue;
                const int row = cid >> 3, ch = cid & 7;
                const int r = r0 + row, k = k0 + ch * KCH;
                const elt *q = src + (int64_t)r * ld + k;
                v4i v;
                if (inside || (r < nrows && k + KCH <= K)) {
                    v = *(const v4i_u *)q;                          // the whole chunk exists: one load at any alignment
                } else {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        uint32_t word = 0;
#pragma unroll
                        for (int e = 0; e < 4 / ES; ++e) {
                            const int ki = w * (4 / ES) + e;
                            const uint32_t bits = (r < nrows && k + ki < K) ? bits_of(q, ki) : 0u;
                            word |= bits << (8 * ES * e);
                        }
                        v[w] = (int)word;
                    }
                }
                raw[it][0][0] = v[0]; raw[it][0][1] = v[1]; raw[it][0][2] = v[2]; raw[it][0][3] = v[3];
            }
        } else {
            // blocks of MB rows x KCH k; consecutive lanes take consecutive rows
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int bid = tid + it * NT;
                if (BLOCKS % NT != 0 && bid >= BLOCKS) continue;
                const int rblk = bid % RBLKS, kch = bid / RBLKS;
                const int rb = r0 + rblk * MB;
#pragma unroll
                for (int kk = 0; kk < KCH; ++kk) {
                    const int k = k0 + kch * KCH + kk;
                    const elt *q = src + (int64_t)k * ld + rb;
                    if (inside || (k < K && rb + MB <= nrows)) {
                        if constexpr (AW == 4) {
                            const v4i v = *(const v4i_u *)q;
                            raw[it][kk][0] = v[0]; raw[it][kk][1] = v[1]; raw[it][kk][2] = v[2]; raw[it][kk][3] = v[3];
                        } else if constexpr (AW == 2) {
                            const v2i v = *(const v2i_u *)q;
                            raw[it][kk][0] = v[0]; raw[it][kk][1] = v[1];
                        } else {
                            raw[it][kk][0] = *(const i32_u *)q;
                        }
                        continue;
                    }
#pragma unroll
                    for (int w = 0; w < AW; ++w) {
                        uint32_t word = 0;
#pragma unroll
                        for (int e = 0; e < 4 / ES; ++e) {
                            const int ri = w * (4 / ES) + e;
                            const uint32_t bits = (k < K && rb + ri < nrows) ? bits_of(q, ri) : 0u;
                            word |= bits << (8 * ES * e);
                        }
                        raw[it][kk][w] = (int)word;
                    }
                }
            }
        }
    }

    // registers -> LDS rows of this operand (`rows` points at its first tile row in a buffer)
    __device__ __forceinline__ void store(unsigned char *rows, int tid)
    {
        if constexpr (K_CONTIGUOUS) {
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int cid = tid + it * NT;
                if (CHUNKS % NT != 0 && cid >= CHUNKS) continue;
                const int row = cid >> 3, ch = cid & 7;
                v4i v = {raw[it][0][0], raw[it][0][1], raw[it][0][2], raw[it][0][3]};
                *(v4i *)(rows + row * ROWB + ch * 16) = v;
            }
        } else {
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int bid = tid + it * NT;
                if (BLOCKS % NT != 0 && bid >= BLOCKS) continue;
                const int rblk = bid % RBLKS, kch = bid / RBLKS;
                unsigned char *dst = rows + (rblk * MB) * ROWB + kch * 16;
                if constexpr (ES == 1) {
                    v4i out[MB];
                    Transpose<DT, MB>::all(raw[it], out);
#pragma unroll
                    for (int c = 0; c < MB; ++c) *(v4i *)(dst + c * ROWB) = out[c];
                } else {
#pragma unroll
                    for (int c = 0; c < MB; ++c) *(v4i *)(dst + c * ROWB) = Transpose<DT, MB>::chunk(raw[it], c);
                }
            }
        }
    }
};

// A_KC: A has K contiguous (a transposed A of a column-major problem); B_NC: B has N contiguous (a
// transposed B).  The canonical problem is <false, false>.
template <class T, bool A_KC = false, bool B_NC = false>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel(const Params p)
{
    typedef typename T::DT DT;
    typedef typename DT::elt elt;
    typedef typename DT::accv accv;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, ROWB = T::ROWB;
    constexpr int TM = T::TM, TN = T::TN;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave % T::WAVES_M) * T::WM;
    const int wn0 = (wave / T::WAVES_M) * T::WN;

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    // a tile that sticks out of C is moved back to end at the edge (when the matrix has a whole tile of
    // rows / columns): all its loads are whole vectors, and it stores only the part it owns
    const int m_own = tm * BM, n_own = tn * BN;
    const int m0 = (m_own + BM > p.M && p.M >= BM) ? p.M - BM : m_own;
    const int n0 = (n_own + BN > p.N && p.N >= BN) ? p.N - BN : n_own;

    // ---- which part of K (loop L2, possibly split)
    const int z = blockIdx.y;
    const int kt_begin = z * p.ktiles_per_split;
    int kt_end = kt_begin + p.ktiles_per_split;
    if (kt_end > p.ktiles) kt_end = p.ktiles;
    const int nkt = kt_end - kt_begin;

    const elt *__restrict__ A = (const elt *)p.A;
    const elt *__restrict__ B = (const elt *)p.B;
    // interior tiles take whole-vector loads whatever the alignment of the operands
    const bool tile_in_a = (m0 + BM <= p.M);
    const bool tile_in_b = (n0 + BN <= p.N);

    accv acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    StagedOperand<T, BM, A_KC> opa;
    StagedOperand<T, BN, !B_NC> opb;

    // ---- global -> registers for K step kt
    auto load_tiles = [&](int kt) {
        const int k0 = kt * BK;
        const bool kfull = (k0 + BK <= p.K);
        opa.load(A, p.lda, m0, k0, p.M, p.K, tile_in_a && kfull, tid);
        opb.load(B, p.ldb, n0, k0, p.N, p.K, tile_in_b && kfull, tid);
    };
    // ---- registers -> LDS buffer `buf` (the packing step): rows of 128 bytes, K contiguous
    auto store_tiles = [&](int buf) {
        unsigned char *base = smem + buf * T::STAGE;
        opa.store(base, tid);
        opb.store(base + BM * ROWB, tid);
    };

    // ---- the micro-kernel on one LDS buffer
    auto compute = [&](int buf) { micro_kernel<T>(smem + buf * T::STAGE, wm0, wn0, lane, acc); };

    if (nkt > 0) {
        load_tiles(kt_begin);
        store_tiles(0);
        __syncthreads();
        for (int i = 0; i < nkt; ++i) {
            const bool more = (i + 1 < nkt);
            if (more) load_tiles(kt_begin + i + 1);
            compute(i & 1);
            if (more) store_tiles((i + 1) & 1);
            __syncthreads();
        }
    }

    store_tile<DT, TM, TN>(acc, p, m0, n0, BM, BN, wm0, wn0, lane, z, m_own, n_own);
}

// ---------------------------------------------------------------- helpers
// Sum of the split-K partial tiles in fixed order, then the alpha/beta update.
// VEC: every thread takes 4 consecutive elements of a column with 16-byte accesses (M and ldc multiples
// of 4, C 16-byte aligned, C in the accumulator's type); each element is summed in the same order either way.
template <class acc_t, bool VEC>
__global__ void __launch_bounds__(256) reduce_kernel(const acc_t *__restrict__ ws, acc_t *__restrict__ C, int M, int N,
                                                     int64_t ldc, int split, uint32_t alpha_bits, uint32_t beta_bits,
                                                     int use_beta, int c_type)
{
    // int8 problems are summed as unsigned 32-bit integers (wrapping arithmetic)
    typedef typename std::conditional<__is_same(acc_t, int), uint32_t, acc_t>::type sum_t;
    constexpr int W = VEC ? 4 : 1;
    typedef sum_t vec_t __attribute__((ext_vector_type(W)));
    const int64_t total = (int64_t)M * N;
    const sum_t alpha = __builtin_bit_cast(sum_t, alpha_bits);
    const sum_t beta = __builtin_bit_cast(sum_t, beta_bits);
    for (int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * W; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x * W) {
        const int m = (int)(idx % M);
        const int64_t n = idx / M;
        // the partial tiles are added in the order of their K slices; 8 loads are in flight at a time
        const vec_t *src = (const vec_t *)(ws + idx);
        const int64_t stride = total / W;                       // vectors from one partial tile to the next
        vec_t s = 0;
        int zz = 0;
        for (; zz + 8 <= split; zz += 8) {
            vec_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(zz + u) * stride];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; zz < split; ++zz) s += src[(int64_t)zz * stride];
        vec_t r = alpha * s;
        if constexpr (__is_same(acc_t, int)) {
            vec_t *c = (vec_t *)(C + n * ldc + m);
            if (use_beta) r += beta * (*c);
            *c = r;
        } else {
            if (VEC || c_type == C_WIDE) {
                vec_t *c = (vec_t *)(C + n * ldc + m);
                if (use_beta) r += beta * (*c);
                *c = r;
            } else {
                if (use_beta) r[0] += beta * narrow_load(c_type, C, n * ldc + m);
                narrow_store(c_type, C, n * ldc + m, r[0]);
            }
        }
    }
}

// C <- beta*C (K == 0 or alpha == 0); beta == 0 stores zeros without reading C.
// VEC: 4 consecutive elements of a column per thread with 16-byte accesses (conditions as for reduce_kernel).
template <class acc_t, bool VEC>
__global__ void __launch_bounds__(256) scale_kernel(acc_t *__restrict__ C, int M, int N, int64_t ldc,
                                                    uint32_t beta_bits, int use_beta, int c_type)
{
    typedef typename std::conditional<__is_same(acc_t, int), uint32_t, acc_t>::type sum_t;
    constexpr int W = VEC ? 4 : 1;
    typedef sum_t vec_t __attribute__((ext_vector_type(W)));
    const int64_t total = (int64_t)M * N;
    const sum_t beta = __builtin_bit_cast(sum_t, beta_bits);
    for (int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * W; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x * W) {
        const int m = (int)(idx % M);
        const int64_t n = idx / M;
        if constexpr (!__is_same(acc_t, int) && !VEC) {
            if (c_type != C_WIDE) {
                narrow_store(c_type, C, n * ldc + m, use_beta ? beta * narrow_load(c_type, C, n * ldc + m) : 0.0f);
                continue;
            }
        }
        vec_t *c = (vec_t *)(C + n * ldc + m);
        vec_t v = 0;
        if (use_beta) v = beta * (*c);
        *c = v;
    }
}

}  // namespace mig
