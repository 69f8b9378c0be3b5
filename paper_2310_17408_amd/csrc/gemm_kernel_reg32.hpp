// fp32 GEMM kernel for gfx950 without the packing step: the GPU counterpart of
// the non-packing variant in the paper's Sec. "Edge Cases" (operands taken from
// the matrices as they lie in memory when copying them first is not worth it).
//
// Nothing goes through LDS and there are no barriers.  Every wave owns a
// WM x WN tile of C and loads its MFMA operands from global memory straight
// into the registers the MFMA instructions read:
//   * an fp32 MFMA fragment is one float per lane, so the M-contiguous operand A
//     is read as it lies: for one k a lane loads the TM consecutive m it owns
//     (the wave tile is interleaved in M as in gemm_kernel_dma32.hpp), and the
//     lanes of a group read one contiguous run of a k-row;
//   * of the K-contiguous operand B a lane loads 16 bytes (4 consecutive k) of
//     its own row n, which feed 4 MFMA instructions.
// The lane groups of an MFMA (2 for the 32x32x2 shape, 4 for 16x16x4) take
// different k, so a K step of 16 gives each group KG = 8 or 4 consecutive k.
// DEPTH steps are in flight per wave (rolling register buffers), which is what
// short, latency-bound problems need: the im2row GEMMs with K of a few hundred
// have their whole K range on the way before the first MFMA.  The waves of a
// workgroup cover neighbouring tiles, so that the panels they share meet in the
// CU's vector cache.
//
// WAVES_K waves can share one tile of C, each taking a contiguous part of the
// workgroup's K range; their partial tiles meet in LDS after the K loop (one
// barrier) and are summed in fixed order by the first of them.  Problems with
// few tiles and a long K get their parallelism this way without a second
// kernel and without partial tiles in global memory.
//
// Rows of A or B beyond M or N are replaced by rows that exist (they only feed
// rows and columns of C that are never stored); a partial last K step is loaded
// element by element with zeros beyond K.  Loads need 4-byte alignment only.
//
// IM2ROW: the K-contiguous operand B is the im2row matrix of a channels-last image (the transform
// the paper's Sec. "Rectangular Matrices" takes its GEMM sizes from), read from the image in place;
// row n is an output pixel.
//   IM2ROW_TAPS: Cin is a multiple of the K step, so a step lies inside one filter tap (r, s), whose
//     position in the image is wave-uniform; a lane adds the offset of its pixel and skips the load
//     (zeros) where the tap falls outside the image.
//   IM2ROW_RUNS: any Cin (the first layer of a network has 3).  For one filter row r the kw*Cin
//     elements (s, c) are one contiguous run of the image row, so k = r*(kw*Cin) + e and element e of
//     the run is inside the image for lo <= e < hi, two bounds per pixel.  Elements are loaded one by
//     one.
#pragma once
#include "gemm_kernel.hpp"
#include <type_traits>

namespace mig {

#define MIG_GLOBAL __attribute__((address_space(1)))
typedef float f2u __attribute__((ext_vector_type(2), aligned(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float v2f32 __attribute__((ext_vector_type(2)));

template <int BS_, int TM_, int TN_, int WAVES_M_, int WAVES_N_, int WAVES_K_, int DEPTH_, int MINB_>
struct RegTile {
    typedef F32 DT;
    static constexpr int BS = BS_, TM = TM_, TN = TN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, WAVES_K = WAVES_K_;
    static constexpr int DEPTH = DEPTH_, MINB = MINB_;
    static constexpr int WMN = WAVES_M * WAVES_N;   // wave tiles per workgroup; each is shared by WAVES_K waves
    static constexpr int NW = WMN * WAVES_K, NT = NW * 64;
    static constexpr int G = 64 / BS;          // lane groups of an MFMA; each takes its own k
    static constexpr int BK = 16;              // K elements per step
    static constexpr int KG = BK / G;          // consecutive k per lane group and step = MFMAs per block and step
    static constexpr int WM = BS * TM, WN = BS * TN;
    static constexpr int BM = WAVES_M * WM, BN = WAVES_N * WN;
    static constexpr int ACC = BS * BS / 64;   // accumulator registers per block
    static constexpr int RED_FLOATS = (WAVES_K - 1) * WMN * TM * TN * ACC * 64;   // partial tiles handed over in LDS
    static constexpr int LDS_BYTES = RED_FLOATS * 4, STAGE = 0;
    // a lane's byte offset from its wave's first row must fit 32 bits
    static constexpr int64_t MAX_LDA = ((int64_t)1 << 32) / (4 * BK) - 64;
    static constexpr int64_t MAX_LDB = ((int64_t)1 << 32) / (4 * WN) - 64;
    static_assert(BS == 32 || BS == 16, "MFMA block of 32x32 (k = 2) or 16x16 (k = 4)");
    static_assert(TM == 1 || TM == 2 || TM == 4, "a lane reads 1, 2 or 4 consecutive m");
    static_assert(DEPTH >= 1, "at least one step in flight");
    static_assert(NT <= 1024 && LDS_BYTES <= 64 * 1024, "workgroup limits");
};

template <int BS> struct RegMma;
template <> struct RegMma<32> {
    typedef v16f accv;
    static __device__ __forceinline__ void run(float rowop, float colop, accv &c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(rowop, colop, c, 0, 0, 0);
    }
    // column n (inside the block) of accumulator register v for lane group g
    static __device__ __forceinline__ int col(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }
};
template <> struct RegMma<16> {
    typedef v4f accv;
    static __device__ __forceinline__ void run(float rowop, float colop, accv &c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(rowop, colop, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int col(int v, int g) { return 4 * g + v; }
};

// The micro-kernel on the operands of one K step held in registers.
template <class T>
struct RegMicro {
    typedef typename RegMma<T::BS>::accv accv;
    struct aset { float v[T::KG][T::TM]; };    // per k of the lane's group: the TM rows m the lane owns
    struct bset { float v[T::TN][T::KG]; };    // per block column: KG consecutive k of the lane's row n
    static __device__ __forceinline__ void mma(const aset &xa, const bset &xb, accv (&acc)[T::TM][T::TN])
    {
#pragma unroll
        for (int t = 0; t < T::KG; ++t)
#pragma unroll
            for (int i = 0; i < T::TM; ++i)
#pragma unroll
                for (int j = 0; j < T::TN; ++j) RegMma<T::BS>::run(xb.v[j][t], xa.v[t][i], acc[i][j]);
    }
};

enum { IM2ROW_NONE = 0, IM2ROW_TAPS = 1, IM2ROW_RUNS = 2 };

template <class T, int IM2ROW = IM2ROW_NONE>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel_reg32(const Params p)
{
    constexpr int BS = T::BS, TM = T::TM, TN = T::TN, KG = T::KG, BK = T::BK, D = T::DEPTH, ACC = T::ACC;
    typedef RegMicro<T> Micro;
    typedef typename Micro::accv accv;
    typedef typename Micro::aset aset;
    typedef typename Micro::bset bset;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane % BS, g = lane / BS;
    // Which elements of B (rows n with K contiguous) a lane loads.  In the MFMA layout neighbouring lanes hold
    // neighbouring rows, and a 16-byte load per lane then touches 64 different 64-byte pieces of memory per
    // instruction, which the vector cache takes one per cycle (measured: 4-8 % of the run time).  With 16 x 16
    // blocks a K step is 64 bytes of a row: four neighbouring lanes load the four 16-byte chunks of one row (16
    // pieces per instruction), and each value is moved to the lane that multiplies it just before its MFMAs.
    constexpr bool COAL = (BS == 16) && (IM2ROW != IM2ROW_RUNS);
    static_assert(!COAL || KG == 4, "a lane loads one 16-byte chunk per block column");
    // (rows 8 ... 15 take their chunks in the order 2, 3, 0, 1: the permutation then reads 32 different banks per
    // half wave)
    const int rb = COAL ? lane / 4 : r;                        // row of a block whose elements this lane loads
    const int gb = COAL ? (lane % 4) ^ ((lane >> 5) << 1) : g; // and which KG consecutive k of it
    const int b_from = (4 * r + (g ^ ((r >> 3) << 1))) * 4;    // COAL: byte index of the lane that loaded this lane's operands

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    constexpr int WK = T::WAVES_K, WMN = T::WMN;
    const int wmn = wave % WMN, wk = wave / WMN;
    const int mw = tm * T::BM + (wmn % T::WAVES_M) * T::WM;    // this wave's tile of C
    const int nw = tn * T::BN + (wmn / T::WAVES_M) * T::WN;
    if (mw >= p.M || nw >= p.N) {                              // so is it for all waves that share the tile
        if constexpr (WK > 1) __syncthreads();
        return;
    }

    const int z = blockIdx.y;
    int k_begin = z * p.ktiles_per_split * BK;
    int k_end = k_begin + p.ktiles_per_split * BK;
    if (k_end > p.K) k_end = p.K;
    if constexpr (WK > 1) {
        // this wave's part of the workgroup's K range, in whole steps (the last part may be short or empty)
        const int steps = (k_end - k_begin + BK - 1) / BK;
        const int per = (steps + WK - 1) / WK;
        k_begin += wk * per * BK;
        if (k_begin + per * BK < k_end) k_end = k_begin + per * BK;
    }
    const int klen = k_end > k_begin ? k_end - k_begin : 0;
    const int nfull = klen / BK, tail = IM2ROW == IM2ROW_TAPS ? 0 : klen % BK;   // whole steps when a step lies in a tap

    // ---- which rows this lane reads.  Lanes whose rows lie beyond M or N read rows that exist.
    const int mrow = mw + TM * r;                              // first of the lane's TM rows of A and C
    // TM > 1: a lane straddling M must read its rows one by one
    const bool a_rows_one_by_one = (TM > 1) && (mw + T::WM > p.M) && (p.M % TM != 0);
    // byte offsets from the wave's first row of the step: k = KG*g + t of the lane's group, row i of the lane
    uint32_t aoff[KG][TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int m = mrow + i;
        if (a_rows_one_by_one) m = m < p.M ? m : p.M - 1;
        else if (mrow + TM > p.M) m = p.M - TM + i;            // M is a multiple of TM here, so this lane is all outside
#pragma unroll
        for (int t = 0; t < KG; ++t) aoff[t][i] = (uint32_t)(((int64_t)(KG * g + t) * p.lda + (m - mw)) * 4);
    }
    uint32_t boff[TN];
    int ih0[IM2ROW ? TN : 1], iw0[IM2ROW == IM2ROW_TAPS ? TN : 1];   // IM2ROW: image position of the pixel's tap (0, 0)
    int run_lo[IM2ROW == IM2ROW_RUNS ? TN : 1], run_hi[IM2ROW == IM2ROW_RUNS ? TN : 1];   // part of a run inside the image
    const int run = p.conv.kw * p.conv.Cin;                    // IM2ROW_RUNS: elements of K per filter row
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int n = nw + BS * j + rb;
        n = n < p.N ? n : p.N - 1;
        if constexpr (IM2ROW) {
            const int per_image = p.conv.Hout * p.conv.Wout;
            const int b = n / per_image, rem = n - b * per_image;
            const int oh = rem / p.conv.Wout, ow = rem - oh * p.conv.Wout;
            ih0[j] = oh * p.conv.stride_h - p.conv.pad_h;
            const int iw = ow * p.conv.stride_w - p.conv.pad_w;
            if constexpr (IM2ROW == IM2ROW_TAPS) {
                iw0[j] = iw;
            } else {
                run_lo[j] = iw < 0 ? -iw * p.conv.Cin : 0;
                const int hi = (p.conv.W - iw) * p.conv.Cin;
                run_hi[j] = hi < run ? hi : run;
            }
            // from the address the tap (0, 0) of a pixel at (0, 0) without padding would have: never negative
            boff[j] = (uint32_t)((((int64_t)(b * p.conv.H + oh * p.conv.stride_h) * p.conv.W + ow * p.conv.stride_w) *
                                      p.conv.Cin + (IM2ROW == IM2ROW_TAPS ? KG * gb : 0)) * 4);
        } else {
            boff[j] = (uint32_t)(((int64_t)(n - nw) * p.ldb + KG * gb) * 4);
        }
    }
    const MIG_GLOBAL unsigned char *a_wave =
        (const MIG_GLOBAL unsigned char *)((const float *)p.A + (int64_t)k_begin * p.lda + mw);
    // IM2ROW: the tap (tap_r, tap_s) and the channel tap_c the wave's next step starts at; b_wave points
    // pad_h rows and pad_w pixels before that tap of pixel (0, 0) (an address that is only ever used
    // with a lane offset that brings it inside the image)
    int tap_r = 0, tap_s = 0, tap_c = 0;
    const MIG_GLOBAL unsigned char *b_wave;
    if constexpr (IM2ROW == IM2ROW_RUNS) {
        // pad_h rows and pad_w pixels before the image: what a pixel's offset counts from
        b_wave = (const MIG_GLOBAL unsigned char *)((const float *)p.B -
                 ((int64_t)p.conv.pad_h * p.conv.W + p.conv.pad_w) * p.conv.Cin);
    } else if constexpr (IM2ROW == IM2ROW_TAPS) {
        const int tap = k_begin / p.conv.Cin;
        tap_c = k_begin - tap * p.conv.Cin;
        tap_r = tap / p.conv.kw;
        tap_s = tap - tap_r * p.conv.kw;
        b_wave = (const MIG_GLOBAL unsigned char *)((const float *)p.B +
                 ((int64_t)(tap_r - p.conv.pad_h) * p.conv.W + (tap_s - p.conv.pad_w)) * p.conv.Cin + tap_c);
    } else {
        b_wave = (const MIG_GLOBAL unsigned char *)((const float *)p.B + (int64_t)nw * p.ldb + k_begin);
    }
    const int64_t a_row = p.lda * 4, a_step = (int64_t)BK * a_row;

    // ---- loads of the next full K step (no bounds to check); steps are loaded in order.  The step's
    // base addresses are wave-uniform and live in scalar registers, a lane adds its constant 32-bit
    // offsets (the empty asm statements keep the compiler from merging the two into per-lane
    // 64-bit pointers, which would cost registers and an addition per load).
    // ---- IM2ROW_RUNS: the lane's KG elements of B from k = kfirst on, for each of its pixels
    const float inv_run = 1.0f / (float)run;
    const int row_floats = p.conv.W * p.conv.Cin;
    int k_lane = k_begin + KG * g;                             // the lane's first k of the next step to load
    auto load_b_runs = [&](int kfirst, bset &xb) {
#pragma unroll
        for (int t = 0; t < KG; ++t) {
            const int k = kfirst + t;
            int rr = (int)((float)k * inv_run);                // k / run, exact after the correction (k < 2^22)
            int e = k - rr * run;
            if (e < 0) { --rr; e += run; }
            if (e >= run) { ++rr; e -= run; }
            const uint32_t ko = (uint32_t)((rr * row_floats + e) * 4);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const bool inside = k < k_end && (uint32_t)(ih0[j] + rr) < (uint32_t)p.conv.H && e >= run_lo[j] && e < run_hi[j];
                float v = 0.0f;
                if (inside) v = *(const MIG_GLOBAL float *)(b_wave + (boff[j] + ko));
                xb.v[j][t] = v;
            }
        }
    };

    const MIG_GLOBAL unsigned char *pa = a_wave, *pb = b_wave;
    auto load_step = [&](auto one_by_one, aset &xa, bset &xb) {
        asm volatile("" : "+s"(pa), "+s"(pb));
#pragma unroll
        for (int t = 0; t < KG; ++t) {
            if constexpr (decltype(one_by_one)::value || TM == 1) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    uint32_t o = aoff[t][i];
                    asm volatile("" : "+v"(o));
                    xa.v[t][i] = *(const MIG_GLOBAL float *)(pa + o);
                }
            } else {
                uint32_t o = aoff[t][0];
                asm volatile("" : "+v"(o));
                if constexpr (TM == 2) {
                    const f2u v = *(const MIG_GLOBAL f2u *)(pa + o);
                    xa.v[t][0] = v[0]; xa.v[t][1] = v[1];
                } else {
                    const f4u v = *(const MIG_GLOBAL f4u *)(pa + o);
                    xa.v[t][0] = v[0]; xa.v[t][1] = v[1]; xa.v[t][2] = v[2]; xa.v[t][3] = v[3];
                }
            }
        }
        if constexpr (IM2ROW == IM2ROW_RUNS) {
            load_b_runs(k_lane, xb);
            k_lane += BK;
            pa += a_step;
            return;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            uint32_t o = boff[j];
            asm volatile("" : "+v"(o));
            bool inside = true;
            if constexpr (IM2ROW == IM2ROW_TAPS)
                inside = (uint32_t)(ih0[j] + tap_r) < (uint32_t)p.conv.H && (uint32_t)(iw0[j] + tap_s) < (uint32_t)p.conv.W;
#pragma unroll
            for (int c = 0; c < KG / 4; ++c) {
                f4u v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (inside) v = *(const MIG_GLOBAL f4u *)(pb + o + 16 * c);
                xb.v[j][4 * c + 0] = v[0]; xb.v[j][4 * c + 1] = v[1]; xb.v[j][4 * c + 2] = v[2]; xb.v[j][4 * c + 3] = v[3];
            }
        }
        pa += a_step;
        pb += BK * 4;
        if constexpr (IM2ROW == IM2ROW_TAPS) {
            // the taps of one filter row are contiguous in the image; the next filter row is one image row on
            tap_c += BK;
            if (tap_c == p.conv.Cin) {
                tap_c = 0;
                if (++tap_s == p.conv.kw) {
                    tap_s = 0;
                    ++tap_r;
                    pb += (int64_t)(p.conv.W - p.conv.kw) * p.conv.Cin * 4;
                }
            }
        }
    };
    // ---- the partial last step: element by element, zeros beyond the K range
    auto load_tail = [&](aset &xa, bset &xb) {
        const MIG_GLOBAL unsigned char *ta_ = a_wave + (int64_t)nfull * a_step;
        const MIG_GLOBAL unsigned char *tb_ = b_wave + (int64_t)nfull * (BK * 4);
#pragma unroll
        for (int t = 0; t < KG; ++t) {
            const bool valid = (KG * g + t) < tail;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int m = mrow + i;
                m = m < p.M ? m : p.M - 1;
                const uint32_t off = (uint32_t)(((int64_t)(KG * g) * p.lda + (m - mw)) * 4);
                xa.v[t][i] = valid ? *(const MIG_GLOBAL float *)(ta_ + t * a_row + off) : 0.0f;
            }
            if constexpr (IM2ROW == IM2ROW_NONE) {
                const bool valid_b = (KG * gb + t) < tail;
#pragma unroll
                for (int j = 0; j < TN; ++j) xb.v[j][t] = valid_b ? *(const MIG_GLOBAL float *)(tb_ + boff[j] + 4 * t) : 0.0f;
            }
        }
        if constexpr (IM2ROW == IM2ROW_RUNS) load_b_runs(k_begin + nfull * BK + KG * g, xb);
    };

    accv acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0;

    aset fa[D], ta;
    bset fb[D], tb;
    // the MFMAs of one step; COAL: its B operands first move from the lanes that loaded them to the lanes of the
    // MFMA layout (a permutation of the wave's lanes through the LDS crossbar, no memory involved)
    auto mma_step = [&](const aset &xa, bset &xb) __attribute__((always_inline)) {
        if constexpr (COAL) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int t = 0; t < KG; ++t)
                    xb.v[j][t] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(b_from, __builtin_bit_cast(int, xb.v[j][t])));
        }
        Micro::mma(xa, xb, acc);
    };
    if (tail) load_tail(ta, tb);                               // the first loads to be issued

    // ---- K loop: D steps in flight.  In the steady state every load is unconditional, so the
    // number of loads outstanding is fixed and each MFMA group waits for exactly its own operands.
    // A K range of at most D steps is fetched whole before its first MFMA; no step is loaded twice.
    auto k_loop = [&](auto one_by_one) {
        if (nfull <= D) {
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (d < nfull) load_step(one_by_one, fa[d], fb[d]);
            if (tail) mma_step(ta, tb);
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (d < nfull) mma_step(fa[d], fb[d]);
            return;
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            load_step(one_by_one, fa[d], fb[d]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (tail) mma_step(ta, tb);                     // its operands are the oldest loads
        __builtin_amdgcn_sched_barrier(0);
        int s = 0;
        for (; s + 2 * D <= nfull; s += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                mma_step(fa[d], fb[d]);
                load_step(one_by_one, fa[d], fb[d]);
                __builtin_amdgcn_sched_barrier(0);             // keep the steps apart: one wait per step
            }
        }
        // D <= nfull - s < 2 D: the buffers hold steps s .. s+D-1, the rest is still to be loaded
        const int rest = nfull - s - D;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            mma_step(fa[d], fb[d]);
            if (d < rest) load_step(one_by_one, fa[d], fb[d]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < rest) mma_step(fa[d], fb[d]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (nfull > 0) {
        if (a_rows_one_by_one) k_loop(std::integral_constant<bool, true>());
        else k_loop(std::integral_constant<bool, false>());
    } else if (tail) {
        mma_step(ta, tb);
    }

    // ---- the waves that share this tile hand their partial tiles to the first of them
    if constexpr (WK > 1) {
        __shared__ float red[T::RED_FLOATS];
        if (wk > 0) {
            float *dst = red + ((wk - 1) * WMN + wmn) * (TM * TN * ACC * 64) + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < ACC; ++v) dst[((i * TN + j) * ACC + v) * 64] = acc[i][j][v];
        }
        __syncthreads();
        if (wk > 0) return;
        for (int q = 1; q < WK; ++q) {
            const float *src = red + ((q - 1) * WMN + wmn) * (TM * TN * ACC * 64) + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < ACC; ++v) acc[i][j][v] += src[((i * TN + j) * ACC + v) * 64];
        }
    }

    // ---- epilogue: per block column n a lane holds the TM consecutive rows m it owns
    {
        const float alpha = __builtin_bit_cast(float, p.alpha_bits);
        const float beta = __builtin_bit_cast(float, p.beta_bits);
        const bool use_beta = p.use_beta != 0;
        const bool interior = (mw + T::WM <= p.M) && (nw + T::WN <= p.N);
        const bool vec_c = (TM > 1) && interior && ((p.ldc % TM) == 0) && (((uintptr_t)p.C % (TM * 4)) == 0) &&
                           p.split <= 1;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int v = 0; v < ACC; ++v) {
                const int n = nw + BS * j + RegMma<BS>::col(v, g);
                if (p.split > 1) {
                    float *ws = (float *)p.ws + ((int64_t)z * p.N + n) * p.M + mrow;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (interior || (mrow + i < p.M && n < p.N)) ws[i] = acc[i][j][v];
                } else {
                    float *c = (float *)p.C + (int64_t)n * p.ldc + mrow;
                    if (vec_c) {
                        if constexpr (TM == 2) {
                            v2f32 o = {alpha * acc[0][j][v], alpha * acc[1][j][v]};
                            if (use_beta) { const v2f32 old = *(const v2f32 *)c; o[0] += beta * old[0]; o[1] += beta * old[1]; }
                            *(v2f32 *)c = o;
                        } else if constexpr (TM == 4) {
                            v4f o = {alpha * acc[0][j][v], alpha * acc[1][j][v], alpha * acc[2][j][v], alpha * acc[3][j][v]};
                            if (use_beta) {
                                const v4f old = *(const v4f *)c;
                                o[0] += beta * old[0]; o[1] += beta * old[1]; o[2] += beta * old[2]; o[3] += beta * old[3];
                            }
                            *(v4f *)c = o;
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            if (interior || (mrow + i < p.M && n < p.N)) {
                                float o = alpha * acc[i][j][v];
                                if (use_beta) o += beta * c[i];
                                c[i] = o;
                            }
                        }
                    }
                }
            }
        }
    }
}

}  // namespace mig
