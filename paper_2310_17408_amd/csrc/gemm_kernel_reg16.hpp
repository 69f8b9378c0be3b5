// fp16 / bf16 / int8 GEMM kernel for gfx950 without the packing step: the 16- and 8-bit counterpart
// of gemm_kernel_reg32.hpp (the non-packing variant of the paper's Sec. "Edge Cases"; its Sec.
// "Data types" re-targets a micro-kernel by changing operand types).
//
// No LDS staging, no barriers in the K loop.  Every wave owns a WM x WN tile of C made of 16 x 16
// blocks for the deep-K MFMA shapes (16x16x32 for 16-bit inputs, 16x16x64 for int8) and loads its
// operands from global memory into registers, DEPTH K steps in flight:
//   * a fragment is KCH consecutive k (16 bytes) of one row; lane l holds row l%16 and the k group
//     l/16 of 4, so a K step is 4*KCH elements;
//   * of the K-contiguous operand B a lane loads its fragment as it lies: 16 bytes of its row n;
//   * of the M-contiguous operand A a lane loads, for each of its KCH k, one 32-bit word = the TM
//     consecutive m it owns (2 halves or 4 bytes; the wave tile is interleaved in M, block i is the
//     rows {TM*l + i}), and transposes the KCH words in registers into its TM fragments.
// WAVES_K waves can share a tile, each taking part of the K range; their partial tiles meet in LDS
// after the K loop and are added in fixed order.  Rows beyond M or N are replaced by rows that
// exist.  The lane whose word of A would straddle M loads the last whole word of the column instead
// and shifts the rows it owns into place when the word is used; in a partial last K step the words
// and fragments that lie wholly inside K are loaded as usual, a fragment that straddles K element by
// element, the rest is zero.  Loads are issued at element alignment (the memory system splits
// misaligned ones).
//
// IM2ROW: the K-contiguous operand B is the im2row matrix of a channels-last image (paper Sec.
// "Rectangular Matrices"), read from the image in place: row n is an output pixel, and with Cin a
// multiple of the K step a step lies inside one filter tap, so a lane's fragment is 16 contiguous
// bytes of the image, or zeros where the tap falls outside it (the load is then not issued).
#pragma once
#include "gemm_kernel_dma.hpp"
#include "gemm_kernel_reg32.hpp"

namespace mig {

// A wave-uniform pointer moved into scalar registers, so that loads take the form "scalar base + 32-bit
// lane offset" and the compiler does not merge the two into per-lane 64-bit pointers.
__device__ __forceinline__ const MIG_GLOBAL unsigned char *scalar_ptr(const MIG_GLOBAL unsigned char *q)
{
    const uint64_t u = (uint64_t)q;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (const MIG_GLOBAL unsigned char *)(((uint64_t)hi << 32) | lo);
}

template <class DT_, int TN_, int WAVES_M_, int WAVES_N_, int WAVES_K_, int DEPTH_, int MINB_>
struct Reg16Tile {
    typedef DT_ DT;
    static constexpr int ES = DT::ES, KCH = DT::KCH;
    static constexpr int TM = 4 / ES;              // rows per 32-bit word of A: 2 halves or 4 bytes
    static constexpr int TN = TN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, WAVES_K = WAVES_K_;
    static constexpr int DEPTH = DEPTH_, MINB = MINB_;
    static constexpr int WMN = WAVES_M * WAVES_N;
    static constexpr int NW = WMN * WAVES_K, NT = NW * 64;
    static constexpr int BK = 4 * KCH;             // K elements per step: 4 lane groups x one fragment
    static constexpr int WM = 16 * TM, WN = 16 * TN;
    static constexpr int BM = WAVES_M * WM, BN = WAVES_N * WN;
    static constexpr int ACC = 4;
    static constexpr int LOADS = KCH + TN;         // load instructions per step
    static constexpr int RED_WORDS = (WAVES_K - 1) * WMN * TM * TN * ACC * 64;
    static constexpr int LDS_BYTES = RED_WORDS * 4, STAGE = 0;
    static constexpr int64_t MAX_LDA = ((int64_t)1 << 32) / (ES * BK) - 64;
    static constexpr int64_t MAX_LDB = ((int64_t)1 << 32) / (ES * WN) - 64;
    static_assert(ES == 1 || ES == 2, "16- and 8-bit inputs");
    static_assert(DEPTH * LOADS <= 63, "loads in flight must fit the counter");
    static_assert(NT <= 1024 && LDS_BYTES <= 64 * 1024, "workgroup limits");
};

// The operands of one K step as loaded (A still with M contiguous in each word) and the micro-kernel
// on them.
template <class T>
struct Reg16Micro {
    typedef typename T::DT DT;
    typedef typename Mma16<DT>::accv accv;
    static constexpr int TM = T::TM, TN = T::TN, KCH = T::KCH, ES = T::ES;
    struct step { int a[KCH]; v4i b[TN]; };

    // KCH words of TM elements each -> TM fragments of KCH consecutive k.  SHIFT: every word is first
    // moved down by `sh` bits (the lane at a ragged edge of M, see the kernel).
    template <bool SHIFT>
    static __device__ __forceinline__ void fragments(const step &x, uint32_t sh, v4i (&fa)[TM])
    {
        uint32_t a[KCH];
#pragma unroll
        for (int t = 0; t < KCH; ++t) a[t] = SHIFT ? (uint32_t)x.a[t] >> sh : (uint32_t)x.a[t];
        if constexpr (ES == 2) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                fa[0][w] = (int)byte_perm(a[2 * w + 1], a[2 * w], 0x05040100u);
                fa[1][w] = (int)byte_perm(a[2 * w + 1], a[2 * w], 0x07060302u);
            }
        } else {
            int raw[16][1];
#pragma unroll
            for (int t = 0; t < 16; ++t) raw[t][0] = (int)a[t];
            Transpose<I8, 4>::all(raw, fa);
        }
    }

    template <bool SHIFT = false>
    static __device__ __forceinline__ void mma(const step &x, accv (&acc)[TM][TN], uint32_t sh = 0)
    {
        v4i fa[TM];
        fragments<SHIFT>(x, sh, fa);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) Mma16<DT>::run(x.b[j], fa[i], acc[i][j]);
    }
};

template <bool V>
struct WithShift { static constexpr bool value = V; };

template <class T, bool IM2ROW = false>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel_reg16(const Params p)
{
    typedef typename T::DT DT;
    typedef typename DT::elt elt;
    typedef typename DT::acc_t acc_t;
    constexpr int TM = T::TM, TN = T::TN, KCH = T::KCH, BK = T::BK, ES = T::ES, D = T::DEPTH, ACC = T::ACC;
    typedef Reg16Micro<T> Micro;
    typedef typename Micro::accv accv;
    typedef typename Micro::step step;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, g = lane >> 4;

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
        const int steps = (k_end - k_begin + BK - 1) / BK;
        const int per = (steps + WK - 1) / WK;
        k_begin += wk * per * BK;
        if (k_begin + per * BK < k_end) k_end = k_begin + per * BK;
    }
    const int klen = k_end > k_begin ? k_end - k_begin : 0;
    const int nfull = klen / BK, tail = klen % BK;

    // ---- which rows this lane reads.  Lanes whose rows lie beyond M or N read rows that exist.
    const int mrow = mw + TM * r;                              // first of the lane's TM rows of A and C
    // a matrix with fewer rows than a word holds is read element by element
    const bool a_by_element = p.M < TM;
    // A lane whose word would reach beyond M reads the last whole word of the column, rows M-TM .. M-1;
    // the rows it owns, mrow .. M-1, then sit `over` elements up in that word and are shifted down
    // before use (what the shift brings in from above stands for rows >= M, which are never stored).
    const int mword = (mrow + TM <= p.M) ? mrow : p.M - TM;
    const int over = (mrow < p.M && mrow + TM > p.M) ? mrow + TM - p.M : 0;
    const uint32_t a_shift = (uint32_t)(8 * ES * over);
    const bool wave_shifts = (mw + T::WM > p.M) && (p.M % TM != 0);   // wave-uniform
    // lane offsets are unsigned: they count from the lowest row any lane of the wave reads
    const int mbase = (p.M - TM < mw && !a_by_element) ? p.M - TM : mw;
    uint32_t aoff[KCH];                                        // byte offsets of the lane's word for k = KCH*g + t
#pragma unroll
    for (int t = 0; t < KCH; ++t)
        aoff[t] = a_by_element ? 0u : (uint32_t)(((int64_t)(KCH * g + t) * p.lda + (mword - mbase)) * ES);
    uint32_t boff[TN];
    int nrow[TN];
    int ih0[IM2ROW ? TN : 1], iw0[IM2ROW ? TN : 1];            // IM2ROW: image position of the pixel's tap (0, 0)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int n = nw + 16 * j + r;
        nrow[j] = n < p.N ? n : p.N - 1;
        if constexpr (IM2ROW) {
            const int per_image = p.conv.Hout * p.conv.Wout;
            const int b = nrow[j] / per_image, rem = nrow[j] - b * per_image;
            const int oh = rem / p.conv.Wout, ow = rem - oh * p.conv.Wout;
            ih0[j] = oh * p.conv.stride_h - p.conv.pad_h;
            iw0[j] = ow * p.conv.stride_w - p.conv.pad_w;
            // from the address the tap (0, 0) of a pixel at (0, 0) without padding would have: never negative
            boff[j] = (uint32_t)((((int64_t)(b * p.conv.H + oh * p.conv.stride_h) * p.conv.W + ow * p.conv.stride_w) *
                                      p.conv.Cin + KCH * g) * ES);
        } else {
            boff[j] = (uint32_t)(((int64_t)(nrow[j] - nw) * p.ldb + KCH * g) * ES);
        }
    }
    const MIG_GLOBAL unsigned char *a_wave =
        (const MIG_GLOBAL unsigned char *)((const elt *)p.A + (int64_t)k_begin * p.lda + mbase);
    // IM2ROW: the tap (tap_r, tap_s) and the channel tap_c the wave's next step starts at; b_wave points pad_h
    // rows and pad_w pixels before that tap of pixel (0, 0) (an address that is only ever used with a lane
    // offset that brings it inside the image)
    int tap_r = 0, tap_s = 0, tap_c = 0;
    const MIG_GLOBAL unsigned char *b_wave;
    if constexpr (IM2ROW) {
        const int tap = k_begin / p.conv.Cin;
        tap_c = k_begin - tap * p.conv.Cin;
        tap_r = tap / p.conv.kw;
        tap_s = tap - tap_r * p.conv.kw;
        b_wave = (const MIG_GLOBAL unsigned char *)((const elt *)p.B +
                 ((int64_t)(tap_r - p.conv.pad_h) * p.conv.W + (tap_s - p.conv.pad_w)) * p.conv.Cin + tap_c);
    } else {
        b_wave = (const MIG_GLOBAL unsigned char *)((const elt *)p.B + (int64_t)nw * p.ldb + k_begin);
    }
    const int64_t a_step = (int64_t)BK * p.lda * ES;

    // ---- element-wise loads of the step that starts `kofs` elements into the wave's K range, of
    // which `kvalid` elements exist (zeros beyond): the partial last step and the waves at a ragged M
    auto load_elements = [&](int kofs, int kvalid, step &x) {
        const MIG_GLOBAL elt *A = (const MIG_GLOBAL elt *)p.A + (int64_t)(k_begin + kofs) * p.lda;
        const MIG_GLOBAL elt *B = (const MIG_GLOBAL elt *)p.B + (k_begin + kofs);
#pragma unroll
        for (int t = 0; t < KCH; ++t) {
            const int k = KCH * g + t;
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < TM; ++e) {
                int m = mrow + e;
                m = m < p.M ? m : p.M - 1;
                uint32_t bits = 0;
                if (k < kvalid) {
                    if constexpr (ES == 2) bits = (uint16_t)A[(int64_t)k * p.lda + m];
                    else bits = (uint8_t)A[(int64_t)k * p.lda + m];
                }
                word |= bits << (8 * ES * e);
            }
            x.a[t] = (int)word;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const MIG_GLOBAL elt *q = B + (int64_t)nrow[j] * p.ldb + KCH * g;
            v4i v;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t word = 0;
#pragma unroll
                for (int e = 0; e < 4 / ES; ++e) {
                    const int ki = w * (4 / ES) + e;
                    uint32_t bits = 0;
                    if (KCH * g + ki < kvalid) {
                        if constexpr (ES == 2) bits = (uint16_t)q[ki];
                        else bits = (uint8_t)q[ki];
                    }
                    word |= bits << (8 * ES * e);
                }
                v[w] = (int)word;
            }
            x.b[j] = v;
        }
    };

    // ---- the partial last step (`kvalid` < BK elements starting `kofs` elements into the wave's K
    // range): words of A for the k that exist; of B whole fragments inside K, single elements of the
    // fragment that straddles K; zeros elsewhere
    auto load_tail = [&](int kofs, int kvalid, step &x) {
        const MIG_GLOBAL unsigned char *sa = a_wave + (int64_t)kofs * p.lda * ES;
        const MIG_GLOBAL elt *B = (const MIG_GLOBAL elt *)p.B + (k_begin + kofs);
#pragma unroll
        for (int t = 0; t < KCH; ++t) {
            int word = 0;
            if (KCH * g + t < kvalid) word = *(const MIG_GLOBAL i32_u *)(sa + aoff[t]);
            x.a[t] = word;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const MIG_GLOBAL elt *q = B + (int64_t)nrow[j] * p.ldb + KCH * g;
            v4i v = {0, 0, 0, 0};
            if (KCH * g + KCH <= kvalid) {
                v = *(const MIG_GLOBAL v4i_u *)q;
            } else if (KCH * g < kvalid) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t word = 0;
#pragma unroll
                    for (int e = 0; e < 4 / ES; ++e) {
                        const int ki = w * (4 / ES) + e;
                        uint32_t bits = 0;
                        if (KCH * g + ki < kvalid) {
                            if constexpr (ES == 2) bits = (uint16_t)q[ki];
                            else bits = (uint8_t)q[ki];
                        }
                        word |= bits << (8 * ES * e);
                    }
                    v[w] = (int)word;
                }
            }
            x.b[j] = v;
        }
    };

    // ---- word-wise loads of the next full K step; steps are loaded in order.  The step's base
    // addresses are wave-uniform scalars, a lane adds its constant 32-bit offsets.
    const MIG_GLOBAL unsigned char *pa = a_wave, *pb = b_wave;
    auto load_step = [&](step &x) {
        const MIG_GLOBAL unsigned char *sa = scalar_ptr(pa), *sb = scalar_ptr(pb);
#pragma unroll
        for (int t = 0; t < KCH; ++t) {
            uint32_t o = aoff[t];
            asm volatile("" : "+v"(o));
            x.a[t] = *(const MIG_GLOBAL i32_u *)(sa + o);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            uint32_t o = boff[j];
            asm volatile("" : "+v"(o));
            if constexpr (IM2ROW) {
                const bool inside = (uint32_t)(ih0[j] + tap_r) < (uint32_t)p.conv.H && (uint32_t)(iw0[j] + tap_s) < (uint32_t)p.conv.W;
                v4i v = {0, 0, 0, 0};
                if (inside) v = *(const MIG_GLOBAL v4i_u *)(sb + o);
                x.b[j] = v;
            } else {
                x.b[j] = *(const MIG_GLOBAL v4i_u *)(sb + o);
            }
        }
        pa += a_step;
        pb += BK * ES;
        if constexpr (IM2ROW) {
            // the taps of one filter row are contiguous in the image; the next filter row is one image row on
            tap_c += BK;
            if (tap_c == p.conv.Cin) {
                tap_c = 0;
                if (++tap_s == p.conv.kw) {
                    tap_s = 0;
                    ++tap_r;
                    pb += (int64_t)(p.conv.W - p.conv.kw) * p.conv.Cin * ES;
                }
            }
        }
    };

    accv acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0;

    step f[D], ft;
    if (tail) {                                                // the first loads to be issued
        if (a_by_element) load_elements(nfull * BK, tail, ft);
        else load_tail(nfull * BK, tail, ft);
    }

    // ---- K loop: D steps in flight (the scheme of gemm_kernel_reg32.hpp); SHIFT: the wave has a lane
    // whose words of A are shifted before use
    auto k_loop = [&](auto shift_tag) {
        constexpr bool SHIFT = decltype(shift_tag)::value;
        if (nfull <= D) {
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (d < nfull) load_step(f[d]);
            if (tail) Micro::template mma<SHIFT>(ft, acc, a_shift);
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (d < nfull) Micro::template mma<SHIFT>(f[d], acc, a_shift);
            return;
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            load_step(f[d]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (tail) Micro::template mma<SHIFT>(ft, acc, a_shift);
        __builtin_amdgcn_sched_barrier(0);
        int s = 0;
        for (; s + 2 * D <= nfull; s += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                Micro::template mma<SHIFT>(f[d], acc, a_shift);
                load_step(f[d]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        const int rest = nfull - s - D;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            Micro::template mma<SHIFT>(f[d], acc, a_shift);
            if (d < rest) load_step(f[d]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d < rest) Micro::template mma<SHIFT>(f[d], acc, a_shift);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (a_by_element) {
        // fewer rows than a word: one step at a time
        if (tail) Micro::mma(ft, acc);
        for (int s = 0; s < nfull; ++s) {
            load_elements(s * BK, BK, ft);
            Micro::mma(ft, acc);
        }
    } else if (wave_shifts) {
        k_loop(WithShift<true>{});
    } else {
        k_loop(WithShift<false>{});
    }

    // ---- the waves that share this tile hand their partial tiles to the first of them
    if constexpr (WK > 1) {
        __shared__ acc_t red[T::RED_WORDS];
        if (wk > 0) {
            acc_t *dst = red + ((wk - 1) * WMN + wmn) * (TM * TN * ACC * 64) + lane;
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
            const acc_t *src = red + ((q - 1) * WMN + wmn) * (TM * TN * ACC * 64) + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < ACC; ++v) {
                        if constexpr (ES == 1) acc[i][j][v] = (int)((uint32_t)acc[i][j][v] + (uint32_t)src[((i * TN + j) * ACC + v) * 64]);
                        else acc[i][j][v] += src[((i * TN + j) * ACC + v) * 64];
                    }
        }
    }

    // ---- epilogue: in block (i, j) a lane holds row m = mrow + i and the columns n = 16*j + 4*g + v
    {
        const acc_t alpha = __builtin_bit_cast(acc_t, p.alpha_bits);
        const acc_t beta = __builtin_bit_cast(acc_t, p.beta_bits);
        const bool use_beta = p.use_beta != 0;
        const bool interior = (mw + T::WM <= p.M) && (nw + T::WN <= p.N);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int v = 0; v < ACC; ++v) {
                const int n = nw + 16 * j + 4 * g + v;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int m = mrow + i;
                    if (!(interior || (m < p.M && n < p.N))) continue;
                    const acc_t a = acc[i][j][v];
                    if (p.split > 1) {
                        ((acc_t *)p.ws)[((int64_t)z * p.N + n) * p.M + m] = a;
                    } else {
                        acc_t *c = (acc_t *)p.C + (int64_t)n * p.ldc + m;
                        if constexpr (ES == 1) {
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

}  // namespace mig
