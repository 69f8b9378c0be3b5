// Workgroup-tile GEMM kernel for gfx950, 16- and 8-bit inputs, whose packing step (Pack A / Pack B of the
// paper's Fig. "Pseudo-code of the BLIS base GEMM algorithm") is a ring of four LDS stages filled by
// global -> LDS transfers that are issued a few at a time between the MFMAs of the micro-kernel.
//
// Same tile layout in LDS, same transfers and same fragment reads as gemm_kernel_dma.hpp (whose DmaTile,
// swizzles and helpers it uses); what differs is the K loop:
//   * a stage is one MFMA K step (32 elements of 16 bits, 64 of 8 bits), and four stages are resident:
//     while stage t is multiplied, t+1 has landed or is about to, t+2 is in flight and the transfers of
//     t+3 are being issued.  A transfer therefore has two stage times to complete, which covers the
//     latency of a miss in the last-level cache, and the wave never waits for the ones it just issued;
//   * the transfers of a stage are issued one after each of the first block rows of the two halves of the
//     stage's MFMAs instead of all at once behind the barrier: the vector-memory unit of a CU takes the
//     transfers of its 8 waves one at a time, and a wave that has a burst of them queued cannot issue
//     MFMAs meanwhile (measured on the 256 x 256 tiles at 8192^3 against two stages of twice the depth
//     filled in one burst: 2.5 % faster for fp16, 4-5 % for bf16 and int8; 7-12 % at 2048^3 on 128 x 128);
//   * the loop is unrolled over the four stages, so that LDS addresses are immediates and the register
//     sets of the double-buffered fragments are fixed.
// There is one barrier per stage, in the middle of its MFMAs: it publishes stage t+1 (every wave has
// waited for its own transfers of it) and retires the buffer of stage t: all fragment reads of stage t
// have been issued and have returned by then, so its buffer may be refilled with stage t+4 afterwards.
// Stages that cannot be moved by transfers alone (edge tiles that cannot be moved inside the matrix, a
// partial last K step, operands that are not 16-byte aligned) are staged through registers with zero
// fill, all at once behind the barrier, and the wave then waits for everything outstanding.
#pragma once
#include "gemm_kernel_dma.hpp"

#include <type_traits>

namespace mig {

// The micro-kernel on one stage: the wave tile cut into 16 x 16 blocks (MFMA 16x16x32 for 16-bit inputs,
// 16x16x64 for int8), taken in two halves of its block rows.  A lane holds row (or column) lane%16 and the
// k group lane/16 of 4: KCH consecutive k per fragment.  The A fragments are double buffered by half, the B
// fragments by the parity of the stage.  A_KC / B_NC as in DmaMicro16.
template <class T, bool A_KC = false, bool B_NC = false>
struct RingMicro16 {
    typedef typename T::DT DT;
    typedef typename Mma16<DT>::accv accv;
    static constexpr int TM = T::WM / 16, TN = T::WN / 16, HM = TM / 2;
    static constexpr int ES = T::ES, KCH = T::KCH, A_ROWB = T::A_ROWB;
    static_assert(T::KSTEPS == 2, "one K step of 4 chunks per stage");
    static_assert(TM % 2 == 0, "two halves of block rows");
    static_assert(!B_NC || T::BM == T::BN, "a transposed B needs a square tile");
    v4i fa[2][HM], fb[2][TN];
    uint32_t aoff[A_KC ? 1 : TM], boff[B_NC ? TN : 1];

    __device__ __forceinline__ void init(int lane, int wm0, int wn0)
    {
        const int r = lane & 15, g = lane >> 4;
        const int x = T::b_swz(r);                      // swizzle of a K-contiguous tile row (period 16 rows)
        const int kr = r / T::LPR, ml = r % T::LPR;     // transposing read: k-row and 8-byte piece of the lane
        if constexpr (B_NC) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nbyte = (wn0 + 16 * j) * ES + 8 * ml;
                const int ch = (nbyte >> 4) ^ T::a_swz(KCH * g + kr);
                boff[j] = T::A_BYTES + (KCH * g + kr) * A_ROWB + (ch << 4) + (nbyte & 15);
            }
        } else {
            boff[0] = T::A_BYTES + (wn0 + r) * T::B_ROWB + ((g ^ x) << 4);
        }
        if constexpr (A_KC) {
            aoff[0] = (wm0 + r) * T::B_ROWB + ((g ^ x) << 4);
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int mbyte = (wm0 + 16 * i) * ES + 8 * ml;
                const int ch = (mbyte >> 4) ^ T::a_swz(KCH * g + kr);
                aoff[i] = (KCH * g + kr) * A_ROWB + (ch << 4) + (mbyte & 15);
            }
        }
    }
    // fragments of the block rows of one half into set `half`
    __device__ __forceinline__ void load_a(const unsigned char *stage, int half)
    {
#pragma unroll
        for (int i = 0; i < HM; ++i) {
            if constexpr (A_KC) fa[half][i] = *(const v4i *)(stage + aoff[0] + (half * HM + i) * 16 * T::B_ROWB);
            else fa[half][i] = DmaMicro<T>::read_a(stage + aoff[half * HM + i]);
        }
    }
    // fragments of all block columns into set `par`
    __device__ __forceinline__ void load_b(const unsigned char *stage, int par)
    {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (B_NC) fb[par][j] = DmaMicro<T>::read_a(stage + boff[j]);
            else fb[par][j] = *(const v4i *)(stage + boff[0] + j * 16 * T::B_ROWB);
        }
    }
    // the MFMAs of one half; f(i) runs after those of block row i (transfers to interleave with them)
    template <class F>
    __device__ __forceinline__ void mma_half(int half, int par, accv (&acc)[TM][TN], F f)
    {
#pragma unroll
        for (int i = 0; i < HM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j) Mma16<DT>::run(fb[par][j], fa[half][i], acc[half * HM + i][j]);
            __builtin_amdgcn_sched_barrier(0);
            f(i);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
};

template <class T, bool A_KC = false, bool B_NC = false>
__global__ void __launch_bounds__(T::NT, T::MINB) gemm_kernel_ring(const Params p)
{
    typedef typename T::DT DT;
    typedef typename DT::elt elt;
    typedef RingMicro16<T, A_KC, B_NC> Micro;
    typedef typename Micro::accv accv;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NW = T::NW, ES = T::ES, KCH = T::KCH;
    constexpr int TM = Micro::TM, TN = Micro::TN, A_CPR = T::A_CPR;
    static_assert(T::NSTAGE == 4, "a ring of four stages");
    // transfers of a stage issued in its first half (after block rows 0 ...) and in its second half
    constexpr int HALF0 = (T::INST + 1) / 2, HALF1 = T::INST - HALF0;
    static_assert(HALF0 <= Micro::HM, "at most one transfer after each block row");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(MIG_LDS unsigned char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave % T::WAVES_M) * T::WM;
    const int wn0 = (wave / T::WAVES_M) * T::WN;

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    // a tile that sticks out of C is moved back to end at the edge when the matrix is at least one tile wide
    // and the moved tile keeps its rows 16-byte aligned; it then stores only the part no other tile owns
    const int m_own = tm * BM, n_own = tn * BN;
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

    // ---- staging: which 16-byte chunk of the A and B tiles this lane moves in transfer j of its wave
    // (transfer block b = wave + NW*j covers A_ROWS_PER_INST k-rows of A, or B_ROWS_PER_INST tile rows of a
    // K-contiguous operand); a lane's offset from the block's first element is the same in every transfer
    const int a_row_in = A_KC ? lane / T::B_CPR : lane / A_CPR, a_pch = A_KC ? lane % T::B_CPR : lane % A_CPR;
    const int b_row_in = B_NC ? lane / A_CPR : lane / T::B_CPR, b_pch = B_NC ? lane % A_CPR : lane % T::B_CPR;
    static_assert((NW * T::A_ROWS_PER_INST) % T::SWZ_PERIOD == 0, "A swizzle must repeat every NW blocks");
    static_assert((NW * T::B_ROWS_PER_INST) % T::B_SWZ_PERIOD == 0, "B swizzle must repeat every NW blocks");
    const int a_ch = A_KC ? a_pch ^ T::b_swz(wave * T::B_ROWS_PER_INST + a_row_in)
                          : a_pch ^ T::a_swz(wave * T::A_ROWS_PER_INST + a_row_in);
    const int b_ch = B_NC ? b_pch ^ T::a_swz(wave * T::A_ROWS_PER_INST + b_row_in)
                          : b_pch ^ T::b_swz(wave * T::B_ROWS_PER_INST + b_row_in);
    const uint32_t a_lane_off = (uint32_t)(((int64_t)a_row_in * p.lda + a_ch * KCH) * ES);
    const uint32_t b_lane_off = (uint32_t)(((int64_t)b_row_in * p.ldb + b_ch * KCH) * ES);
    constexpr int A_RPI = A_KC ? T::B_ROWS_PER_INST : T::A_ROWS_PER_INST;          // tile rows (m or k) per transfer
    constexpr int B_RPI = B_NC ? T::A_ROWS_PER_INST : T::B_ROWS_PER_INST;          // tile rows (k or n) per transfer
    constexpr int A_INST = A_KC ? T::BM * T::B_ROWB / 1024 / NW : T::A_INST;
    constexpr int B_INST = B_NC ? BK * T::A_ROWB / 1024 / NW : T::B_INST;
    static_assert(A_INST + B_INST == T::INST, "square tiles when an operand is transposed");
    const int64_t a_blk_stride = (int64_t)NW * A_RPI * p.lda * ES;                 // bytes between transfers j, j+1
    const int64_t b_blk_stride = (int64_t)NW * B_RPI * p.ldb * ES;
    const int64_t a_step = A_KC ? (int64_t)BK * ES : (int64_t)BK * p.lda * ES;      // bytes from one K step to the next
    const int64_t b_step = B_NC ? (int64_t)BK * p.ldb * ES : (int64_t)BK * ES;
    const unsigned char *a_wave = A_KC ? (const unsigned char *)A + ((int64_t)(m0 + wave * A_RPI) * p.lda) * ES
                                       : (const unsigned char *)A + ((int64_t)wave * A_RPI * p.lda + m0) * ES;
    const unsigned char *b_wave = B_NC ? (const unsigned char *)B + ((int64_t)wave * B_RPI * p.ldb + n0) * ES
                                       : (const unsigned char *)B + ((int64_t)(n0 + wave * B_RPI) * p.ldb) * ES;

    // transfer q (of INST: those of A first) of K step kt into buffer buf; operands inside the matrices, aligned
    auto dma_piece = [&](int kt, int buf, int q) {
        const uint32_t la = lds_base + buf * T::STAGE + wave * 1024;
        if (q < A_INST) lds_dma16(a_wave + (int64_t)kt * a_step + q * a_blk_stride, a_lane_off, la + q * NW * 1024);
        else lds_dma16(b_wave + (int64_t)kt * b_step + (q - A_INST) * b_blk_stride, b_lane_off,
                       la + T::A_BYTES + (q - A_INST) * NW * 1024);
    };

    // the same chunks with zero fill, through registers where the transfer cannot be used
    auto stage_guarded = [&](int kt, int buf) {
        const int k0 = kt * BK;
        const bool kfull = (k0 + BK <= p.K);
        const uint32_t sbase = buf * T::STAGE;
        if (tile_fast_a && kfull) {
#pragma unroll
            for (int j = 0; j < A_INST; ++j) dma_piece(kt, buf, j);
        } else {
#pragma unroll
            for (int j = 0; j < A_INST; ++j) {
                const int blk = wave + NW * j;
                const elt *src;
                int valid;
                if constexpr (A_KC) {
                    const int r = blk * A_RPI + a_row_in, k = k0 + a_ch * KCH;          // tile row m, first k of the chunk
                    src = A + (int64_t)(m0 + r) * p.lda + k;
                    valid = (m0 + r < p.M) ? (p.K - k) : 0;
                } else {
                    const int k = blk * A_RPI + a_row_in, m = m0 + a_ch * KCH;          // tile-local k-row, first m of the chunk
                    src = A + (int64_t)(k0 + k) * p.lda + m;
                    valid = (k0 + k < p.K) ? (p.M - m) : 0;
                }
                valid = valid > KCH ? KCH : valid;
                *(v4i *)(smem + sbase + blk * 1024 + lane * 16) = guarded_chunk<DT>(src, valid);
            }
        }
        if (tile_fast_b && kfull) {
#pragma unroll
            for (int j = 0; j < B_INST; ++j) dma_piece(kt, buf, A_INST + j);
        } else {
#pragma unroll
            for (int j = 0; j < B_INST; ++j) {
                const int blk = wave + NW * j;
                const elt *src;
                int valid;
                if constexpr (B_NC) {
                    const int k = blk * B_RPI + b_row_in, n = n0 + b_ch * KCH;
                    src = B + (int64_t)(k0 + k) * p.ldb + n;
                    valid = (k0 + k < p.K) ? (p.N - n) : 0;
                } else {
                    const int r = blk * B_RPI + b_row_in, k = k0 + b_ch * KCH;
                    src = B + (int64_t)(n0 + r) * p.ldb + k;
                    valid = (n0 + r < p.N) ? (p.K - k) : 0;
                }
                valid = valid > KCH ? KCH : valid;
                *(v4i *)(smem + sbase + T::A_BYTES + blk * 1024 + lane * 16) = guarded_chunk<DT>(src, valid);
            }
        }
    };

    Micro micro;
    micro.init(lane, wm0, wn0);

    accv acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0;

    // the first `nfast` K steps of this workgroup are moved by transfers alone
    int nfast = 0;
    if (tile_fast_a && tile_fast_b) {
        nfast = p.K / BK - kt_begin;
        nfast = nfast < 0 ? 0 : (nfast > nkt ? nkt : nfast);
    }

    // One stage: multiply K step t (relative to kt_begin), resident in buffer b = t % 4 with its fragments
    // of half 0 read into set 0 and its B fragments into set par = t % 2.  Meanwhile K step t+3 is fetched
    // into buffer (b + 3) % 4, which the barrier of the previous stage has retired.  HOT: K steps t+1 ...
    // t+3 exist and are moved by transfers alone (all conditions known at compile time); otherwise the
    // conditions are tested (they are uniform over the workgroup).
    auto stage = [&](auto hot_tag, int b, int par, int t) {
        constexpr bool HOT = decltype(hot_tag)::value;
        const unsigned char *cur = smem + b * T::STAGE;
        const unsigned char *nxt = smem + ((b + 1) & 3) * T::STAGE;
        const int fbuf = (b + 3) & 3;
        const bool more = HOT || (t + 1 < nkt);
        const bool fetch = HOT || (t + 3 < nkt);
        const bool fetch_fast = HOT || (t + 3 < nfast);
        const int kt = kt_begin + t + 3;
        micro.load_a(cur, 1);
        __builtin_amdgcn_sched_barrier(0);
        micro.mma_half(0, par, acc, [&](int row) {
            if (row < HALF0 && fetch_fast) dma_piece(kt, fbuf, row);
        });
        if (more) {
            // K step t+1 has landed when only the transfers issued after its own are outstanding: all of
            // t+2 and the first part of t+3 (transfers complete in order).  A stage that went through
            // registers has fewer transfers, so then everything is waited for.  lgkmcnt(0): this wave's
            // reads of buffer b (and its LDS writes of a guarded stage) are done.
            if (fetch_fast) wait_transfers<T::INST + HALF0>();
            else wait_transfers<0>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            micro.load_a(nxt, 0);
            micro.load_b(nxt, par ^ 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (!HOT && fetch && !fetch_fast) stage_guarded(kt, fbuf);
        __builtin_amdgcn_sched_barrier(0);
        micro.mma_half(1, par, acc, [&](int row) {
            if (row < HALF1 && fetch_fast) dma_piece(kt, fbuf, HALF0 + row);
        });
    };
    typedef std::true_type Hot;
    typedef std::false_type Any;

    if (nkt > 0) {
        // K steps 0, 1, 2 into buffers 0, 1, 2; K step 0 must have landed
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            if (t < nfast) {
#pragma unroll
                for (int q = 0; q < T::INST; ++q) dma_piece(kt_begin + t, t, q);
            } else if (t < nkt) {
                stage_guarded(kt_begin + t, t);
            }
        }
        if (nfast >= 3) wait_transfers<2 * T::INST>();
        else wait_transfers<0>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        micro.load_a(smem, 0);
        micro.load_b(smem, 0);
        __builtin_amdgcn_sched_barrier(0);

        int t = 0;
        for (; t + 7 <= nfast; t += 4) {        // K steps up to t + 6 are moved by transfers alone
            stage(Hot{}, 0, 0, t);
            stage(Hot{}, 1, 1, t + 1);
            stage(Hot{}, 2, 0, t + 2);
            stage(Hot{}, 3, 1, t + 3);
        }
        for (; t < nkt; t += 4) {
            stage(Any{}, 0, 0, t);
            if (t + 1 < nkt) stage(Any{}, 1, 1, t + 1);
            if (t + 2 < nkt) stage(Any{}, 2, 0, t + 2);
            if (t + 3 < nkt) stage(Any{}, 3, 1, t + 3);
        }
    }

    DmaMicro16<T>::store(acc, p, m0, n0, wm0, wn0, lane, z, m_own, n_own);
}

}  // namespace mig
