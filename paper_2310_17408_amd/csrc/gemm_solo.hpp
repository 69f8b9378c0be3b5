// Solo mode: the micro-kernel of a tile configuration run on its own, as in the
// paper's Sec. "Solo Mode" (the micro-kernel invoked directly, KC loop only).
// Every workgroup fills one LDS stage with operands once and then repeats the
// fragment reads and MFMAs of a K step `ksteps` times on it: no global traffic,
// no barriers, no epilogue.  The rate it reaches is what the MFMA pipes, the
// LDS and the clock the chip sustains under that load allow for this tile, i.e.
// the measured ceiling of the corresponding GEMM kernel.
#pragma once
#include "gemm_kernel.hpp"
#include "gemm_kernel_dma.hpp"
#include "gemm_kernel_dma32.hpp"
#include "gemm_kernel_ring.hpp"
#include "gemm_kernel_reg32.hpp"
#include "gemm_kernel_reg16.hpp"

namespace mig {

__device__ int g_solo_sink;   // keeps the accumulators alive; never written in practice

// Operand bits for byte offset `i` of the stage: zeros, or a hash shaped into finite values of the
// data type (fp32 in [0.5,1) with random sign, binary16 with exponent < 16, any int8).
template <int ES>
__device__ __forceinline__ int solo_word(uint32_t i, int fill)
{
    if (fill == 0) return 0;
    uint32_t h = (i + 12345u) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    if (ES == 2) h &= 0xBFFFBFFFu;
    if (ES == 4) h = (h & 0x807FFFFFu) | 0x3F000000u;
    return (int)h;
}

template <int ES, int NT>
__device__ __forceinline__ void solo_fill(unsigned char *smem, int bytes, int fill)
{
    for (int i = threadIdx.x * 16; i < bytes; i += NT * 16) {
        v4i r;
#pragma unroll
        for (int w = 0; w < 4; ++w) r[w] = solo_word<ES>((uint32_t)(i + 4 * w), fill);
        *(v4i *)(smem + i) = r;
    }
    __syncthreads();
}

template <class accv, int TM, int TN>
__device__ __forceinline__ void solo_finish(accv (&acc)[TM][TN])
{
    float r = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) r += (float)acc[i][j][0];
    if (r == 1234567.0f) g_solo_sink = 1;   // integer-valued: reachable for int accumulators too, so nothing is dead code
}

// staged kernels (gemm_kernel.hpp)
template <class T>
__global__ void __launch_bounds__(T::NT, T::MINB) solo_kernel(int ksteps, int fill)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    solo_fill<T::DT::ES, T::NT>(smem, T::STAGE, fill);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;
    typename T::DT::accv acc[T::TM][T::TN];
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    for (int it = 0; it < ksteps; ++it) {
        micro_kernel<T>(smem, wm0, wn0, lane, acc);
        __builtin_amdgcn_sched_barrier(0);
    }
    solo_finish(acc);
}

// direct kernels (gemm_kernel_dma.hpp, gemm_kernel_dma32.hpp): Micro is DmaMicro<T> or Dma32Micro<T>;
// the same register double buffering of fragments as in the GEMM's K loop
template <class T, class Micro>
__global__ void __launch_bounds__(T::NT, T::MINB) solo_kernel_direct(int ksteps, int fill)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    solo_fill<T::DT::ES, T::NT>(smem, T::STAGE, fill);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;
    Micro micro;
    micro.init(lane, wm0, wn0);
    typename Micro::accv acc[T::TM][T::TN];
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    typename Micro::aset fa[2];
    typename Micro::bset fb[2];
    micro.load(smem, 0, fa[0], fb[0]);
    for (int it = 0; it < ksteps; ++it) {
#pragma unroll
        for (int s = 0; s < T::KSTEPS; ++s) {
            // reads of the next step (the first step of the next pass after the last one) under
            // the MFMAs of this step
            micro.load(smem, (s + 1) % T::KSTEPS, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            Micro::mma(fa[s & 1], fb[s & 1], acc);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    solo_finish(acc);
}

// fp16 / bf16 / int8 direct kernels (gemm_kernel_dma.hpp): Micro is DmaMicro<T> or DmaMicro16<T>, which
// hold their own double-buffered fragments
template <class T, class Micro>
__global__ void __launch_bounds__(T::NT, T::MINB) solo_kernel_micro(int ksteps, int fill)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    solo_fill<T::DT::ES, T::NT>(smem, T::STAGE, fill);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;
    Micro micro;
    micro.init(lane, wm0, wn0);
    typename Micro::accv acc[Micro::TM][Micro::TN];
#pragma unroll
    for (int i = 0; i < Micro::TM; ++i)
#pragma unroll
        for (int j = 0; j < Micro::TN; ++j)
#pragma unroll
            for (int v = 0; v < Micro::ACC; ++v) acc[i][j][v] = 0;
    micro.load(smem, 0);
    for (int it = 0; it < ksteps; ++it) {
#pragma unroll
        for (int s = 0; s < Micro::STEPS; ++s) {
            micro.load(smem, (s + 1) % Micro::STEPS);
            micro.mma(s, acc);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    solo_finish(acc);
}

// ring kernels (gemm_kernel_ring.hpp): the two halves of a stage with the fragment reads of the next half
// under them, two passes per iteration so that the register sets alternate as in the GEMM's K loop
template <class T>
__global__ void __launch_bounds__(T::NT, T::MINB) solo_kernel_ring(int ksteps, int fill)
{
    typedef RingMicro16<T> Micro;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    solo_fill<T::DT::ES, T::NT>(smem, T::STAGE, fill);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave % T::WAVES_M) * T::WM, wn0 = (wave / T::WAVES_M) * T::WN;
    Micro micro;
    micro.init(lane, wm0, wn0);
    typename Micro::accv acc[Micro::TM][Micro::TN];
#pragma unroll
    for (int i = 0; i < Micro::TM; ++i)
#pragma unroll
        for (int j = 0; j < Micro::TN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0;
    micro.load_a(smem, 0);
    micro.load_b(smem, 0);
    for (int it = 0; it < ksteps; it += 2) {
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            micro.load_a(smem, 1);
            __builtin_amdgcn_sched_barrier(0);
            micro.mma_half(0, par, acc, [](int) {});
            micro.load_a(smem, 0);
            micro.load_b(smem, par ^ 1);
            __builtin_amdgcn_sched_barrier(0);
            micro.mma_half(1, par, acc, [](int) {});
        }
    }
    solo_finish(acc);
}

// register-direct kernels (gemm_kernel_reg32.hpp): the operands of one K step stay in registers
template <class T>
__global__ void __launch_bounds__(T::NT, T::MINB) solo_kernel_reg(int ksteps, int fill)
{
    typedef RegMicro<T> Micro;
    typename Micro::aset fa;
    typename Micro::bset fb;
#pragma unroll
    for (int t = 0; t < T::KG; ++t) {
#pragma unroll
        for (int i = 0; i < T::TM; ++i)
            fa.v[t][i] = __builtin_bit_cast(float, solo_word<4>((uint32_t)(threadIdx.x * 64 + t * 4 + i) * 4u, fill));
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
            fb.v[j][t] = __builtin_bit_cast(float, solo_word<4>((uint32_t)(threadIdx.x * 64 + 32 + t * 4 + j) * 4u, fill));
    }
    typename Micro::accv acc[T::TM][T::TN];
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int v = 0; v < T::ACC; ++v) acc[i][j][v] = 0;
    for (int it = 0; it < ksteps; ++it) {
        Micro::mma(fa, fb, acc);
        __builtin_amdgcn_sched_barrier(0);
    }
    solo_finish(acc);
}

// register-direct kernels for 16- and 8-bit inputs (gemm_kernel_reg16.hpp): the operands of one K step
// stay in registers; every pass repeats the register transposes of A and the MFMAs
template <class T>
__global__ void __launch_bounds__(T::NT, T::MINB) solo_kernel_reg16(int ksteps, int fill)
{
    typedef Reg16Micro<T> Micro;
    typename Micro::step x;
#pragma unroll
    for (int t = 0; t < T::KCH; ++t) x.a[t] = solo_word<T::ES>((uint32_t)(threadIdx.x * 64 + t) * 4u, fill);
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
        for (int w = 0; w < 4; ++w) x.b[j][w] = solo_word<T::ES>((uint32_t)(threadIdx.x * 64 + 32 + 4 * j + w) * 4u, fill);
    typename Micro::accv acc[T::TM][T::TN];
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int v = 0; v < T::ACC; ++v) acc[i][j][v] = 0;
    for (int it = 0; it < ksteps; ++it) {
        Micro::mma(x, acc);
        __builtin_amdgcn_sched_barrier(0);
    }
    solo_finish(acc);
}

}  // namespace mig
