// Host-side launchers of the tile kernels and the constructors of their table entries: shared by the
// per-data-type table files (gemm_table_f32.hip, ...), each of which instantiates only its own kernels.
#pragma once
#include "gemm_kernel.hpp"
#include "gemm_kernel_dma.hpp"
#include "gemm_kernel_dma32.hpp"
#include "gemm_kernel_dma32t.hpp"
#include "gemm_kernel_ring.hpp"
#include "gemm_kernel_reg32.hpp"
#include "gemm_kernel_reg16.hpp"
#include "gemm_solo.hpp"
#include "gemm_table.h"


namespace mig {


template <class T, class K>
static hipError_t launch_solo(K kernel, int workgroups, int ksteps, int fill, hipStream_t stream)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                T::STAGE);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)workgroups), dim3(T::NT), T::STAGE, stream, ksteps, fill);
    return hipGetLastError();
}
template <class T>
static hipError_t solo_staged(int wg, int ks, int fill, hipStream_t st) { return launch_solo<T>(&solo_kernel<T>, wg, ks, fill, st); }
template <class T, class Micro>
static hipError_t solo_dma(int wg, int ks, int fill, hipStream_t st)
{
    return launch_solo<T>(&solo_kernel_micro<T, Micro>, wg, ks, fill, st);
}
template <class T>
static hipError_t solo_dma32(int wg, int ks, int fill, hipStream_t st)
{
    return launch_solo<T>(&solo_kernel_direct<T, Dma32Micro<T>>, wg, ks, fill, st);
}

template <class T, bool A_KC, bool B_NC>
static hipError_t launch_tile_variant(const Params &p, hipStream_t stream)
{
    static bool attr_done[64] = {false};          // per device: allow LDS beyond the default limit
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<T, A_KC, B_NC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel<T, A_KC, B_NC>), grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}

// the staged kernel in the orientation the problem has
template <class T>
static hipError_t launch_tile(const Params &p, hipStream_t stream)
{
    if (p.a_kc) return p.b_nc ? launch_tile_variant<T, true, true>(p, stream) : launch_tile_variant<T, true, false>(p, stream);
    return p.b_nc ? launch_tile_variant<T, false, true>(p, stream) : launch_tile_variant<T, false, false>(p, stream);
}

template <class T, class Micro>
static hipError_t launch_tile_dma(const Params &p, hipStream_t stream)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel_dma<T, Micro>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_dma<T, Micro>), grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <class T, class Micro = DmaMicro<T>>
static constexpr KernelInfo info_dma(const char *name, int prio, int eff_pct, int floor_ns, int setup_ns = 0)
{
    return KernelInfo{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile_dma<T, Micro>, prio, eff_pct, floor_ns,
                      setup_ns, &solo_dma<T, Micro>, T::MINB, 0, 0, 0, 0, 0, 0, 0.0, 30};
}
// the 16x16-block micro-kernel in one operand orientation: A canonical or with K contiguous
// (Params::a_kc), B canonical or, on square tiles, with N contiguous (Params::b_nc)
template <class T, bool A_KC, bool B_NC>
static hipError_t launch_dma16_variant(const Params &p, hipStream_t stream)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel_dma<T, DmaMicro16<T, A_KC, B_NC>, A_KC, B_NC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_dma<T, DmaMicro16<T, A_KC, B_NC>, A_KC, B_NC>), grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}
template <class T>
static hipError_t launch_tile_dma16(const Params &p, hipStream_t stream)
{
    if constexpr (T::BM == T::BN) {
        if (p.b_nc) return p.a_kc ? launch_dma16_variant<T, true, true>(p, stream) : launch_dma16_variant<T, false, true>(p, stream);
    } else {
        if (p.b_nc) return hipErrorInvalidValue;        // the selector never asks for it (b_nc_ok == 0)
    }
    return p.a_kc ? launch_dma16_variant<T, true, false>(p, stream) : launch_dma16_variant<T, false, false>(p, stream);
}
template <class T>
static constexpr KernelInfo info_dma16(const char *name, int prio, int eff_pct, int floor_ns, int setup_ns = 0)
{
    KernelInfo k = info_dma<T, DmaMicro16<T>>(name, prio, eff_pct, floor_ns, setup_ns);
    k.launch = &launch_tile_dma16<T>;
    k.a_kc_ok = 1;
    k.b_nc_ok = (T::BM == T::BN) ? 1 : 0;
    return k;
}

// the ring kernel in one operand orientation (as launch_dma16_variant)
template <class T, bool A_KC, bool B_NC>
static hipError_t launch_ring_variant(const Params &p, hipStream_t stream)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel_ring<T, A_KC, B_NC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_ring<T, A_KC, B_NC>), grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}
template <class T>
static hipError_t launch_tile_ring(const Params &p, hipStream_t stream)
{
    if constexpr (T::BM == T::BN) {
        if (p.b_nc) return p.a_kc ? launch_ring_variant<T, true, true>(p, stream) : launch_ring_variant<T, false, true>(p, stream);
    } else {
        if (p.b_nc) return hipErrorInvalidValue;        // the selector never asks for it (b_nc_ok == 0)
    }
    return p.a_kc ? launch_ring_variant<T, true, false>(p, stream) : launch_ring_variant<T, false, false>(p, stream);
}
template <class T>
static hipError_t solo_ring(int wg, int ks, int fill, hipStream_t st)
{
    return launch_solo<T>(&solo_kernel_ring<T>, wg, ks, fill, st);
}
template <class T>
static constexpr KernelInfo info_ring(const char *name, int prio, int eff_pct, int floor_ns, int setup_ns = 0)
{
    KernelInfo k = info_dma<T, DmaMicro16<T>>(name, prio, eff_pct, floor_ns, setup_ns);
    k.launch = &launch_tile_ring<T>;
    k.solo = &solo_ring<T>;
    k.a_kc_ok = 1;
    k.b_nc_ok = (T::BM == T::BN) ? 1 : 0;
    return k;
}

// the fp32 direct kernel for transposed operands (gemm_ex): A with K contiguous and / or B with N contiguous
template <class T, bool A_KC, bool B_NC>
static hipError_t launch_dma32t_variant(const Params &p, hipStream_t stream)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel_dma32t<T, A_KC, B_NC>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_dma32t<T, A_KC, B_NC>), grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <class T, bool TRANSPOSED_TOO>
static hipError_t launch_tile_dma32(const Params &p, hipStream_t stream)
{
    if (p.a_kc || p.b_nc) {
        if constexpr (TRANSPOSED_TOO) {
            if (p.a_kc) return p.b_nc ? launch_dma32t_variant<T, true, true>(p, stream) : launch_dma32t_variant<T, true, false>(p, stream);
            return launch_dma32t_variant<T, false, true>(p, stream);
        } else {
            return hipErrorInvalidValue;                // the selector never asks for it (a_kc_ok == b_nc_ok == 0)
        }
    }
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel_dma32<T>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL(gemm_kernel_dma32<T>, grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <class T>
static hipError_t launch_tile_dma32_im2row(const Params &p, hipStream_t stream)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel_dma32<T, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_dma32<T, true>), grid, dim3(T::NT), T::LDS_BYTES, stream, p);
    return hipGetLastError();
}

// TRANSPOSED_TOO: the configuration also takes transposed operands (through gemm_kernel_dma32t)
template <class T, bool TRANSPOSED_TOO = false>
static constexpr KernelInfo info_dma32(const char *name, int prio, int eff_pct, int floor_ns, int setup_ns = 0)
{
    KernelInfo k{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile_dma32<T, TRANSPOSED_TOO>, prio, eff_pct, floor_ns, setup_ns,
                 &solo_dma32<T>, T::MINB, 0, 0, 0, 0, 0, 0, 0.0, 0, 0, &launch_tile_dma32_im2row<T>, nullptr};
    k.a_kc_ok = TRANSPOSED_TOO ? 1 : 0;
    k.b_nc_ok = TRANSPOSED_TOO ? 1 : 0;
    return k;
}

template <class T>
static hipError_t launch_tile_reg32(const Params &p, hipStream_t stream)
{
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL(gemm_kernel_reg32<T>, grid, dim3(T::NT), 0, stream, p);   // its LDS is static
    return hipGetLastError();
}
template <class T>
static hipError_t launch_tile_reg32_im2row(const Params &p, hipStream_t stream)
{
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_reg32<T, IM2ROW_TAPS>), grid, dim3(T::NT), 0, stream, p);
    return hipGetLastError();
}
template <class T>
static hipError_t launch_tile_reg32_im2row_runs(const Params &p, hipStream_t stream)
{
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_reg32<T, IM2ROW_RUNS>), grid, dim3(T::NT), 0, stream, p);
    return hipGetLastError();
}
template <class T>
static hipError_t solo_reg32(int wg, int ks, int fill, hipStream_t st)
{
    hipLaunchKernelGGL(solo_kernel_reg<T>, dim3((unsigned)wg), dim3(T::NT), 0, st, ks, fill);
    return hipGetLastError();
}

template <class T>
static constexpr KernelInfo info_reg32(const char *name, int prio, int eff_pct, int step_ns, int setup_ns,
                                       int waves_per_simd)
{
    return KernelInfo{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile_reg32<T>, prio, eff_pct, step_ns, setup_ns,
                      &solo_reg32<T>, T::MINB, T::MAX_LDA, T::MAX_LDB, T::WM, T::WN, T::WAVES_K, waves_per_simd,
                      (T::WM * T::WN <= 256 ? 12.5e6 : 9.5e6) - (T::WAVES_K > 1 ? 1.0e6 : 0.0), 0, 0,
                      &launch_tile_reg32_im2row<T>, &launch_tile_reg32_im2row_runs<T>};
}

template <class T>
static hipError_t launch_tile_reg16(const Params &p, hipStream_t stream)
{
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_reg16<T, false>), grid, dim3(T::NT), 0, stream, p);   // its LDS is static
    return hipGetLastError();
}
template <class T>
static hipError_t launch_tile_reg16_im2row(const Params &p, hipStream_t stream)
{
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.split, 1);
    hipLaunchKernelGGL((gemm_kernel_reg16<T, true>), grid, dim3(T::NT), 0, stream, p);
    return hipGetLastError();
}
template <class T>
static hipError_t solo_reg16(int wg, int ks, int fill, hipStream_t st)
{
    hipLaunchKernelGGL(solo_kernel_reg16<T>, dim3((unsigned)wg), dim3(T::NT), 0, st, ks, fill);
    return hipGetLastError();
}
template <class T>
static constexpr KernelInfo info_reg16(const char *name, int prio, int eff_pct, int step_ns, int setup_ns,
                                       int waves_per_simd, double fill_bytes_per_us, int unaligned_pct = 80)
{
    return KernelInfo{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile_reg16<T>, prio, eff_pct, step_ns, setup_ns,
                      &solo_reg16<T>, T::MINB, T::MAX_LDA, T::MAX_LDB, T::WM, T::WN, T::WAVES_K, waves_per_simd,
                      fill_bytes_per_us, unaligned_pct, 0, &launch_tile_reg16_im2row<T>, nullptr};
}

template <class T>
static constexpr KernelInfo info(const char *name, int prio, int eff_pct, int floor_ns, int setup_ns = 0)
{
    return KernelInfo{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile<T>, prio, eff_pct, floor_ns, setup_ns,
                      &solo_staged<T>, T::MINB, 0, 0, 0, 0, 0, 0, 0.0, T::DT::ES == 4 ? 0 : 30, 1};
}

// Staged kernels:  dtype BM   BN  waves  MB  min workgroups per CU
// Direct-to-LDS:    dtype BM   BN  waves  fragment steps per stage, stages, min workgroups per CU
// Register-direct:  MFMA block, blocks per wave tile (m, n), waves (m, n, k), K steps in flight, min workgroups per CU
typedef Tile<F32, 128, 128, 2, 2, 4, 2> F32_128x128;
typedef Tile<F32, 256, 128, 4, 2, 4, 1> F32_256x128;
typedef Tile<F32, 64, 64, 2, 2, 2, 2> F32_64x64;
typedef Tile<F16, 256, 256, 2, 2, 8, 1> F16_256x256;
typedef Tile<F16, 128, 128, 2, 2, 8, 2> F16_128x128;
typedef Tile<F16, 64, 64, 2, 2, 2, 2> F16_64x64;
typedef Tile<BF16, 256, 256, 2, 2, 8, 1> BF16_256x256;
typedef Tile<BF16, 128, 128, 2, 2, 8, 2> BF16_128x128;
typedef Tile<BF16, 64, 64, 2, 2, 2, 2> BF16_64x64;
typedef Tile<I8, 256, 256, 2, 2, 8, 1> I8_256x256;
typedef Tile<I8, 128, 128, 2, 2, 4, 2> I8_128x128;
typedef Tile<I8, 64, 64, 2, 2, 4, 2> I8_64x64;


}  // namespace mig
