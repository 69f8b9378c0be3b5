// Kernel table: the family of tile configurations ("one micro-kernel per
// shape" in the paper's Sec. "Edge Cases") instantiated from the template in
// gemm_kernel.hpp, plus the launchers the host side calls through gemm_table.h.
#include "gemm_kernel.hpp"
#include "gemm_kernel_dma.hpp"
#include "gemm_kernel_dma32.hpp"
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

template <class T>
static hipError_t launch_tile_dma32(const Params &p, hipStream_t stream)
{
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

template <class T>
static constexpr KernelInfo info_dma32(const char *name, int prio, int eff_pct, int floor_ns, int setup_ns = 0)
{
    return KernelInfo{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile_dma32<T>, prio, eff_pct, floor_ns, setup_ns,
                      &solo_dma32<T>, T::MINB, 0, 0, 0, 0, 0, 0, 0.0, 0, 0, &launch_tile_dma32_im2row<T>, nullptr};
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
    hipLaunchKernelGGL(gemm_kernel_reg16<T>, grid, dim3(T::NT), 0, stream, p);   // its LDS is static
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
                                       int waves_per_simd, double fill_bytes_per_us)
{
    return KernelInfo{name, T::BM, T::BN, T::BK, T::NT, T::LDS_BYTES, &launch_tile_reg16<T>, prio, eff_pct, step_ns, setup_ns,
                      &solo_reg16<T>, T::MINB, T::MAX_LDA, T::MAX_LDB, T::WM, T::WN, T::WAVES_K, waves_per_simd,
                      fill_bytes_per_us, 30};
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

// name, open to automatic selection (> 0), % of the solo-mode rate reached on large problems,
// ns per K step of a workgroup that is alone on its CU, ns of fixed cost per launch beyond the launch itself.
// Register-direct kernels: % of the MFMA rate reached when many waves share a SIMD, ns per K step of a
// wave alone on its SIMD, ns of fixed cost, waves per SIMD.  All measured (graph replay, MI355X).
static const KernelInfo k_f32[] = {
    info<F32_128x128>("f32_128x128_w64x64", 0, 80, 2200, 1500),
    info<F32_256x128>("f32_256x128_w64x64", 0, 82, 3600, 1500),
    info<F32_64x64>("f32_64x64_w32x32", 1, 74, 780, 1500),
    info_dma32<Dma32Tile<64, 64, 2, 2, 4, 5, 2>>("f32_64x64_w32x32_dma_s5", 0, 75, 800, 2700),
    info_dma32<Dma32Tile<64, 64, 2, 2, 4, 2, 4>>("f32_64x64_w32x32_dma", 1, 85, 600, 1500),
    info_dma32<Dma32Tile<128, 64, 2, 2, 4, 2, 3>>("f32_128x64_w64x32_dma", 1, 93, 1300, 2700),
    info_dma32<Dma32Tile<128, 128, 2, 2, 4, 2, 2>>("f32_128x128_w64x64_dma", 1, 95, 2000, 2700),
    info_reg32<RegTile<16, 1, 1, 2, 2, 1, 12, 4>>("f32_32x32_w16x16_reg", 1, 45, 128, 0, 4),
    info_reg32<RegTile<16, 2, 2, 2, 2, 1, 8, 2>>("f32_64x64_w32x32_reg16", 1, 60, 360, 0, 2),
    info_reg32<RegTile<16, 1, 1, 1, 1, 4, 12, 4>>("f32_16x16_k4_reg", 1, 45, 150, 400, 4),
    info_reg32<RegTile<16, 1, 1, 1, 1, 8, 12, 2>>("f32_16x16_k8_reg", 1, 45, 150, 900, 4),
    info_reg32<RegTile<32, 1, 1, 1, 1, 4, 6, 2>>("f32_32x32_k4_reg", 1, 60, 335, 650, 3),
    info_reg32<RegTile<16, 2, 2, 1, 1, 4, 8, 2>>("f32_32x32_k4_reg16", 1, 60, 420, 800, 2),
};
static const KernelInfo k_f16[] = {
    info<F16_256x256>("f16_256x256_w128x128", 0, 50, 2500, 1500),
    info<F16_128x128>("f16_128x128_w64x64", 0, 47, 1700, 1500),
    info<F16_64x64>("f16_64x64_w32x32", 1, 30, 700, 1500),
    info_dma<DmaTile<F16, 128, 128, 2, 2, 4, 2, 2>>("f16_128x128_w64x64_dma", 0, 72, 880, 1500),
    info_dma<DmaTile<F16, 256, 256, 2, 4, 4, 2, 1>>("f16_256x256_w128x64_dma", 0, 82, 1800, 1500),
    info_dma16<DmaTile<F16, 256, 256, 2, 4, 4, 2, 1>>("f16_256x256_w128x64_dma16", 1, 87, 1700, 3000),
    info_dma16<DmaTile<F16, 128, 128, 2, 2, 4, 2, 2>>("f16_128x128_w64x64_dma16", 1, 75, 850, 3000),
    info_reg16<Reg16Tile<F16, 2, 2, 2, 1, 4, 3>>("f16_64x64_w32x32_reg", 1, 20, 300, 1200, 1, 12.5e6),
    info_reg16<Reg16Tile<F16, 2, 1, 1, 4, 4, 3>>("f16_32x32_k4_reg", 1, 20, 350, 900, 1, 11.0e6),
    info_dma16<DmaTile<F16, 128, 64, 2, 2, 4, 2, 3>>("f16_128x64_w64x32_dma16", 1, 55, 400, 3000),
    info_reg16<Reg16Tile<F16, 1, 1, 1, 4, 4, 4>>("f16_32x16_k4_reg", 1, 20, 250, 900, 1, 11.0e6),
};
static const KernelInfo k_bf16[] = {
    info<BF16_256x256>("bf16_256x256_w128x128", 0, 50, 2500, 1500),
    info<BF16_128x128>("bf16_128x128_w64x64", 0, 47, 1700, 1500),
    info<BF16_64x64>("bf16_64x64_w32x32", 1, 30, 700, 1500),
    info_dma<DmaTile<BF16, 128, 128, 2, 2, 4, 2, 2>>("bf16_128x128_w64x64_dma", 0, 72, 880, 1500),
    info_dma<DmaTile<BF16, 256, 256, 2, 4, 4, 2, 1>>("bf16_256x256_w128x64_dma", 0, 82, 1800, 1500),
    info_dma16<DmaTile<BF16, 256, 256, 2, 4, 4, 2, 1>>("bf16_256x256_w128x64_dma16", 1, 87, 1700, 3000),
    info_dma16<DmaTile<BF16, 128, 128, 2, 2, 4, 2, 2>>("bf16_128x128_w64x64_dma16", 1, 75, 850, 3000),
    info_reg16<Reg16Tile<BF16, 2, 2, 2, 1, 4, 3>>("bf16_64x64_w32x32_reg", 1, 20, 300, 1200, 1, 12.5e6),
    info_reg16<Reg16Tile<BF16, 2, 1, 1, 4, 4, 3>>("bf16_32x32_k4_reg", 1, 20, 350, 900, 1, 11.0e6),
    info_dma16<DmaTile<BF16, 128, 64, 2, 2, 4, 2, 3>>("bf16_128x64_w64x32_dma16", 1, 55, 400, 3000),
    info_reg16<Reg16Tile<BF16, 1, 1, 1, 4, 4, 4>>("bf16_32x16_k4_reg", 1, 20, 250, 900, 1, 11.0e6),
};
static const KernelInfo k_i8[] = {
    info<I8_256x256>("i8_256x256_w128x128", 0, 35, 2500, 1500),
    info<I8_128x128>("i8_128x128_w64x64", 0, 47, 800, 1500),
    info<I8_64x64>("i8_64x64_w32x32", 1, 25, 1000, 2000),
    info_dma<DmaTile<I8, 128, 128, 2, 2, 4, 2, 2>>("i8_128x128_w64x64_dma", 0, 62, 880, 1500),
    info_dma<DmaTile<I8, 256, 256, 2, 4, 4, 2, 1>>("i8_256x256_w128x64_dma", 0, 75, 1800, 1500),
    info_dma16<DmaTile<I8, 256, 256, 2, 4, 4, 2, 1>>("i8_256x256_w128x64_dma16", 1, 80, 1700, 3000),
    info_dma16<DmaTile<I8, 128, 128, 2, 2, 4, 2, 2>>("i8_128x128_w64x64_dma16", 1, 65, 850, 3000),
    info_reg16<Reg16Tile<I8, 2, 2, 2, 1, 3, 2>>("i8_128x64_w64x32_reg", 1, 20, 400, 1200, 1, 9.5e6),
    info_reg16<Reg16Tile<I8, 2, 1, 1, 4, 3, 2>>("i8_64x32_k4_reg", 1, 20, 700, 1200, 1, 7.0e6),
    info_reg16<Reg16Tile<I8, 1, 1, 1, 4, 3, 2>>("i8_64x16_k4_reg", 1, 20, 450, 900, 1, 9.5e6),
    info_dma16<DmaTile<I8, 128, 64, 2, 2, 4, 2, 3>>("i8_128x64_w64x32_dma16", 1, 45, 400, 3000),
};

int kernel_count(int dtype)
{
    switch (dtype) {
    case 0: return (int)(sizeof(k_f32) / sizeof(k_f32[0]));
    case 1: return (int)(sizeof(k_f16) / sizeof(k_f16[0]));
    case 2: return (int)(sizeof(k_i8) / sizeof(k_i8[0]));
    case 3: return (int)(sizeof(k_bf16) / sizeof(k_bf16[0]));
    default: return 0;
    }
}

const KernelInfo *kernel_info(int dtype, int id)
{
    if (id < 0 || id >= kernel_count(dtype)) return nullptr;
    return dtype == 0 ? &k_f32[id] : dtype == 1 ? &k_f16[id] : dtype == 2 ? &k_i8[id] : &k_bf16[id];
}

static unsigned blocks_for(int64_t total)
{
    int64_t b = (total + 255) / 256;
    if (b > 8192) b = 8192;
    if (b < 1) b = 1;
    return (unsigned)b;
}

hipError_t launch_reduce(int dtype, const void *ws, void *C, int M, int N, int64_t ldc, int split,
                         uint32_t alpha_bits, uint32_t beta_bits, int use_beta, hipStream_t stream, int c_type)
{
    const unsigned g = blocks_for((int64_t)M * N);
    if (dtype == 2)
        hipLaunchKernelGGL(reduce_kernel<int>, dim3(g), dim3(256), 0, stream, (const int *)ws, (int *)C, M, N, ldc,
                           split, alpha_bits, beta_bits, use_beta, C_WIDE);
    else
        hipLaunchKernelGGL(reduce_kernel<float>, dim3(g), dim3(256), 0, stream, (const float *)ws, (float *)C, M, N,
                           ldc, split, alpha_bits, beta_bits, use_beta, c_type);
    return hipGetLastError();
}

hipError_t launch_im2row_matrix(const float *image, float *matrix, int64_t rows, int64_t K, const Im2row &g,
                                hipStream_t stream)
{
    hipLaunchKernelGGL(im2row_matrix_kernel, dim3(blocks_for(rows * K)), dim3(256), 0, stream, image, matrix, rows, K, g);
    return hipGetLastError();
}

hipError_t launch_scale(int dtype, void *C, int M, int N, int64_t ldc, uint32_t beta_bits, int use_beta,
                        hipStream_t stream, int c_type)
{
    const unsigned g = blocks_for((int64_t)M * N);
    if (dtype == 2)
        hipLaunchKernelGGL(scale_kernel<int>, dim3(g), dim3(256), 0, stream, (int *)C, M, N, ldc, beta_bits, use_beta, C_WIDE);
    else
        hipLaunchKernelGGL(scale_kernel<float>, dim3(g), dim3(256), 0, stream, (float *)C, M, N, ldc, beta_bits,
                           use_beta, c_type);
    return hipGetLastError();
}

}  // namespace mig
