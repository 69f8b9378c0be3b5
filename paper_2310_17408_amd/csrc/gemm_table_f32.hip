// The f32 configurations of the kernel table (one translation unit per data type, so that they compile side by side).
#include "gemm_launchers.hpp"

namespace mig {

// name, open to automatic selection (> 0), % of the solo-mode rate reached on large problems,
// ns per K step of a workgroup that is alone on its CU, ns of fixed cost per launch beyond the launch itself.
// Register-direct kernels: % of the MFMA rate reached when many waves share a SIMD, ns per K step of a
// wave alone on its SIMD, ns of fixed cost, waves per SIMD.  All measured (graph replay, MI355X).
static const KernelInfo k_f32[] = {
    info<F32_128x128>("f32_128x128_w64x64", 0, 80, 2200, 1500),
    info<F32_256x128>("f32_256x128_w64x64", 0, 82, 3600, 1500),
    info<F32_64x64>("f32_64x64_w32x32", 1, 74, 780, 1500),
    info_dma32<Dma32Tile<64, 64, 2, 2, 4, 5, 2>>("f32_64x64_w32x32_dma_s5", 0, 75, 800, 2700),
    info_dma32<Dma32Tile<64, 64, 2, 2, 4, 2, 4>, true>("f32_64x64_w32x32_dma", 1, 85, 600, 1500),
    info_dma32<Dma32Tile<128, 64, 2, 2, 4, 2, 3>, true>("f32_128x64_w64x32_dma", 1, 93, 1300, 2700),
    info_dma32<Dma32Tile<128, 128, 2, 2, 4, 2, 2>, true>("f32_128x128_w64x64_dma", 1, 95, 2000, 2700),
    info_reg32<RegTile<16, 1, 1, 2, 2, 1, 12, 4>>("f32_32x32_w16x16_reg", 1, 45, 120, 0, 4),
    info_reg32<RegTile<16, 2, 2, 2, 2, 1, 8, 2>>("f32_64x64_w32x32_reg16", 1, 60, 360, 0, 2),
    info_reg32<RegTile<16, 1, 1, 1, 1, 4, 12, 4>>("f32_16x16_k4_reg", 1, 45, 160, 400, 4),
    info_reg32<RegTile<16, 1, 1, 1, 1, 8, 12, 2>>("f32_16x16_k8_reg", 1, 45, 140, 300, 4),
    info_reg32<RegTile<32, 1, 1, 1, 1, 4, 6, 2>>("f32_32x32_k4_reg", 1, 60, 335, 650, 3),
    info_reg32<RegTile<16, 2, 2, 1, 1, 4, 8, 2>>("f32_32x32_k4_reg16", 1, 60, 390, 600, 2),
};
const KernelInfo *kernel_table_f32(int *count)
{
    *count = (int)(sizeof(k_f32) / sizeof(k_f32[0]));
    return k_f32;
}

}  // namespace mig
