// The i8 configurations of the kernel table (one translation unit per data type, so that they compile side by side).
#include "gemm_launchers.hpp"

namespace mig {

// name, open to automatic selection (> 0), % of the solo-mode rate reached on large problems,
// ns per K step of a workgroup that is alone on its CU, ns of fixed cost per launch beyond the launch itself.
// Register-direct kernels: % of the MFMA rate reached when many waves share a SIMD, ns per K step of a
// wave alone on its SIMD, ns of fixed cost, waves per SIMD.  All measured (graph replay, MI355X).
static const KernelInfo k_i8[] = {
    info<I8_256x256>("i8_256x256_w128x128", 0, 35, 2500, 1500),
    info<I8_128x128>("i8_128x128_w64x64", 0, 47, 800, 1500),
    info<I8_64x64>("i8_64x64_w32x32", 1, 25, 1000, 2000),
    info_dma<DmaTile<I8, 128, 128, 2, 2, 4, 2, 2>>("i8_128x128_w64x64_dma", 0, 62, 880, 1500),
    info_dma<DmaTile<I8, 256, 256, 2, 4, 4, 2, 1>>("i8_256x256_w128x64_dma", 0, 75, 1800, 1500),
    info_dma16<DmaTile<I8, 256, 256, 2, 4, 4, 2, 1>>("i8_256x256_w128x64_dma16", 0, 80, 1700, 3000),
    info_dma16<DmaTile<I8, 128, 128, 2, 2, 4, 2, 2>>("i8_128x128_w64x64_dma16", 1, 65, 850, 3000),
    info_reg16<Reg16Tile<I8, 2, 2, 2, 1, 3, 2>>("i8_128x64_w64x32_reg", 1, 20, 400, 1200, 1, 9.5e6),
    info_reg16<Reg16Tile<I8, 2, 1, 1, 4, 3, 2>>("i8_64x32_k4_reg", 1, 20, 700, 1200, 1, 7.0e6),
    info_reg16<Reg16Tile<I8, 1, 1, 1, 4, 3, 2>>("i8_64x16_k4_reg", 1, 20, 450, 900, 1, 9.5e6),
    info_dma16<DmaTile<I8, 128, 64, 2, 2, 4, 2, 3>>("i8_128x64_w64x32_dma16", 1, 45, 400, 3000),
    info_ring<DmaTile<I8, 256, 256, 2, 4, 2, 4, 1>>("i8_256x256_w128x64_ring", 1, 79, 900, 3000),
    info_ring<DmaTile<I8, 128, 128, 2, 4, 2, 4, 2>>("i8_128x128_w64x32_ring", 1, 64, 320, 3000),
};
const KernelInfo *kernel_table_i8(int *count)
{
    *count = (int)(sizeof(k_i8) / sizeof(k_i8[0]));
    return k_i8;
}

}  // namespace mig
