// The bf16 configurations of the kernel table (one translation unit per data type, so that they compile side by side).
#include "gemm_launchers.hpp"

namespace mig {

// name, open to automatic selection (> 0), % of the solo-mode rate reached on large problems,
// ns per K step of a workgroup that is alone on its CU, ns of fixed cost per launch beyond the launch itself.
// Register-direct kernels: % of the MFMA rate reached when many waves share a SIMD, ns per K step of a
// wave alone on its SIMD, ns of fixed cost, waves per SIMD.  All measured (graph replay, MI355X).
static const KernelInfo k_bf16[] = {
    info<BF16_256x256>("bf16_256x256_w128x128", 0, 50, 2500, 1500),
    info<BF16_128x128>("bf16_128x128_w64x64", 0, 47, 1700, 1500),
    info<BF16_64x64>("bf16_64x64_w32x32", 1, 30, 700, 1500),
    info_dma<DmaTile<BF16, 128, 128, 2, 2, 4, 2, 2>>("bf16_128x128_w64x64_dma", 0, 72, 880, 1500),
    info_dma<DmaTile<BF16, 256, 256, 2, 4, 4, 2, 1>>("bf16_256x256_w128x64_dma", 0, 82, 1800, 1500),
    info_dma16<DmaTile<BF16, 256, 256, 2, 4, 4, 2, 1>>("bf16_256x256_w128x64_dma16", 0, 87, 1700, 3000),
    info_dma16<DmaTile<BF16, 128, 128, 2, 2, 4, 2, 2>>("bf16_128x128_w64x64_dma16", 1, 75, 850, 3000),
    info_reg16<Reg16Tile<BF16, 2, 2, 2, 1, 4, 3>>("bf16_64x64_w32x32_reg", 1, 20, 300, 1200, 1, 12.5e6),
    info_reg16<Reg16Tile<BF16, 2, 1, 1, 4, 4, 3>>("bf16_32x32_k4_reg", 1, 20, 350, 900, 1, 11.0e6),
    info_dma16<DmaTile<BF16, 128, 64, 2, 2, 4, 2, 3>>("bf16_128x64_w64x32_dma16", 1, 55, 400, 3000),
    info_reg16<Reg16Tile<BF16, 1, 1, 1, 4, 4, 4>>("bf16_32x16_k4_reg", 1, 20, 250, 900, 1, 11.0e6),
    info_ring<DmaTile<BF16, 256, 256, 2, 4, 2, 4, 1>>("bf16_256x256_w128x64_ring", 1, 90, 740, 3000),
    info_ring<DmaTile<BF16, 128, 128, 2, 4, 2, 4, 2>>("bf16_128x128_w64x32_ring", 1, 75, 310, 3000),
};
const KernelInfo *kernel_table_bf16(int *count)
{
    *count = (int)(sizeof(k_bf16) / sizeof(k_bf16[0]));
    return k_bf16;
}

}  // namespace mig
