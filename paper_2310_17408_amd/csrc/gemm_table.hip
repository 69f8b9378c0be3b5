// Kernel table: the family of tile configurations ("one micro-kernel per
// shape" in the paper's Sec. "Edge Cases") instantiated from the template in
// gemm_kernel.hpp, plus the launchers the host side calls through gemm_table.h.
#include "gemm_kernel.hpp"
#include "gemm_table.h"

namespace mig {

// defined in gemm_table_f32.hip, gemm_table_f16.hip, gemm_table_bf16.hip, gemm_table_i8.hip
const KernelInfo *kernel_table_f32(int *count);
const KernelInfo *kernel_table_f16(int *count);
const KernelInfo *kernel_table_bf16(int *count);
const KernelInfo *kernel_table_i8(int *count);

static const KernelInfo *table_of(int dtype, int *count)
{
    switch (dtype) {
    case 0: return kernel_table_f32(count);
    case 1: return kernel_table_f16(count);
    case 2: return kernel_table_i8(count);
    case 3: return kernel_table_bf16(count);
    default: *count = 0; return nullptr;
    }
}

// The im2row transform written out (paper Sec. "Rectangular Matrices"): element (row, k) of the
// matrix, row = (b, oh, ow), k = (r, s, c), is the image element the tap (r, s) of that output pixel
// meets, or zero outside the image.  Used for geometries the fused kernels do not take.
template <class E>
__global__ void __launch_bounds__(256) im2row_matrix_kernel(const E *__restrict__ image, E *__restrict__ matrix,
                                                            int64_t rows, int64_t K, const Im2row g)
{
    const int64_t total = rows * K;
    const int per_image = g.Hout * g.Wout;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = idx / K;
        const int k = (int)(idx - row * K);
        const int tap = k / g.Cin, c = k - tap * g.Cin;
        const int r = tap / g.kw, s = tap - r * g.kw;
        const int b = (int)(row / per_image), rem = (int)(row - (int64_t)b * per_image);
        const int oh = rem / g.Wout, ow = rem - oh * g.Wout;
        const int ih = oh * g.stride_h - g.pad_h + r, iw = ow * g.stride_w - g.pad_w + s;
        E v = 0;                                              // all-zero bits are the value 0 in every type
        if ((uint32_t)ih < (uint32_t)g.H && (uint32_t)iw < (uint32_t)g.W)
            v = image[(((int64_t)b * g.H + ih) * g.W + iw) * g.Cin + c];
        matrix[idx] = v;
    }
}

int kernel_count(int dtype)
{
    int n = 0;
    table_of(dtype, &n);
    return n;
}

const KernelInfo *kernel_info(int dtype, int id)
{
    int n = 0;
    const KernelInfo *t = table_of(dtype, &n);
    return (t && id >= 0 && id < n) ? &t[id] : nullptr;
}

static unsigned blocks_for(int64_t total)
{
    int64_t b = (total + 255) / 256;
    if (b > (1 << 20)) b = 1 << 20;                  // measured: grid-stride loops of many rounds stream slower
    if (b < 1) b = 1;
    return (unsigned)b;
}

hipError_t launch_reduce(int dtype, const void *ws, void *C, int M, int N, int64_t ldc, int split,
                         uint32_t alpha_bits, uint32_t beta_bits, int use_beta, hipStream_t stream, int c_type)
{
    const bool vec = M % 4 == 0 && ldc % 4 == 0 && (uintptr_t)C % 16 == 0 && (uintptr_t)ws % 16 == 0 &&
                     (dtype == 2 || c_type == C_WIDE);
    const unsigned g = blocks_for(vec ? (int64_t)M * N / 4 : (int64_t)M * N);
    if (dtype == 2) {
        if (vec)
            hipLaunchKernelGGL((reduce_kernel<int, true>), dim3(g), dim3(256), 0, stream, (const int *)ws, (int *)C, M, N, ldc,
                               split, alpha_bits, beta_bits, use_beta, C_WIDE);
        else
            hipLaunchKernelGGL((reduce_kernel<int, false>), dim3(g), dim3(256), 0, stream, (const int *)ws, (int *)C, M, N, ldc,
                               split, alpha_bits, beta_bits, use_beta, C_WIDE);
    } else {
        if (vec)
            hipLaunchKernelGGL((reduce_kernel<float, true>), dim3(g), dim3(256), 0, stream, (const float *)ws, (float *)C, M, N,
                               ldc, split, alpha_bits, beta_bits, use_beta, c_type);
        else
            hipLaunchKernelGGL((reduce_kernel<float, false>), dim3(g), dim3(256), 0, stream, (const float *)ws, (float *)C, M, N,
                               ldc, split, alpha_bits, beta_bits, use_beta, c_type);
    }
    return hipGetLastError();
}

hipError_t launch_im2row_matrix(int es, const void *image, void *matrix, int64_t rows, int64_t K, const Im2row &g,
                                hipStream_t stream)
{
    const dim3 grid(blocks_for(rows * K));
    if (es == 4)
        hipLaunchKernelGGL(im2row_matrix_kernel<uint32_t>, grid, dim3(256), 0, stream, (const uint32_t *)image, (uint32_t *)matrix, rows, K, g);
    else if (es == 2)
        hipLaunchKernelGGL(im2row_matrix_kernel<uint16_t>, grid, dim3(256), 0, stream, (const uint16_t *)image, (uint16_t *)matrix, rows, K, g);
    else
        hipLaunchKernelGGL(im2row_matrix_kernel<uint8_t>, grid, dim3(256), 0, stream, (const uint8_t *)image, (uint8_t *)matrix, rows, K, g);
    return hipGetLastError();
}

hipError_t launch_scale(int dtype, void *C, int M, int N, int64_t ldc, uint32_t beta_bits, int use_beta,
                        hipStream_t stream, int c_type)
{
    const bool vec = M % 4 == 0 && ldc % 4 == 0 && (uintptr_t)C % 16 == 0 && (dtype == 2 || c_type == C_WIDE);
    const unsigned g = blocks_for(vec ? (int64_t)M * N / 4 : (int64_t)M * N);
    if (dtype == 2) {
        if (vec) hipLaunchKernelGGL((scale_kernel<int, true>), dim3(g), dim3(256), 0, stream, (int *)C, M, N, ldc, beta_bits, use_beta, C_WIDE);
        else hipLaunchKernelGGL((scale_kernel<int, false>), dim3(g), dim3(256), 0, stream, (int *)C, M, N, ldc, beta_bits, use_beta, C_WIDE);
    } else {
        if (vec) hipLaunchKernelGGL((scale_kernel<float, true>), dim3(g), dim3(256), 0, stream, (float *)C, M, N, ldc, beta_bits, use_beta, c_type);
        else hipLaunchKernelGGL((scale_kernel<float, false>), dim3(g), dim3(256), 0, stream, (float *)C, M, N, ldc, beta_bits, use_beta, c_type);
    }
    return hipGetLastError();
}

}  // namespace mig
