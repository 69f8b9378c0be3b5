// Host-side view of the kernel table (no device code in this header).
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

namespace mig {

// Geometry of a convolution whose im2row matrix is the canonical B (one row per output pixel, K =
// kh*kw*Cin contiguous), read from the channels-last image in place: row n = (b, oh, ow), column
// k = (r, s, c) is image[b][oh*stride_h - pad_h + r][ow*stride_w - pad_w + s][c], zero outside the image.
struct Im2row {
    int H, W, Cin, kw;
    int stride_h, stride_w, pad_h, pad_w;
    int Hout, Wout;
};

// One canonical problem (C column-major, A with M contiguous, B with K contiguous)
// and how the grid covers it.
struct Params {
    const void *A;
    const void *B;
    void *C;
    void *ws;              // partial tiles [split][N][M] when split > 1
    int64_t lda, ldb, ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int ktiles;            // number of BK steps covering K
    int ktiles_per_split;  // BK steps per blockIdx.y slice
    int split;             // gridDim.y
    uint32_t alpha_bits, beta_bits;
    int use_beta;          // beta != 0: the old C is read
    int vecA, vecB;        // operand rows are 16-byte aligned (direct global -> LDS transfers of 16 bytes)
    int a_kc, b_nc;        // transposed operands: A has K contiguous / B has N contiguous (staged kernels only)
    int group_m;           // tiles per column group in the tile order
    int xcd_remap;         // deal contiguous tile ranges to the 8 XCDs
    Im2row conv;           // implicit-im2row launches only: B is the image, ldb is unused
    int c_type;            // how C is stored: C_WIDE as the accumulators (fp32 / int32), C_F16, C_BF16 (16-bit inputs only)
};
enum { C_WIDE = 0, C_F16 = 1, C_BF16 = 2 };

struct KernelInfo {
    const char *name;
    int BM, BN, BK;   // workgroup tile; BK = K elements per step
    int threads;
    int lds_bytes;
    hipError_t (*launch)(const Params &, hipStream_t);
    // prio > 0: open to automatic selection (the host's timing model picks among these);
    // prio 0: only by explicit request.  eff_pct: the share of its micro-kernel's solo-mode rate
    // that the whole kernel reaches on large problems (measured), used by the timing model.
    int prio;
    int eff_pct;
    int step_floor_ns;       // time of one K step when the workgroup has its CU to itself (latency-bound)
    int setup_ns;            // fixed cost per launch beyond the launch itself (prologue of the kernel)
    // Solo mode: `workgroups` workgroups repeat the micro-kernel of one K step `ksteps` times on
    // operands resident in LDS (fill 0: zeros, 1: pseudo-random finite values).
    hipError_t (*solo)(int workgroups, int ksteps, int fill, hipStream_t);
    int min_blocks_per_cu;   // workgroups per CU the kernel is built to co-reside with
    int64_t max_lda, max_ldb;  // largest canonical leading dimensions the kernel's 32-bit lane offsets allow (0: any)
    // Register-direct kernels (0 for the others): the tile of C one wave owns, the number of waves
    // that share it along K, waves per SIMD that fit, and the rate at which the chip fills the
    // vector caches for wave tiles of that size (bytes per microsecond).  For these kernels
    // step_floor_ns is the time of one K step of a wave that has its SIMD to itself.
    int wave_m, wave_n, waves_k, waves_per_simd;
    double fill_bytes_per_us;
    // Speed, in % of its normal one, when an operand's rows are not 16-byte aligned (0 = 100): the
    // fp16/int8 kernels then load through misaligned vectors, which the memory system splits, and the
    // direct ones stage every tile through registers.
    int unaligned_pct;
    int transposed_ok;       // takes A with K contiguous and B with N contiguous as well (Params::a_kc, b_nc)
    // the same configuration with B read through the im2row map of Params::conv (nullptr: not built):
    // for Cin a multiple of the K step (a step lies in one filter tap), and for any Cin (element by element)
    hipError_t (*launch_im2row)(const Params &, hipStream_t);
    hipError_t (*launch_im2row_runs)(const Params &, hipStream_t);
    int a_kc_ok;             // takes A with K contiguous (Params::a_kc) at its normal speed
    int b_nc_ok;             // takes B with N contiguous (Params::b_nc) at its normal speed
};

int kernel_count(int dtype);                       // dtype: 0 fp32, 1 fp16, 2 int8, 3 bf16
const KernelInfo *kernel_info(int dtype, int id);  // nullptr if out of range

hipError_t launch_reduce(int dtype, const void *ws, void *C, int M, int N, int64_t ldc, int split,
                         uint32_t alpha_bits, uint32_t beta_bits, int use_beta, hipStream_t stream, int c_type = C_WIDE);
// The im2row matrix [rows][K] (row-major, K = kh*kw*Cin, kh given by K) of a channels-last image whose
// elements have `es` bytes (4, 2 or 1), in the same type.
hipError_t launch_im2row_matrix(int es, const void *image, void *matrix, int64_t rows, int64_t K, const Im2row &g,
                                hipStream_t stream);
hipError_t launch_scale(int dtype, void *C, int M, int N, int64_t ldc, uint32_t beta_bits, int use_beta,
                        hipStream_t stream, int c_type = C_WIDE);

}  // namespace mig
