// Host-only exerciser of the library's argument checks, quick returns, selection model, workspace sizing
// and convolution geometry, meant to be built with -fsanitize=address,undefined (see
// tests/test_sanitized_host.py).  The kernel table and the launchers are replaced by stand-ins that record
// what would have been launched, so no GPU and no HIP runtime is needed; every pointer handed to the entry
// points is a fake device address that must never be dereferenced by host code.
#include "../../include/mi_gemm.h"
#include "../../paper_2310_17408_amd/csrc/gemm_table.h"

#include <limits.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

using namespace mig;

static int g_launches = 0, g_reduces = 0, g_scales = 0, g_matrices = 0;
static Params g_last;

static hipError_t fake_launch(const Params &p, hipStream_t) { g_last = p; ++g_launches; return hipSuccess; }
static hipError_t fake_solo(int, int, int, hipStream_t) { return hipSuccess; }

// one table for every data type: an LDS-staged tile, a large one, two register-direct ones (one sharing
// a tile along K) - the kinds of entries the timing model distinguishes
static KernelInfo make(const char *name, int bm, int bn, int bk, int prio, int eff, int floor_ns, int setup_ns, int minb,
                       int wave_m, int wave_n, int waves_k, int waves_per_simd, double fill, bool conv)
{
    KernelInfo k;
    memset(&k, 0, sizeof(k));
    k.name = name; k.BM = bm; k.BN = bn; k.BK = bk; k.threads = 256; k.lds_bytes = 0; k.launch = &fake_launch;
    k.prio = prio; k.eff_pct = eff; k.step_floor_ns = floor_ns; k.setup_ns = setup_ns; k.solo = &fake_solo;
    k.min_blocks_per_cu = minb; k.max_lda = waves_k ? ((int64_t)1 << 26) : 0; k.max_ldb = k.max_lda;
    k.wave_m = wave_m; k.wave_n = wave_n; k.waves_k = waves_k; k.waves_per_simd = waves_per_simd; k.fill_bytes_per_us = fill;
    k.unaligned_pct = 30; k.transposed_ok = waves_k ? 0 : 1;
    if (conv) { k.launch_im2row = &fake_launch; k.launch_im2row_runs = waves_k ? &fake_launch : nullptr; }
    k.a_kc_ok = 0; k.b_nc_ok = 0;
    return k;
}
static const KernelInfo g_table[] = {
    make("t_64x64", 64, 64, 32, 1, 60, 700, 1500, 4, 0, 0, 0, 0, 0.0, true),
    make("t_128x128", 128, 128, 32, 1, 90, 900, 1500, 2, 0, 0, 0, 0, 0.0, true),
    make("t_256x256", 256, 256, 64, 1, 88, 800, 3000, 1, 0, 0, 0, 0, 0.0, false),
    make("t_32x32_reg", 32, 32, 16, 1, 20, 300, 1200, 4, 16, 16, 1, 2, 12.5e6, true),
    make("t_32x32_k4_reg", 32, 32, 16, 1, 20, 350, 900, 4, 32, 32, 4, 1, 9.5e6, true),
    make("t_only_by_request", 64, 64, 16, 0, 50, 700, 1500, 2, 0, 0, 0, 0, 0.0, false),
};
namespace mig {
int kernel_count(int dtype) { return (dtype >= 0 && dtype < 4) ? (int)(sizeof(g_table) / sizeof(g_table[0])) : 0; }
const KernelInfo *kernel_info(int dtype, int id) { return (id >= 0 && id < kernel_count(dtype)) ? &g_table[id] : nullptr; }
hipError_t launch_reduce(int, const void *, void *, int, int, int64_t, int, uint32_t, uint32_t, int, hipStream_t, int) { ++g_reduces; return hipSuccess; }
hipError_t launch_im2row_matrix(int, const void *, void *, int64_t, int64_t, const Im2row &, hipStream_t) { ++g_matrices; return hipSuccess; }
hipError_t launch_scale(int, void *, int, int, int64_t, uint32_t, int, hipStream_t, int) { ++g_scales; return hipSuccess; }
}
extern "C" const char *hipGetErrorString(hipError_t) { return "hip error (stand-in)"; }
extern "C" hipError_t hipGetDevice(int *) { return hipErrorNoDevice; }      // the model then plans for the whole chip
extern "C" hipError_t hipDeviceGetAttribute(int *, hipDeviceAttribute_t, int) { return hipErrorNoDevice; }

static int g_failed = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++g_failed; } } while (0)

int main()
{
    float *const P = (float *)0x100000;            // a 16-byte aligned fake device address
    void *const WS = (void *)0x4000000;
    // ---- argument checks, in the order of the prototype
    EXPECT(gemm_f32(7, 8, 8, 8, 1.f, P, 8, P, 8, 0.f, P, 8, nullptr, 0, nullptr) == -1);
    EXPECT(gemm_f32(0, -1, 8, 8, 1.f, P, 8, P, 8, 0.f, P, 8, nullptr, 0, nullptr) == -2);
    EXPECT(gemm_f32(0, (int64_t)INT_MAX + 1, 8, 8, 1.f, P, (int64_t)INT_MAX + 1, P, 8, 0.f, P, (int64_t)INT_MAX + 1, nullptr, 0, nullptr) == -2);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, P, 7, P, 8, 0.f, P, 8, nullptr, 0, nullptr) == -7);
    EXPECT(gemm_f32(1, 8, 9, 10, 1.f, P, 9, P, 9, 0.f, P, 9, nullptr, 0, nullptr) == -7);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, P, 8, P, 7, 0.f, P, 8, nullptr, 0, nullptr) == -9);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, P, 8, P, 8, 0.f, P, 7, nullptr, 0, nullptr) == -12);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, P, 8, P, 8, 0.f, P, 8, (char *)WS + 4, 64, nullptr) == -13);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, nullptr, 8, P, 8, 0.f, P, 8, nullptr, 0, nullptr) == -6);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, P, 8, nullptr, 8, 0.f, P, 8, nullptr, 0, nullptr) == -8);
    EXPECT(gemm_f32(0, 8, 8, 8, 1.f, P, 8, P, 8, 0.f, nullptr, 8, nullptr, 0, nullptr) == -11);
    EXPECT(g_launches == 0 && g_scales == 0);
    // ---- quick returns
    EXPECT(gemm_f32(0, 0, 8, 8, 1.f, nullptr, 1, nullptr, 8, 0.f, nullptr, 1, nullptr, 0, nullptr) == 0 && g_launches == 0);
    EXPECT(gemm_f32(0, 8, 8, 0, 1.f, nullptr, 8, nullptr, 1, 1.f, P, 8, nullptr, 0, nullptr) == 0 && g_scales == 0);
    EXPECT(gemm_f32(0, 8, 8, 0, 1.f, nullptr, 8, nullptr, 1, 2.f, P, 8, nullptr, 0, nullptr) == 0 && g_scales == 1);
    EXPECT(gemm_i8(0, 8, 8, 8, 0, nullptr, 8, nullptr, 8, 0, (int32_t *)P, 8, nullptr, 0, nullptr) == 0 && g_scales == 2);
    // ---- launches: canonical form, row-major swap, split clamped to the workspace
    EXPECT(gemm_f32(0, 300, 200, 150, 1.5f, P, 300, P + 4, 150, 0.5f, P + 8, 300, nullptr, 0, nullptr) == 0 && g_launches == 1);
    EXPECT(g_last.M == 300 && g_last.N == 200 && g_last.K == 150 && g_last.split == 1 && g_last.use_beta == 1);
    EXPECT(gemm_f16(1, 300, 200, 150, 1.f, (const uint16_t *)P, 150, (const uint16_t *)P, 200, 0.f, P, 200, nullptr, 0, nullptr) == 0);
    EXPECT(g_last.M == 200 && g_last.N == 300 && g_last.lda == 200 && g_last.ldb == 150 && g_last.use_beta == 0);
    const size_t need = gemm_workspace_bytes(MI_GEMM_F32, 49, 512, 4608);
    EXPECT(need >= (size_t)2 * 49 * 512 * 4);
    EXPECT(gemm_f32(0, 49, 512, 4608, 1.f, P, 49, P, 4608, 0.f, P, 49, WS, need, nullptr) == 0);
    EXPECT(g_last.split > 1 && g_reduces == 1 && (size_t)g_last.split * 49 * 512 * 4 <= need);
    EXPECT(gemm_f32(0, 49, 512, 4608, 1.f, P, 49, P, 4608, 0.f, P, 49, WS, (size_t)49 * 512 * 4 * 2 + 100, nullptr) == 0 && g_last.split <= 2);
    EXPECT(gemm_f32(0, 49, 512, 4608, 1.f, P, 49, P, 4608, 0.f, P, 49, nullptr, 0, nullptr) == 0 && g_last.split == 1);
    // forced configuration and split, also far beyond what K has steps for
    EXPECT(gemm_force_kernel(MI_GEMM_F32, 5, 1000) == 0);
    EXPECT(gemm_f32(0, 64, 64, 100, 1.f, P, 64, P, 100, 0.f, P, 64, WS, (size_t)1 << 30, nullptr) == 0 && gemm_last_kernel_id() == 5);
    EXPECT(g_last.split >= 1 && g_last.split <= 7 && g_last.ktiles_per_split * g_last.split >= g_last.ktiles);
    EXPECT(gemm_force_kernel(MI_GEMM_F32, -1, 0) == 0 && gemm_force_kernel(MI_GEMM_F32, 6, 0) == -1 && gemm_force_kernel(9, 0, 0) == -1);
    // ---- the largest legal sizes: no arithmetic may overflow on the way to a decision
    int kid = -1, split = 0;
    for (int dtype = 0; dtype < 4; ++dtype) {
        EXPECT(gemm_select(dtype, 0, INT_MAX, INT_MAX, INT_MAX, (size_t)-1, &kid, &split) == 0 && kid >= 0 && split >= 1);
        EXPECT(gemm_select(dtype, 1, 1, INT_MAX, INT_MAX, 0, &kid, &split) == 0 && split == 1);
        EXPECT(gemm_select(dtype, 0, INT_MAX, 1, 1, 1 << 20, &kid, &split) == 0);
        gemm_workspace_bytes(dtype, INT_MAX, INT_MAX, INT_MAX);
        gemm_workspace_bytes(dtype, 1, 1, INT_MAX);
        EXPECT(gemm_workspace_bytes(dtype, (int64_t)INT_MAX + 1, 1, 1) == 0 && gemm_workspace_bytes(dtype, 0, 5, 5) == 0);
        EXPECT(gemm_predict_us(dtype, 0, INT_MAX, INT_MAX, INT_MAX, 1) > 0.0 && gemm_predict_us(dtype, 99, 8, 8, 8, 1) < 0.0);
        for (int i = 0; i < 300; ++i)          // more distinct problems than the per-thread tables hold
            EXPECT(gemm_select(dtype, i & 1, 17 + 13 * i, 5 + 7 * i, 64 + 31 * i, (size_t)i << 16, &kid, &split) == 0);
    }
    EXPECT(gemm_select(4, 0, 8, 8, 8, 0, &kid, &split) == -1 && gemm_select(0, 2, 8, 8, 8, 0, &kid, &split) == -2);
    EXPECT(gemm_select(0, 0, 0, 8, 8, 0, &kid, &split) == -3 && gemm_select(0, 0, 8, 8, (int64_t)INT_MAX + 1, 0, nullptr, nullptr) == -5);
    // leading dimensions that some configurations cannot address: the choice skips them
    EXPECT(gemm_f32(0, 300, 40, 24, 1.f, P, ((int64_t)1 << 26) + 8, P, 24, 0.f, P, 300, nullptr, 0, nullptr) == 0);
    EXPECT(kernel_info(0, gemm_last_kernel_id())->max_lda == 0);
    // ---- gemm_ex: its own argument positions
    const float one = 1.f, zero = 0.f;
    EXPECT(gemm_ex(9, 0, 0, 0, 8, 8, 8, &one, P, 8, P, 8, &zero, P, 8, nullptr, 0, nullptr) == -1);
    EXPECT(gemm_ex(0, 5, 0, 0, 8, 8, 8, &one, P, 8, P, 8, &zero, P, 8, nullptr, 0, nullptr) == -2);
    EXPECT(gemm_ex(0, 0, 2, 0, 8, 8, 8, &one, P, 8, P, 8, &zero, P, 8, nullptr, 0, nullptr) == -3);
    EXPECT(gemm_ex(0, 0, 0, 1, 8, 9, 10, &one, P, 8, P, 8, &zero, P, 8, nullptr, 0, nullptr) == -12);   // stored B is N x K: ldb >= 9
    EXPECT(gemm_ex(0, 0, 1, 1, 8, 9, 10, &one, P, 10, P, 9, &zero, P, 8, nullptr, 0, nullptr) == 0 && g_last.a_kc == 1 && g_last.b_nc == 1);
    EXPECT(gemm_ex(0, 0, 0, 0, 8, 8, 8, nullptr, P, 8, P, 8, &zero, P, 8, nullptr, 0, nullptr) == -8);
    EXPECT(strlen(gemm_ex_status_string(-12)) > 0 && strlen(gemm_status_string(-7)) > 0 && strlen(gemm_status_string(3)) > 0);
    // ---- convolution geometry at its limits
    int64_t Hout, Wout, M, N, K;
    EXPECT(conv2d_im2row_shape(1, 224, 224, 3, 64, 7, 7, 2, 2, 3, 3, &Hout, &Wout, &M, &N, &K) == 0 && M == 12544 && N == 64 && K == 147);
    EXPECT(conv2d_im2row_shape(1, 1 << 20, 1 << 20, 1, 1, 1, 1, 1, 1, 0, 0, &Hout, &Wout, &M, &N, &K) == -1);   // too many pixels
    EXPECT(conv2d_im2row_shape(1, 1 << 10, 1 << 10, 1 << 20, 1, 1 << 10, 1 << 10, 1, 1, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr) == -4);   // kh*kw*Cin = 2^40
    EXPECT(conv2d_im2row_shape(INT_MAX, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, nullptr, nullptr, &M, nullptr, nullptr) == 0 && M == INT_MAX);
    EXPECT(conv2d_im2row_shape(1, 4, 4, 1, 1, 9, 1, 1, 1, 2, 0, nullptr, nullptr, nullptr, nullptr, nullptr) == -10);
    EXPECT(conv2d_im2row_workspace_bytes(1, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1) >= (size_t)3136 * 576 * 4);
    g_launches = g_matrices = 0;
    EXPECT(conv2d_im2row_f32(1, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1, 1.f, P, P, 0.f, P, nullptr, 0, nullptr) == 0 && g_launches == 1 && g_matrices == 0);
    EXPECT(conv2d_im2row_last_path() == 1);
    // huge padding: offsets of padded positions would not fit the kernels' 32-bit arithmetic, so the matrix path is required
    EXPECT(conv2d_im2row_f32(1, 4, 4, 1 << 19, 8, 3, 3, 1, 1, 1 << 11, 1 << 11, 1.f, P, P, 0.f, P, nullptr, 0, nullptr) == -18);
    EXPECT(conv2d_im2row_force_path(3) == -1 && conv2d_im2row_force_path(0) == 0);
    EXPECT(im2row_f32(1, 8, 8, 4, 3, 3, 1, 1, 1, 1, P, P, nullptr) == 0 && g_matrices == 1);
    // the convolution for the other data types: its own argument positions; in place when Cin is a multiple of the
    // K step of a configuration (the stand-ins' 16 and 32), through the matrix otherwise
    const int32_t ione = 1, izero = 0;
    g_launches = g_matrices = 0;
    EXPECT(conv2d_im2row_ex(7, 1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1, &one, P, P, &zero, P, nullptr, 0, nullptr) == -1);
    EXPECT(conv2d_im2row_ex(MI_GEMM_F16, 1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1, nullptr, P, P, &zero, P, nullptr, 0, nullptr) == -13);
    EXPECT(conv2d_im2row_ex(MI_GEMM_F16, 1, 14, 14, 32, 40, 0, 3, 2, 2, 1, 1, &one, P, P, &zero, P, nullptr, 0, nullptr) == -7);   // kh is the 7th
    EXPECT(conv2d_im2row_ex(MI_GEMM_F16, 1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1, &one, nullptr, P, &zero, P, nullptr, 0, nullptr) == -14);
    EXPECT(conv2d_im2row_ex(MI_GEMM_F16, 1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1, &one, P, P, &zero, P, nullptr, 0, nullptr) == 0 && g_launches == 1 && g_matrices == 0);
    EXPECT(conv2d_im2row_ex(MI_GEMM_I8, 1, 14, 14, 32, 40, 3, 3, 2, 2, 1, 1, &ione, P, P, &izero, P, nullptr, 0, nullptr) == 0 && g_launches == 2);
    EXPECT(conv2d_im2row_ex(MI_GEMM_I8, 1, 14, 14, 32, 3, 3, 3, 2, 2, 1, 1, &ione, P, P, &izero, P, nullptr, 0, nullptr) == -19);   // Cout < 4: needs the matrix
    const size_t cws = conv2d_im2row_ex_workspace_bytes(MI_GEMM_I8, 1, 14, 14, 32, 3, 3, 3, 2, 2, 1, 1);
    EXPECT(cws >= 49 * 288 && cws < 49 * 288 * 4);
    EXPECT(conv2d_im2row_ex(MI_GEMM_I8, 1, 14, 14, 32, 3, 3, 3, 2, 2, 1, 1, &ione, P, P, &izero, P, WS, cws, nullptr) == 0 && g_matrices == 1);
    EXPECT(conv2d_im2row_ex_workspace_bytes(9, 1, 14, 14, 32, 3, 3, 3, 2, 2, 1, 1) == 0);
    EXPECT(strlen(conv2d_im2row_ex_status_string(-19)) > 0 && strlen(conv2d_im2row_ex_status_string(-8)) > 0);
    EXPECT(im2row_f32(1, 8, 8, 4, 3, 3, 0, 1, 1, 1, P, P, nullptr) == -7);
    printf("%s (%d launches recorded)\n", g_failed ? "FAILED" : "ok", g_launches);
    return g_failed ? 1 : 0;
}
