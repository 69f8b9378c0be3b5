// C-ABI entry points: argument checks, quick returns, layout canonicalisation,
// tile selection and launch.  Host code only; the kernels are instantiated in the
// gemm_table*.hip files.  Declarations and the full contract are in include/mi_gemm.h.
#include "../../include/mi_gemm.h"
#include "gemm_table.h"

#include <hip/hip_runtime_api.h>
#include <limits.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

using namespace mig;

namespace {

constexpr int kChipCu = 256;     // compute units of a whole MI355X: the part the rate constants below were measured on
constexpr int MAX_SPLIT = 32;    // upper limit of the K split

struct Forced { int id = -1; int split = 0; };
constexpr int NUM_DTYPES = 4;
// the override of gemm_force_kernel belongs to the calling thread, like the last_* reports: a test or a
// tuning run on one thread never changes what another thread's calls select
thread_local Forced t_forced[NUM_DTYPES];
thread_local int t_last_id = -1;
thread_local int t_last_split = 0;

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// What the selector settles on for one canonical problem.
struct Choice { int id; int split; int ktiles_per_split; };

// ---------------------------------------------------------------------------
// Tile and split selection by a small analytical model: the analogue of the
// paper's choice of the micro-kernel size that matches the problem (Secs. "Edge
// Cases", "Squared Matrices") and of the blocking-parameter model it cites for
// the packed buffers.  For every candidate (tile configuration, K split) the
// predicted time is
//     launch + fixed cost + main + reduce(split)
// Kernels that stage tiles in LDS:
//     main    = max(sum over rounds of steps * step_time(r), staged_bytes / staging_bandwidth)
//     rounds  = whole rounds that fill every slot (CUs * workgroups per CU), then one partial round with
//               r = fewer workgroups per CU, which run faster
//     steps   = ceil(K steps / split)
//     step_time(r) = max(r co-resident workgroups * MFMA time of one K step, latency of a step);
//                 the latency is 2.2 times longer when a dimension is smaller than the tile, because
//                 such a tile cannot be moved inside the matrix and is staged through registers
// Register-direct kernels (every wave streams its own operands):
//     main    = max(rounds * steps per wave * step time of a lone wave,
//                   MFMA time of all wave tiles, bytes all waves load / cache fill rate of the busy CUs)
//     rounds  = waves / (SIMDs * waves per SIMD), at least 1
// reduce = second launch + split partial tiles written and read back.
// The constants are measured on MI355X with HIP-graph replays: sustained MFMA rate per data type
// (solo mode on random data), 17 TB/s from L2 into LDS for GEMM-like tile streams, 4 TB/s for the
// partial-tile round trip, 2.5 us per launch, 3.0 us for the second launch.
// ---------------------------------------------------------------------------
constexpr double kSustainedTflops[NUM_DTYPES] = {157.3 * 0.97, 2516.6 * 0.58, 5033.2 * 0.61, 2516.6 * 0.58};
constexpr double kStagingBytesPerUs = 17.0e6;
constexpr double kStepFloorUs = 0.75;
constexpr double kGuardedStepFactor = 2.2;
constexpr double kReduceBytesPerUs = 4.0e6;
constexpr double kLaunchUs = 2.5, kReduceLaunchUs = 3.0;
constexpr int kMaxAutoSplit = 16;

// Compute units of the device the model plans for: read once per process from the device that is current at the
// first call (a partition of the chip has fewer than the whole part); 256 when no device can be asked.
int num_cu()
{
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            return v;
        return kChipCu;
    }();
    return n;
}

// How much longer a K step of a staged fp32 kernel takes when B has N contiguous (its tile goes through
// the register transposes and, with bank conflicts, into LDS), alone or together with a K-contiguous A:
// measured at 1024^3 ... 4096^3, the smaller the tile the more.  1 for every other kernel, data type and
// orientation (the 16- and 8-bit types have direct kernels for these orientations).
// How operands are aligned, as far as the kernels care: ALIGN_FULL = the rows of both canonical operands are
// 16-byte aligned (vector loads, global -> LDS transfers); ALIGN_WORDS = the K-contiguous operand's rows are, and
// the rows of the M-contiguous one are 4-byte aligned (what the 16- and 8-bit register-direct kernels load: 16-byte
// fragments of the one, 32-bit words of the other); ALIGN_NONE = neither.
enum { ALIGN_NONE = 0, ALIGN_WORDS = 1, ALIGN_FULL = 2 };

double staged_orientation_factor(int dtype, const KernelInfo *ki, bool a_kc, bool b_nc, int align = ALIGN_FULL)
{
    if (dtype != MI_GEMM_F32 || !(a_kc || b_nc)) return 1.0;
    // the direct fp32 kernels take transposed operands at their normal speed when rows are 16-byte aligned;
    // otherwise every tile of theirs goes through guarded loads and registers (measured 2.2 ... 3.2 times
    // slower at 2050^3 and 1026^3, against which the staged kernels' factors below compete)
    if (!ki->transposed_ok) return align == ALIGN_FULL ? 1.0 : 2.6;
    if (!b_nc) return 1.0;
    const int area = ki->BM * ki->BN;
    if (area <= 64 * 64) return a_kc ? 1.85 : 2.6;
    if (area <= 128 * 128) return a_kc ? 1.45 : 1.9;
    return a_kc ? 1.15 : 1.45;
}

double predict_us(int dtype, const KernelInfo *ki, int64_t M, int64_t N, int64_t K, int split, int align = ALIGN_FULL,
                  double step_factor = 1.0)
{
    static const int es[NUM_DTYPES] = {4, 2, 1, 2};
    const double tiles = (double)(ceil_div(M, ki->BM) * ceil_div(N, ki->BN));
    const double ktiles = (double)ceil_div(K, ki->BK);
    const double steps = (double)ceil_div((int64_t)ktiles, split);
    const double eff = (ki->eff_pct > 0 ? ki->eff_pct : 100) / 100.0;
    const int NUM_CU = num_cu();
    const double part = (double)NUM_CU / kChipCu;             // share of the whole chip's MFMA and fill rates
    double main_us;
    if (ki->waves_k > 0) {
        const double wave_tiles = tiles * (ki->BM / ki->wave_m) * (ki->BN / ki->wave_n);
        const double waves = wave_tiles * ki->waves_k * split;
        double rounds = waves / (4.0 * NUM_CU * ki->waves_per_simd);
        if (rounds < 1.0) rounds = 1.0;
        const double steps_per_wave = (double)ceil_div((int64_t)steps, ki->waves_k);
        const double chain = rounds * steps_per_wave * ki->step_floor_ns * 1e-3;
        const double mfma = 2.0 * wave_tiles * ki->wave_m * ki->wave_n * ktiles * ki->BK /
                            (kSustainedTflops[dtype] * 1e6 * eff * part);
        // the fill rate is a sum over CUs: with fewer workgroups than CUs less of it is there (measured:
        // about the square root of the busy share, since a CU alone in its part of the chip fills faster)
        const double busy = (tiles * split < NUM_CU ? sqrt(tiles * split / NUM_CU) : 1.0) * part;
        const double fill = wave_tiles * ktiles * (double)(ki->wave_m + ki->wave_n) * ki->BK * es[dtype] /
                            (ki->fill_bytes_per_us * busy);
        main_us = chain > mfma ? chain : mfma;
        if (fill > main_us) main_us = fill;
        // operands whose rows are not 16-byte aligned: the 16- and 8-bit kernels issue their 4- and 16-byte loads
        // at element alignment and the memory system splits them.  The step constants were fitted over aligned
        // and ragged shapes alike, so this is the part of the slowdown they do not carry (tiny ragged shapes
        // measure 2 ... 3 times the K loop of their aligned twins, large ones 1.1 ... 1.9 times)
        if (align == ALIGN_NONE && ki->unaligned_pct > 0) main_us *= 100.0 / ki->unaligned_pct;
    } else {
        const int occ = ki->min_blocks_per_cu > 0 ? ki->min_blocks_per_cu : 1;
        const double wgs = tiles * split;
        const double mfma_step = step_factor * 2.0 * ki->BM * ki->BN * ki->BK / (kSustainedTflops[dtype] * 1e6 / kChipCu) / eff;
        double floor_us = step_factor * (ki->step_floor_ns > 0 ? ki->step_floor_ns * 1e-3 : kStepFloorUs);
        if (M < ki->BM || N < ki->BN) floor_us *= kGuardedStepFactor;
        // time of one K step on a CU that runs `resident` workgroups side by side
        auto step_us = [&](double resident) {
            double step = resident * mfma_step;
            if (step < floor_us) step = floor_us;
            if (align != ALIGN_FULL && ki->unaligned_pct > 0) step *= 100.0 / ki->unaligned_pct;
            return step;
        };
        // whole rounds with every slot of every CU taken, then the rest: fewer workgroups per CU, each of
        // which runs faster than in a full round (alone on its CU: as fast as its latency allows)
        const double slots = (double)NUM_CU * occ;
        const double full = (double)(int64_t)(wgs / slots);
        const double rest = wgs - full * slots;
        main_us = full * steps * step_us(occ);
        if (rest > 0.0) {
            // the CUs that got the most workgroups finish last
            main_us += steps * step_us((double)ceil_div((int64_t)rest, NUM_CU));
        }
        const double staged = tiles * ktiles * (double)(ki->BM + ki->BN) * ki->BK * es[dtype];
        if (main_us < staged / (kStagingBytesPerUs * part)) main_us = staged / (kStagingBytesPerUs * part);
    }
    double reduce_us = 0.0;
    if (split > 1) reduce_us = kReduceLaunchUs + (double)split * (double)M * (double)N * 8.0 / kReduceBytesPerUs;
    return kLaunchUs + ki->setup_ns * 1e-3 + main_us + reduce_us;
}

// Best split for one configuration (used directly when the configuration is forced).
int auto_split(int dtype, const KernelInfo *ki, int64_t M, int64_t N, int64_t K, int64_t max_split, int align = ALIGN_FULL,
               double step_factor = 1.0)
{
    const int64_t ktiles = ceil_div(K, ki->BK);
    int best = 1;
    double best_us = predict_us(dtype, ki, M, N, K, 1, align, step_factor);
    // the fastest split, if it beats the unsplit launch clearly (the second launch and the workspace traffic
    // must pay for themselves)
    const double unsplit = best_us;
    for (int s = 2; s <= kMaxAutoSplit && s <= max_split && 2 * s <= ktiles; ++s) {
        const double t = predict_us(dtype, ki, M, N, K, s, align, step_factor);
        if (t < best_us && t < unsplit * 0.92) { best_us = t; best = s; }
    }
    return best;
}

// Leading dimensions (canonical problem) a configuration can address.
bool can_address(const KernelInfo *ki, int64_t lda, int64_t ldb)
{
    return (ki->max_lda == 0 || lda <= ki->max_lda) && (ki->max_ldb == 0 || ldb <= ki->max_ldb);
}

// Best (configuration, split) over the configurations open to automatic selection (prio > 0).
int auto_kernel(int dtype, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t max_split_bytes_per_mn,
                int align, bool a_kc, bool b_nc)
{
    const int n = kernel_count(dtype);
    int best = -1;
    double best_us = 0.0;
    // does a configuration open to selection take these operand orientations at its normal speed?
    auto direct = [&](const KernelInfo *ki) { return (!a_kc || ki->a_kc_ok) && (!b_nc || ki->b_nc_ok); };
    bool any_direct = false;
    for (int id = 0; id < n; ++id) any_direct = any_direct || (kernel_info(dtype, id)->prio > 0 && direct(kernel_info(dtype, id)));
    for (int id = 0; id < n; ++id) {
        const KernelInfo *ki = kernel_info(dtype, id);
        // canonical operands: the configurations open to selection.  Transposed operands: where the data type
        // has direct kernels for that orientation, those and the staged ones open to selection (the constants
        // of the others are not calibrated against the direct kernels); else every staged configuration
        const bool takes = !(a_kc || b_nc) ? ki->prio > 0
                           : any_direct    ? ki->prio > 0 && (direct(ki) || ki->transposed_ok)
                                           : ki->transposed_ok != 0;
        if (!takes) continue;
        if (!can_address(ki, lda, ldb)) continue;
        const double f = staged_orientation_factor(dtype, ki, a_kc, b_nc, align);
        const int s = auto_split(dtype, ki, M, N, K, max_split_bytes_per_mn, align, f);
        double t = predict_us(dtype, ki, M, N, K, s, align, f);
        if (s > 1) t *= 1.03;           // a tie between a split and an unsplit configuration goes to the unsplit one
        if (best < 0 || t < best_us) { best = id; best_us = t; }
    }
    return best < 0 ? 0 : best;
}

Choice choose_uncached(int dtype, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t fit, int align,
                       bool a_kc, bool b_nc, const Forced f)
{
    Choice c;
    const bool forced = f.id >= 0 && f.id < kernel_count(dtype) && can_address(kernel_info(dtype, f.id), lda, ldb) &&
                        (!(a_kc || b_nc) || kernel_info(dtype, f.id)->transposed_ok ||
                         ((!a_kc || kernel_info(dtype, f.id)->a_kc_ok) && (!b_nc || kernel_info(dtype, f.id)->b_nc_ok)));
    c.id = forced ? f.id : auto_kernel(dtype, M, N, K, lda, ldb, fit, align, a_kc, b_nc);
    const KernelInfo *ki = kernel_info(dtype, c.id);
    const int64_t ktiles = ceil_div(K, ki->BK);
    int64_t s = f.split >= 1 ? f.split : auto_split(dtype, ki, M, N, K, fit, align, staged_orientation_factor(dtype, ki, a_kc, b_nc, align));
    if (s > ktiles) s = ktiles;
    if (s > fit) s = fit;
    if (s < 1) s = 1;
    c.ktiles_per_split = (int)ceil_div(ktiles, s);
    c.split = (int)ceil_div(ktiles, c.ktiles_per_split);   // every slice gets at least one step
    return c;
}

// The model is evaluated once per distinct problem and thread: an inference loop repeats a handful of
// shapes, and a GEMM of a few microseconds cannot afford ten evaluations of a timing model per call.
// Everything the choice depends on is in the key; a leading dimension beyond what some configuration
// can address (rare: rows 2^28 bytes apart) bypasses the table.
struct ChoiceKey {
    int64_t M, N, K;
    int32_t forced_split;
    uint32_t bits;      // dtype, alignment class, a_kc, b_nc, fit, forced id + 1
    bool operator==(const ChoiceKey &o) const
    {
        return M == o.M && N == o.N && K == o.K && forced_split == o.forced_split && bits == o.bits;
    }
};
struct ChoiceSlot { ChoiceKey key; Choice choice; bool used; };
constexpr int kChoiceSlots = 256;       // direct-mapped; a collision just re-evaluates
thread_local ChoiceSlot t_choice[kChoiceSlots];

// Smallest leading dimension that some configuration of the data type cannot address (INT64_MAX: none).
int64_t smallest_ld_limit(int dtype)
{
    int64_t m = INT64_MAX;
    for (int id = 0; id < kernel_count(dtype); ++id) {
        const KernelInfo *ki = kernel_info(dtype, id);
        if (ki->max_lda > 0 && ki->max_lda < m) m = ki->max_lda;
        if (ki->max_ldb > 0 && ki->max_ldb < m) m = ki->max_ldb;
    }
    return m;
}

int64_t addressing_limit(int dtype)
{
    static const int64_t limit[NUM_DTYPES] = {smallest_ld_limit(0), smallest_ld_limit(1), smallest_ld_limit(2),
                                              smallest_ld_limit(3)};
    return limit[dtype];
}

Choice choose(int dtype, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, size_t ws_bytes, bool have_ws,
              int align, bool a_kc = false, bool b_nc = false)
{
    const Forced f = t_forced[dtype];
    // how many partial tiles the workspace can hold
    const unsigned __int128 per = (unsigned __int128)M * (unsigned __int128)N * 4u;
    int64_t fit = (have_ws && per > 0) ? (int64_t)((unsigned __int128)ws_bytes / per) : 0;
    if (fit > MAX_SPLIT) fit = MAX_SPLIT;
    if (fit < 1) fit = 1;
    const int64_t limit = addressing_limit(dtype);
    if (lda > limit || ldb > limit || f.id >= 254) return choose_uncached(dtype, M, N, K, lda, ldb, fit, align, a_kc, b_nc, f);
    ChoiceKey key;
    key.M = M; key.N = N; key.K = K;
    key.forced_split = f.split;
    key.bits = (uint32_t)dtype | ((uint32_t)align << 2) | (a_kc ? 16u : 0u) | (b_nc ? 32u : 0u) | ((uint32_t)fit << 6) |
               ((uint32_t)(f.id + 1) << 12);
    uint64_t h = (uint64_t)M * 0x9E3779B97F4A7C15ull ^ (uint64_t)N * 0xC2B2AE3D27D4EB4Full ^ (uint64_t)K * 0x165667B19E3779F9ull ^
                 ((uint64_t)key.bits << 32 | (uint32_t)key.forced_split) * 0xD6E8FEB86659FD93ull;
    ChoiceSlot &slot = t_choice[(h >> 40) % kChoiceSlots];
    if (slot.used && slot.key == key) return slot.choice;
    slot.choice = choose_uncached(dtype, M, N, K, lda, ldb, fit, align, a_kc, b_nc, f);
    slot.key = key;
    slot.used = true;
    return slot.choice;
}

// Alignment class of a canonical problem: rows of A (M contiguous unless a_kc) and of B (K contiguous unless b_nc)
int alignment_class(bool vec_a, bool vec_b, bool a_words, bool a_kc, bool b_nc)
{
    if (vec_a && vec_b) return ALIGN_FULL;
    return (!a_kc && !b_nc && vec_b && a_words) ? ALIGN_WORDS : ALIGN_NONE;
}

bool aligned16(const void *p, int64_t ld, int es)
{
    // 16-byte vectors / direct LDS transfers; lane offsets inside a transfer are 32-bit
    return ((uintptr_t)p % 16 == 0) && ((ld * es) % 16 == 0) && (ld * es < ((int64_t)1 << 27));
}

// Status codes are those of the gemm_f32 / f16 / bf16 / i8 argument list: -k for its k-th argument.
// transa / transb: op(A) = A^T / op(B) = B^T (gemm_ex only; checked by the caller).
int run(int dtype, int es, int layout, int64_t M, int64_t N, int64_t K, uint32_t alpha_bits, bool alpha_zero,
        const void *A, int64_t lda, const void *B, int64_t ldb, uint32_t beta_bits, bool beta_zero, bool beta_one,
        void *C, int64_t ldc, void *ws, size_t ws_bytes, void *stream_, bool transa = false, bool transb = false,
        int c_type = C_WIDE)
{
    t_last_id = -1;
    t_last_split = 0;
    if (layout != MI_GEMM_COL_MAJOR && layout != MI_GEMM_ROW_MAJOR) return -1;
    if (M < 0 || M > INT_MAX) return -2;
    if (N < 0 || N > INT_MAX) return -3;
    if (K < 0 || K > INT_MAX) return -4;
    const bool col = (layout == MI_GEMM_COL_MAJOR);
    const int64_t one = 1;
    // the stored A is M x K, or K x M when transposed; the stored B is K x N, or N x K; a leading
    // dimension spans the contiguous extent of the stored matrix
    const int64_t a_span = (col != transa) ? M : K, b_span = (col != transb) ? K : N;
    if (lda < (a_span > one ? a_span : one)) return -7;
    if (ldb < (b_span > one ? b_span : one)) return -9;
    if (ldc < (col ? (M > one ? M : one) : (N > one ? N : one))) return -12;
    if (ws != nullptr && (uintptr_t)ws % 16 != 0) return -13;
    if (M == 0 || N == 0) return 0;
    if (C == nullptr) return -11;
    const bool no_product = (K == 0) || alpha_zero;
    if (!no_product && A == nullptr) return -6;
    if (!no_product && B == nullptr) return -8;

    hipStream_t stream = (hipStream_t)stream_;

    // canonical form: C' column-major M' x N'.  A row-major problem is the
    // column-major problem C^T = B^T A^T on the same buffers.
    // Canonical A has M' contiguous unless a_kc, canonical B has K contiguous unless b_nc.
    int64_t Mc = M, Nc = N;
    const void *Ac = A, *Bc = B;
    int64_t ldac = lda, ldbc = ldb;
    bool a_kc = transa, b_nc = transb;
    if (!col) {
        Mc = N; Nc = M;
        Ac = B; ldac = ldb;
        Bc = A; ldbc = lda;
        a_kc = transb; b_nc = transa;
    }

    if (no_product) {
        if (beta_one) return 0;
        hipError_t e = launch_scale(dtype, C, (int)Mc, (int)Nc, ldc, beta_bits, beta_zero ? 0 : 1, stream, c_type);
        return e == hipSuccess ? 0 : (int)e;
    }

    const bool vec_a = aligned16(Ac, ldac, es), vec_b = aligned16(Bc, ldbc, es);
    const bool a_words = (uintptr_t)Ac % 4 == 0 && (ldac * es) % 4 == 0;
    const Choice ch = choose(dtype, Mc, Nc, K, ldac, ldbc, ws_bytes, ws != nullptr,
                             alignment_class(vec_a, vec_b, a_words, a_kc, b_nc), a_kc, b_nc);
    const KernelInfo *ki = kernel_info(dtype, ch.id);

    Params p;
    memset(&p, 0, sizeof(p));
    p.A = Ac; p.B = Bc; p.C = C; p.ws = ws;
    p.lda = ldac; p.ldb = ldbc; p.ldc = ldc;
    p.M = (int)Mc; p.N = (int)Nc; p.K = (int)K;
    p.tiles_m = (int)ceil_div(Mc, ki->BM);
    p.tiles_n = (int)ceil_div(Nc, ki->BN);
    if ((int64_t)p.tiles_m * p.tiles_n > INT_MAX) return -2;
    p.ktiles = (int)ceil_div(K, ki->BK);
    p.ktiles_per_split = ch.ktiles_per_split;
    p.split = ch.split;
    p.alpha_bits = alpha_bits;
    p.beta_bits = beta_bits;
    p.use_beta = beta_zero ? 0 : 1;
    p.vecA = vec_a ? 1 : 0;
    p.vecB = vec_b ? 1 : 0;
    p.a_kc = a_kc ? 1 : 0;
    p.b_nc = b_nc ? 1 : 0;
    p.group_m = 8;
    p.xcd_remap = ((int64_t)p.tiles_m * p.tiles_n >= 64) ? 1 : 0;
    if (const char *e = getenv("MIG_GROUP_M")) p.group_m = atoi(e);   // EXPERIMENT
    if (const char *e = getenv("MIG_XCD")) p.xcd_remap = atoi(e);     // EXPERIMENT
    p.c_type = c_type;

    hipError_t e = ki->launch(p, stream);
    if (e != hipSuccess) return (int)e;
    if (p.split > 1) {
        e = launch_reduce(dtype, ws, C, p.M, p.N, ldc, p.split, alpha_bits, beta_bits, p.use_beta, stream, c_type);
        if (e != hipSuccess) return (int)e;
    }
    t_last_id = ch.id;
    t_last_split = ch.split;
    return 0;
}

uint32_t bits_of(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }

// ---------------------------------------------------------------------------
// Convolution through the im2row GEMM.  The problem is the row-major GEMM
//   output[M x N] = alpha * im2row(image)[M x K] * filter[K x N] + beta * output,
// M = batch*Hout*Wout, N = Cout, K = kh*kw*Cin; in canonical (column-major) form the filter is
// the M-contiguous operand and the im2row matrix the K-contiguous one.
// ---------------------------------------------------------------------------
struct ConvGeometry {
    int64_t M, N, K;
    Im2row g;
};
thread_local int t_conv_path = 0;
thread_local int t_conv_forced_path = 0;     // per thread, like the GEMM override
// forming the matrix, measured: about 5 us plus its bytes at 1.35 TB/s (a launch, one element per thread)
constexpr double kIm2rowFixedUs = 5.0, kIm2rowBytesPerUs = 1.35e6;
constexpr double kIm2rowLdsFactor = 1.32, kIm2rowRegFactor = 1.08;

// 0, or -k for the k-th argument of conv2d_im2row_f32 (Cout is not checked when it is 0: im2row_f32)
int conv_geometry(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw, int64_t stride_h,
                  int64_t stride_w, int64_t pad_h, int64_t pad_w, bool with_cout, ConvGeometry *out)
{
    const int64_t lim = 1 << 20;       // per extent; products are checked below
    if (batch < 1 || batch > INT_MAX) return -1;
    if (H < 1 || H > lim) return -2;
    if (W < 1 || W > lim) return -3;
    if (Cin < 1 || Cin > lim) return -4;
    if (with_cout && (Cout < 1 || Cout > INT_MAX)) return -5;
    if (kh < 1 || kh > lim) return -6;
    if (kw < 1 || kw > lim) return -7;
    if (stride_h < 1 || stride_h > lim) return -8;
    if (stride_w < 1 || stride_w > lim) return -9;
    if (pad_h < 0 || pad_h > lim || H + 2 * pad_h < kh) return -10;
    if (pad_w < 0 || pad_w > lim || W + 2 * pad_w < kw) return -11;
    const int64_t Hout = (H + 2 * pad_h - kh) / stride_h + 1, Wout = (W + 2 * pad_w - kw) / stride_w + 1;
    const unsigned __int128 M = (unsigned __int128)batch * (unsigned __int128)(Hout * Wout);
    const unsigned __int128 K = (unsigned __int128)(kh * kw) * (unsigned __int128)Cin;
    if (M > (unsigned __int128)INT_MAX) return -1;
    if (K > (unsigned __int128)INT_MAX) return -4;
    out->M = (int64_t)M; out->N = Cout; out->K = (int64_t)K;
    out->g = Im2row{(int)H, (int)W, (int)Cin, (int)kw, (int)stride_h, (int)stride_w, (int)pad_h, (int)pad_w, (int)Hout, (int)Wout};
    return 0;
}

// The fused kernels read the image through 32-bit lane offsets; the element-by-element variant splits
// k into (filter row, element of the run) in single precision, exact below 2^22.
bool conv_fused_ok(int64_t batch, const ConvGeometry &c, int es = 4)
{
    const unsigned __int128 image_bytes = (unsigned __int128)batch * c.g.H * c.g.W * (unsigned __int128)c.g.Cin * (unsigned)es;
    // the kernels also form offsets of padded positions ((W - iw)*Cin, -iw*Cin, rows above and below the
    // image) in 32-bit integers: the padded image of one batch entry must fit them as well
    const unsigned __int128 padded_row = (unsigned __int128)(c.g.W + 2 * (int64_t)c.g.pad_w) * (unsigned __int128)c.g.Cin;
    const unsigned __int128 padded_image = (unsigned __int128)(c.g.H + 2 * (int64_t)c.g.pad_h) * padded_row;
    return image_bytes < ((unsigned __int128)1 << 31) && padded_image < ((unsigned __int128)1 << 29);
}

// How configuration ki can read the im2row matrix in place: a K step inside one filter tap (Cin a multiple
// of its K step; the direct-to-LDS kernels also need a 16-byte aligned image), element by element along
// filter rows (register-direct kernels, K below 2^22), or not at all.
typedef hipError_t (*LaunchFn)(const Params &, hipStream_t);
LaunchFn conv_fused_launcher(const KernelInfo *ki, const ConvGeometry &c, bool image_aligned)
{
    const bool lds_kernel = ki->waves_k == 0;
    if (ki->launch_im2row && c.g.Cin % ki->BK == 0 && (!lds_kernel || image_aligned)) return ki->launch_im2row;
    if (ki->launch_im2row_runs && c.K < ((int64_t)1 << 22)) return ki->launch_im2row_runs;
    return nullptr;
}

// Best fused configuration (canonical problem N x M x K) for a workspace that holds `fit` partial tiles;
// -1 if none.
int conv_fused_kernel(int dtype, const ConvGeometry &c, int64_t fit, bool image_aligned, double *us)
{
    int best = -1;
    double best_us = 0.0;
    const Forced f = t_forced[dtype];
    for (int id = 0; id < kernel_count(dtype); ++id) {
        const KernelInfo *ki = kernel_info(dtype, id);
        if (!conv_fused_launcher(ki, c, image_aligned) || !can_address(ki, c.N, 0)) continue;
        if (f.id >= 0 ? id != f.id : ki->prio <= 0) continue;
        int s = auto_split(dtype, ki, c.N, c.M, c.K, fit);
        // a direct-to-LDS kernel that would need its K split (few tiles, every step latency-bound) loses to
        // the register-direct kernels in every layer measured: it competes unsplit only
        if (ki->waves_k == 0 && f.split < 1) s = 1;
        double t = predict_us(dtype, ki, c.N, c.M, c.K, s);
        // measured against the GEMM on a matrix that exists: the direct-to-LDS kernels pay for the clamped
        // addresses and the zeroing between the wait and the barrier of every K step, the register-direct
        // ones for the masks of their loads
        t = kLaunchUs + (t - kLaunchUs) * (ki->waves_k == 0 ? kIm2rowLdsFactor : kIm2rowRegFactor);
        if (best < 0 || t < best_us) { best = id; best_us = t; }
    }
    if (us) *us = best_us;
    return best;
}

size_t round16(size_t x) { return (x + 15) & ~(size_t)15; }

// The convolution entry points.  Status codes are those of conv2d_im2row_f32's argument list.
int conv_run(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw, int64_t stride_h,
             int64_t stride_w, int64_t pad_h, int64_t pad_w, uint32_t alpha_bits, bool alpha_zero, const void *image,
             const void *filter, uint32_t beta_bits, bool beta_zero, bool beta_one, void *output, void *workspace,
             size_t workspace_bytes, void *stream)
{
    static const int kEs[NUM_DTYPES] = {4, 2, 1, 2};
    const int es = kEs[dtype];
    t_conv_path = 0;
    t_last_id = -1;
    t_last_split = 0;
    ConvGeometry c;
    const int bad = conv_geometry(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, true, &c);
    if (bad) return bad;
    if (workspace != nullptr && (uintptr_t)workspace % 16 != 0) return -17;
    if (output == nullptr) return -16;
    if (alpha_zero) {
        // output <- beta * output: the GEMM's quick path (K = 0 reads neither operand)
        return run(dtype, es, MI_GEMM_ROW_MAJOR, c.M, c.N, 0, 0, true, nullptr, 1, nullptr, c.N, beta_bits, beta_zero, beta_one,
                   output, c.N, nullptr, 0, stream);
    }
    if (image == nullptr) return -13;
    if (filter == nullptr) return -14;
    const size_t ws_bytes = workspace ? workspace_bytes : 0;
    const size_t matrix_bytes = round16((size_t)c.M * (size_t)c.K * (size_t)es);

    // fused: the im2row matrix is never formed
    const unsigned __int128 per = (unsigned __int128)c.M * (unsigned __int128)c.N * 4u;
    int64_t fit = ws_bytes > 0 ? (int64_t)((unsigned __int128)ws_bytes / per) : 0;
    if (fit > MAX_SPLIT) fit = MAX_SPLIT;
    if (fit < 1) fit = 1;
    double fused_us = 0.0;
    const bool image_aligned = (uintptr_t)image % 16 == 0;
    // the 16- and 8-bit kernels read the filter in words of 4 bytes along Cout: fewer channels go through the matrix
    const bool fusable = conv_fused_ok(batch, c, es) && (es == 4 || c.N >= 4 / es);
    const int fused_id = fusable ? conv_fused_kernel(dtype, c, fit, image_aligned, &fused_us) : -1;
    // explicit: the matrix in the workspace, then the GEMM with what is left of it
    const bool explicit_fits = ws_bytes >= matrix_bytes;
    bool fused = fused_id >= 0;
    if (t_conv_forced_path == 2 || !fused) {
        if (!explicit_fits) return -18;
        fused = false;
    } else if (t_conv_forced_path == 0 && explicit_fits && t_forced[dtype].id < 0) {
        const int gid = auto_kernel(dtype, c.N, c.M, c.K, c.N, c.K, 1, true, false, false);
        const double explicit_us = predict_us(dtype, kernel_info(dtype, gid), c.N, c.M, c.K, 1) + kIm2rowFixedUs +
                                   (double)matrix_bytes / kIm2rowBytesPerUs;
        if (explicit_us < fused_us) fused = false;
    }

    hipStream_t st = (hipStream_t)stream;
    if (!fused) {
        hipError_t e = launch_im2row_matrix(es, image, workspace, c.M, c.K, c.g, st);
        if (e != hipSuccess) return (int)e;
        const int rc = run(dtype, es, MI_GEMM_ROW_MAJOR, c.M, c.N, c.K, alpha_bits, false, workspace, c.K, filter, c.N, beta_bits,
                           beta_zero, beta_one, output, c.N, ws_bytes > matrix_bytes ? (char *)workspace + matrix_bytes : nullptr,
                           ws_bytes - matrix_bytes, stream);
        if (rc == 0) t_conv_path = 2;
        return rc < 0 ? -17 : rc;      // the GEMM's own argument checks cannot fail here except through the workspace
    }

    const KernelInfo *ki = kernel_info(dtype, fused_id);
    const Forced f = t_forced[dtype];
    const int64_t ktiles = ceil_div(c.K, ki->BK);
    int64_t sp = f.split >= 1 ? f.split : (ki->waves_k == 0 ? 1 : auto_split(dtype, ki, c.N, c.M, c.K, fit));
    if (sp > ktiles) sp = ktiles;
    if (sp > fit) sp = fit;
    if (sp < 1) sp = 1;
    Params p;
    memset(&p, 0, sizeof(p));
    p.A = filter; p.B = image; p.C = output; p.ws = workspace;
    p.lda = c.N; p.ldb = 0; p.ldc = c.N;
    p.M = (int)c.N; p.N = (int)c.M; p.K = (int)c.K;
    p.tiles_m = (int)ceil_div(c.N, ki->BM);
    p.tiles_n = (int)ceil_div(c.M, ki->BN);
    if ((int64_t)p.tiles_m * p.tiles_n > INT_MAX) return -1;
    p.ktiles = (int)ktiles;
    p.ktiles_per_split = (int)ceil_div(ktiles, sp);
    p.split = (int)ceil_div(ktiles, p.ktiles_per_split);
    p.alpha_bits = alpha_bits;
    p.beta_bits = beta_bits;
    p.use_beta = beta_zero ? 0 : 1;
    p.group_m = 8;
    p.xcd_remap = ((int64_t)p.tiles_m * p.tiles_n >= 64) ? 1 : 0;
    p.conv = c.g;
    p.vecA = aligned16(filter, c.N, es) ? 1 : 0;
    hipError_t e = conv_fused_launcher(ki, c, image_aligned)(p, st);
    if (e != hipSuccess) return (int)e;
    if (p.split > 1) {
        e = launch_reduce(dtype, workspace, output, p.M, p.N, p.ldc, p.split, p.alpha_bits, p.beta_bits, p.use_beta, st);
        if (e != hipSuccess) return (int)e;
    }
    t_last_id = fused_id;
    t_last_split = p.split;
    t_conv_path = 1;
    return 0;
}

}  // namespace

extern "C" {

int gemm_f32(int layout, int64_t M, int64_t N, int64_t K, float alpha, const float *A, int64_t lda, const float *B,
             int64_t ldb, float beta, float *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream)
{
    return run(MI_GEMM_F32, 4, layout, M, N, K, bits_of(alpha), alpha == 0.0f, A, lda, B, ldb, bits_of(beta),
               beta == 0.0f, beta == 1.0f, C, ldc, workspace, workspace_bytes, stream);
}

int gemm_f16(int layout, int64_t M, int64_t N, int64_t K, float alpha, const uint16_t *A, int64_t lda,
             const uint16_t *B, int64_t ldb, float beta, float *C, int64_t ldc, void *workspace,
             size_t workspace_bytes, void *stream)
{
    return run(MI_GEMM_F16, 2, layout, M, N, K, bits_of(alpha), alpha == 0.0f, A, lda, B, ldb, bits_of(beta),
               beta == 0.0f, beta == 1.0f, C, ldc, workspace, workspace_bytes, stream);
}

int gemm_bf16(int layout, int64_t M, int64_t N, int64_t K, float alpha, const uint16_t *A, int64_t lda,
              const uint16_t *B, int64_t ldb, float beta, float *C, int64_t ldc, void *workspace,
              size_t workspace_bytes, void *stream)
{
    return run(MI_GEMM_BF16, 2, layout, M, N, K, bits_of(alpha), alpha == 0.0f, A, lda, B, ldb, bits_of(beta),
               beta == 0.0f, beta == 1.0f, C, ldc, workspace, workspace_bytes, stream);
}

int gemm_f16_c16(int layout, int64_t M, int64_t N, int64_t K, float alpha, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb, float beta, uint16_t *C, int64_t ldc, void *workspace,
                 size_t workspace_bytes, void *stream)
{
    return run(MI_GEMM_F16, 2, layout, M, N, K, bits_of(alpha), alpha == 0.0f, A, lda, B, ldb, bits_of(beta),
               beta == 0.0f, beta == 1.0f, C, ldc, workspace, workspace_bytes, stream, false, false, C_F16);
}

int gemm_bf16_c16(int layout, int64_t M, int64_t N, int64_t K, float alpha, const uint16_t *A, int64_t lda,
                  const uint16_t *B, int64_t ldb, float beta, uint16_t *C, int64_t ldc, void *workspace,
                  size_t workspace_bytes, void *stream)
{
    return run(MI_GEMM_BF16, 2, layout, M, N, K, bits_of(alpha), alpha == 0.0f, A, lda, B, ldb, bits_of(beta),
               beta == 0.0f, beta == 1.0f, C, ldc, workspace, workspace_bytes, stream, false, false, C_BF16);
}

int gemm_i8(int layout, int64_t M, int64_t N, int64_t K, int32_t alpha, const int8_t *A, int64_t lda, const int8_t *B,
            int64_t ldb, int32_t beta, int32_t *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream)
{
    return run(MI_GEMM_I8, 1, layout, M, N, K, (uint32_t)alpha, alpha == 0, A, lda, B, ldb, (uint32_t)beta, beta == 0,
               beta == 1, C, ldc, workspace, workspace_bytes, stream);
}

int gemm_ex(int dtype, int layout, int transa, int transb, int64_t M, int64_t N, int64_t K, const void *alpha,
            const void *A, int64_t lda, const void *B, int64_t ldb, const void *beta, void *C, int64_t ldc,
            void *workspace, size_t workspace_bytes, void *stream)
{
    static const int es[NUM_DTYPES] = {4, 2, 1, 2};
    if (dtype < 0 || dtype >= NUM_DTYPES) return -1;
    if (transa != 0 && transa != 1) return -3;
    if (transb != 0 && transb != 1) return -4;
    if (alpha == nullptr) return -8;
    if (beta == nullptr) return -13;
    int rc;
    if (dtype == MI_GEMM_I8) {
        const int32_t a = *(const int32_t *)alpha, b = *(const int32_t *)beta;
        rc = run(dtype, 1, layout, M, N, K, (uint32_t)a, a == 0, A, lda, B, ldb, (uint32_t)b, b == 0, b == 1, C, ldc,
                 workspace, workspace_bytes, stream, transa != 0, transb != 0);
    } else {
        const float a = *(const float *)alpha, b = *(const float *)beta;
        rc = run(dtype, es[dtype], layout, M, N, K, bits_of(a), a == 0.0f, A, lda, B, ldb, bits_of(b), b == 0.0f,
                 b == 1.0f, C, ldc, workspace, workspace_bytes, stream, transa != 0, transb != 0);
    }
    // run() numbers the arguments of gemm_f32; here layout is the 2nd and M the 5th
    if (rc == -1) return -2;
    if (rc < -1) return rc - 3;
    return rc;
}

size_t gemm_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K)
{
    if (dtype < 0 || dtype >= NUM_DTYPES || M <= 0 || N <= 0 || K <= 0) return 0;
    if (M > INT_MAX || N > INT_MAX || K > INT_MAX) return 0;
    // callers size a workspace per call site and problem: remember the last few answers of this thread
    struct Slot { int dtype; int64_t M, N, K; size_t bytes; bool used; };
    constexpr int kSlots = 64;
    thread_local Slot t_slots[kSlots];
    Slot &slot = t_slots[((uint64_t)M * 0x9E3779B97F4A7C15ull ^ (uint64_t)N * 0xC2B2AE3D27D4EB4Full ^
                          (uint64_t)K * 0x165667B19E3779F9ull ^ (uint64_t)dtype) >> 40 & (kSlots - 1)];
    if (slot.used && slot.dtype == dtype && slot.M == M && slot.N == N && slot.K == K) return slot.bytes;
    // the largest split the model would give any configuration, in either orientation (a row-major call
    // runs the transposed problem), for aligned and unaligned operands, and for every slowdown the model
    // applies to transposed operands (gemm_ex on the fp32 kernels)
    static const bool kOrient[4][2] = {{false, false}, {true, false}, {false, true}, {true, true}};
    int64_t smax = 1;
    for (int id = 0; id < kernel_count(dtype); ++id) {
        const KernelInfo *ki = kernel_info(dtype, id);
        for (int o = 0; o < 4; ++o) {
            for (int align = ALIGN_NONE; align <= ALIGN_FULL; ++align) {
                const double f = staged_orientation_factor(dtype, ki, kOrient[o][0], kOrient[o][1], align);
                if (o > 0 && f == 1.0) continue;                // as the canonical orientation
                const int64_t s1 = auto_split(dtype, ki, M, N, K, MAX_SPLIT, align, f);
                const int64_t s2 = auto_split(dtype, ki, N, M, K, MAX_SPLIT, align, f);
                if (s1 > smax) smax = s1;
                if (s2 > smax) smax = s2;
            }
        }
    }
    const size_t bytes = smax <= 1 ? 0 : (size_t)smax * (size_t)M * (size_t)N * 4u;
    slot.dtype = dtype; slot.M = M; slot.N = N; slot.K = K; slot.bytes = bytes; slot.used = true;
    return bytes;
}

const char *gemm_status_string(int status)
{
    static const char *const arg[] = {
        "ok", "argument 1 (layout) is not MI_GEMM_COL_MAJOR or MI_GEMM_ROW_MAJOR",
        "argument 2 (M) is negative or too large", "argument 3 (N) is negative or too large",
        "argument 4 (K) is negative or too large", "argument 5 (alpha) is illegal", "argument 6 (A) is NULL",
        "argument 7 (lda) is smaller than the extent of A's contiguous dimension", "argument 8 (B) is NULL",
        "argument 9 (ldb) is smaller than the extent of B's contiguous dimension", "argument 10 (beta) is illegal",
        "argument 11 (C) is NULL", "argument 12 (ldc) is smaller than the extent of C's contiguous dimension",
        "argument 13 (workspace) is not 16-byte aligned", "argument 14 (workspace_bytes) is illegal",
        "argument 15 (stream) is illegal"};
    if (status <= 0 && status >= -15) return arg[-status];
    if (status > 0) return hipGetErrorString((hipError_t)status);
    return "unknown status";
}

const char *gemm_ex_status_string(int status)
{
    if (status == MI_GEMM_STATUS_STATIC_WS_TOO_SMALL)
        return "gemm_ex_static_ws: the K split of this problem needs more scratch than the library's fixed array "
               "holds; use gemm_ex with a workspace";
    if (status == -1) return "argument 1 (dtype) is not MI_GEMM_F32, MI_GEMM_F16, MI_GEMM_I8 or MI_GEMM_BF16";
    if (status == -2) return gemm_status_string(-1);
    if (status == -3) return "argument 3 (transa) is not 0 or 1";
    if (status == -4) return "argument 4 (transb) is not 0 or 1";
    if (status == -8) return "argument 8 (alpha) is NULL";
    if (status == -13) return "argument 13 (beta) is NULL";
    if (status <= -5 && status >= -18) {
        // the same text with the position in gemm_ex's list
        static thread_local char buf[160];
        const char *legacy = gemm_status_string(status + 3);
        const char *paren = strchr(legacy, '(');
        snprintf(buf, sizeof(buf), "argument %d %s", -status, paren ? paren : legacy);
        return buf;
    }
    return gemm_status_string(status);
}

int gemm_kernel_count(int dtype) { return (dtype >= 0 && dtype < NUM_DTYPES) ? kernel_count(dtype) : 0; }

const char *gemm_kernel_name(int dtype, int id)
{
    const KernelInfo *ki = (dtype >= 0 && dtype < NUM_DTYPES) ? kernel_info(dtype, id) : nullptr;
    return ki ? ki->name : "";
}

int gemm_force_kernel(int dtype, int id, int split)
{
    if (dtype < 0 || dtype >= NUM_DTYPES) return -1;
    if (id < -1 || id >= kernel_count(dtype)) return -1;
    t_forced[dtype].id = id;
    t_forced[dtype].split = split > 0 ? split : 0;
    return 0;
}

int gemm_kernel_tile(int dtype, int id, int *bm, int *bn, int *bk, int *workgroups_per_cu)
{
    const KernelInfo *ki = (dtype >= 0 && dtype < NUM_DTYPES) ? kernel_info(dtype, id) : nullptr;
    if (!ki) return -1;
    if (bm) *bm = ki->BM;
    if (bn) *bn = ki->BN;
    if (bk) *bk = ki->BK;
    if (workgroups_per_cu) *workgroups_per_cu = ki->min_blocks_per_cu;
    return 0;
}

int gemm_select(int dtype, int layout, int64_t M, int64_t N, int64_t K, size_t workspace_bytes, int *kernel_id,
                int *split)
{
    if (dtype < 0 || dtype >= NUM_DTYPES) return -1;
    if (layout != MI_GEMM_COL_MAJOR && layout != MI_GEMM_ROW_MAJOR) return -2;
    if (M <= 0 || M > INT_MAX) return -3;
    if (N <= 0 || N > INT_MAX) return -4;
    if (K <= 0 || K > INT_MAX) return -5;
    const bool col = (layout == MI_GEMM_COL_MAJOR);
    // tight leading dimensions and 16-byte aligned base addresses: canonical A has M' contiguous,
    // canonical B has K contiguous
    static const int es[NUM_DTYPES] = {4, 2, 1, 2};
    const int64_t Mc = col ? M : N, Nc = col ? N : M;
    const int align = alignment_class((Mc * es[dtype]) % 16 == 0, (K * es[dtype]) % 16 == 0, (Mc * es[dtype]) % 4 == 0, false, false);
    const Choice ch = choose(dtype, Mc, Nc, K, Mc, K, workspace_bytes, workspace_bytes > 0, align);
    if (kernel_id) *kernel_id = ch.id;
    if (split) *split = ch.split;
    return 0;
}

double gemm_predict_us(int dtype, int id, int64_t M, int64_t N, int64_t K, int split)
{
    const KernelInfo *ki = (dtype >= 0 && dtype < NUM_DTYPES) ? kernel_info(dtype, id) : nullptr;
    if (!ki || M <= 0 || N <= 0 || K <= 0 || split <= 0 || M > INT_MAX || N > INT_MAX || K > INT_MAX) return -1.0;
    // as gemm_select for a column-major problem: tight leading dimensions, aligned base addresses
    static const int es[NUM_DTYPES] = {4, 2, 1, 2};
    const int align = alignment_class((M * es[dtype]) % 16 == 0, (K * es[dtype]) % 16 == 0, (M * es[dtype]) % 4 == 0, false, false);
    return predict_us(dtype, ki, M, N, K, split, align);
}

int gemm_solo(int dtype, int id, int workgroups, int ksteps, int fill, void *stream)
{
    const KernelInfo *ki = (dtype >= 0 && dtype < NUM_DTYPES) ? kernel_info(dtype, id) : nullptr;
    if (!ki) return dtype < 0 || dtype >= NUM_DTYPES ? -1 : -2;
    if (workgroups < 1 || workgroups > (1 << 20)) return -3;
    if (ksteps < 0) return -4;
    if (fill != 0 && fill != 1) return -5;
    hipError_t e = ki->solo(workgroups, ksteps, fill, (hipStream_t)stream);
    return e == hipSuccess ? 0 : (int)e;
}

int conv2d_im2row_f32(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                      int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, float alpha, const float *image,
                      const float *filter, float beta, float *output, void *workspace, size_t workspace_bytes,
                      void *stream)
{
    return conv_run(MI_GEMM_F32, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, bits_of(alpha), alpha == 0.0f,
                    image, filter, bits_of(beta), beta == 0.0f, beta == 1.0f, output, workspace, workspace_bytes, stream);
}

int conv2d_im2row_ex(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                     int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, const void *alpha, const void *image,
                     const void *filter, const void *beta, void *output, void *workspace, size_t workspace_bytes,
                     void *stream)
{
    if (dtype < 0 || dtype >= NUM_DTYPES) return -1;
    if (alpha == nullptr) return -13;
    if (beta == nullptr) return -16;
    int rc;
    if (dtype == MI_GEMM_I8) {
        const int32_t a = *(const int32_t *)alpha, b = *(const int32_t *)beta;
        rc = conv_run(dtype, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, (uint32_t)a, a == 0, image, filter,
                      (uint32_t)b, b == 0, b == 1, output, workspace, workspace_bytes, stream);
    } else {
        const float a = *(const float *)alpha, b = *(const float *)beta;
        rc = conv_run(dtype, batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, bits_of(a), a == 0.0f, image, filter,
                      bits_of(b), b == 0.0f, b == 1.0f, output, workspace, workspace_bytes, stream);
    }
    return rc < 0 ? rc - 1 : rc;        // conv_run numbers the arguments of conv2d_im2row_f32; here dtype comes first
}

int im2row_f32(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t kh, int64_t kw, int64_t stride_h, int64_t stride_w,
               int64_t pad_h, int64_t pad_w, const float *image, float *matrix, void *stream)
{
    ConvGeometry c;
    int bad = conv_geometry(batch, H, W, Cin, 0, kh, kw, stride_h, stride_w, pad_h, pad_w, false, &c);
    if (bad) return bad <= -5 ? bad + 1 : bad;       // this list has no Cout
    if (image == nullptr) return -11;
    if (matrix == nullptr) return -12;
    hipError_t e = launch_im2row_matrix(4, image, matrix, c.M, c.K, c.g, (hipStream_t)stream);
    return e == hipSuccess ? 0 : (int)e;
}

int conv2d_im2row_shape(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                        int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int64_t *Hout, int64_t *Wout,
                        int64_t *M, int64_t *N, int64_t *K)
{
    ConvGeometry c;
    const int bad = conv_geometry(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, true, &c);
    if (bad) return bad;
    if (Hout) *Hout = c.g.Hout;
    if (Wout) *Wout = c.g.Wout;
    if (M) *M = c.M;
    if (N) *N = c.N;
    if (K) *K = c.K;
    return 0;
}

size_t conv2d_im2row_workspace_bytes(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                                     int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w)
{
    ConvGeometry c;
    if (conv_geometry(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, true, &c)) return 0;
    // room for the im2row matrix and for the GEMM's (or the fused kernel's) partial tiles
    return round16((size_t)c.M * (size_t)c.K * 4u) + round16(gemm_workspace_bytes(MI_GEMM_F32, c.M, c.N, c.K));
}

size_t conv2d_im2row_ex_workspace_bytes(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh,
                                        int64_t kw, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w)
{
    static const size_t es[NUM_DTYPES] = {4, 2, 1, 2};
    ConvGeometry c;
    if (dtype < 0 || dtype >= NUM_DTYPES) return 0;
    if (conv_geometry(batch, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, true, &c)) return 0;
    return round16((size_t)c.M * (size_t)c.K * es[dtype]) + round16(gemm_workspace_bytes(dtype, c.M, c.N, c.K));
}

const char *conv2d_im2row_ex_status_string(int status)
{
    if (status == -1) return "argument 1 (dtype) is not MI_GEMM_F32, MI_GEMM_F16, MI_GEMM_I8 or MI_GEMM_BF16";
    if (status == -13) return "argument 13 (alpha) is NULL";
    if (status == -16) return "argument 16 (beta) is NULL";
    if (status < -1 && status >= -19) {
        // the text of conv2d_im2row_f32's list with the position in this one
        static thread_local char buf[200];
        const char *text = conv2d_im2row_status_string(status + 1);
        const char *paren = strchr(text, '(');
        snprintf(buf, sizeof(buf), "argument %d %s", -status, paren ? paren : text);
        return buf;
    }
    return conv2d_im2row_status_string(status);
}

const char *conv2d_im2row_status_string(int status)
{
    static const char *const arg[] = {
        "ok", "argument 1 (batch) is not positive or the output has too many pixels", "argument 2 (H) is out of range",
        "argument 3 (W) is out of range", "argument 4 (Cin) is out of range or kh*kw*Cin is too large",
        "argument 5 (Cout) is out of range", "argument 6 (kh) is out of range", "argument 7 (kw) is out of range",
        "argument 8 (stride_h) is out of range", "argument 9 (stride_w) is out of range",
        "argument 10 (pad_h) is negative, too large, or the padded image is lower than the filter",
        "argument 11 (pad_w) is negative, too large, or the padded image is narrower than the filter",
        "argument 12 (alpha) is illegal", "argument 13 (image) is NULL", "argument 14 (filter) is NULL",
        "argument 15 (beta) is illegal", "argument 16 (output) is NULL",
        "argument 17 (workspace) is not 16-byte aligned",
        "argument 18 (workspace_bytes): this geometry needs the im2row matrix and the workspace is too small for it"};
    if (status == 0) return arg[0];
    if (status < 0 && status >= -18) return arg[-status];
    if (status > 0) return hipGetErrorString((hipError_t)status);
    return "unknown status";
}

int conv2d_im2row_force_path(int path)
{
    if (path < 0 || path > 2) return -1;
    t_conv_forced_path = path;
    return 0;
}

int conv2d_im2row_last_path(void) { return t_conv_path; }

int gemm_last_kernel_id(void) { return t_last_id; }
int gemm_last_split(void) { return t_last_split; }

}  // extern "C"
