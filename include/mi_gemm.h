/*
 * mi_gemm - general matrix multiplication C = alpha*A*B + beta*C on one MI355X.
 *
 * The operation is the GEMM of the paper's Sec. II-A (A is M x K, B is K x N,
 * C is M x N) in the alpha/beta form of its reference micro-kernel (Fig. "Exo
 * code for GEMM micro-kernel").  The implementation follows the structure of
 * the paper's Fig. "Pseudo-code of the BLIS base GEMM algorithm" re-mapped to
 * the GPU: loops L1 and L3 become the grid of workgroup tiles, loop L2 becomes
 * the K loop of a workgroup (optionally split over workgroups), the packing
 * routines become the staging of operand tiles into LDS, loops L4/L5 become the
 * waves of a workgroup and their MFMA blocks, and the micro-kernel (L6) is a
 * chain of MFMA instructions on accumulators held in registers.
 *
 * Common conventions for the GEMM entry points (gemm_f32, gemm_f16, gemm_bf16,
 * gemm_i8, gemm_f16_c16, gemm_bf16_c16; gemm_ex adds transposed operands,
 * gemm_ex_static_ws needs no workspace, the convolution calls further down
 * state their own arguments)
 * --------------------------------------------------------------------------
 * layout   MI_GEMM_COL_MAJOR: X(i,j) is X[i + j*ldx];  MI_GEMM_ROW_MAJOR:
 *          X(i,j) is X[i*ldx + j].  One layout applies to A, B and C.  Only
 *          gemm_ex has transpose flags.
 * M, N, K  >= 0.  M == 0 or N == 0: nothing is touched.  K == 0 or alpha == 0:
 *          C <- beta*C and A, B are never read.
 * A, B, C  DEVICE pointers owned by the caller; A and B are only read, C is
 *          read (unless beta == 0) and written.  beta == 0 means C is
 *          overwritten and its old contents - NaN and Inf included - are never
 *          read.  C must not overlap A, B or the workspace.  Only natural
 *          element alignment is required; 16-byte aligned base pointers and
 *          leading dimensions that are multiples of 16 bytes select the fast
 *          loaders.
 * lda/b/c  leading dimensions in elements: column-major lda >= max(1,M),
 *          ldb >= max(1,K), ldc >= max(1,M); row-major lda >= max(1,K),
 *          ldb >= max(1,N), ldc >= max(1,N).
 * workspace, workspace_bytes
 *          optional DEVICE scratch owned by the caller, used when the K loop
 *          is split over several workgroups (few output tiles, long K).  It
 *          may be NULL / 0: the library then runs without splitting.  The
 *          library itself never allocates device memory.  A size of at least
 *          gemm_workspace_bytes(...) allows every split the selector may pick.
 *          The base must be 16-byte aligned.
 * stream   a hipStream_t passed as void*; NULL is the default stream.  Calls
 *          are asynchronous on that stream; the library never synchronises.
 *
 * Return value: 0 on success; -k if the k-th argument (1-based, in the order
 * of the prototype) is illegal, in which case nothing was launched; a positive
 * value is a HIP error code from the launch.  gemm_status_string() describes
 * any of them.
 *
 * Results are deterministic: the same call (same arguments, workspace size
 * included) on the same data gives the same bits, because a split K loop is
 * reduced in fixed order.  A different workspace size may change the split and
 * with it the floating-point rounding order; int8 results never depend on it.
 */
#ifndef MI_GEMM_H
#define MI_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MI_GEMM_COL_MAJOR = 0, MI_GEMM_ROW_MAJOR = 1 };
enum { MI_GEMM_F32 = 0, MI_GEMM_F16 = 1, MI_GEMM_I8 = 2, MI_GEMM_BF16 = 3 };

/* fp32 inputs and output, true fp32 MFMA arithmetic (no reduced-precision
 * splitting), fp32 accumulation.  Paper Sec. II-A; alpha/beta as in its
 * reference micro-kernel. */
int gemm_f32(int layout, int64_t M, int64_t N, int64_t K,
             float alpha, const float *A, int64_t lda,
             const float *B, int64_t ldb,
             float beta, float *C, int64_t ldc,
             void *workspace, size_t workspace_bytes, void *stream);

/* IEEE binary16 inputs (bit patterns), fp32 accumulation, fp32 C in and out.
 * The data-type retargeting of the paper's Sec. "Data types". */
int gemm_f16(int layout, int64_t M, int64_t N, int64_t K,
             float alpha, const uint16_t *A, int64_t lda,
             const uint16_t *B, int64_t ldb,
             float beta, float *C, int64_t ldc,
             void *workspace, size_t workspace_bytes, void *stream);

/* bfloat16 inputs (bit patterns: the upper 16 bits of an fp32), fp32 accumulation,
 * fp32 C in and out.  Another precision of the paper's Sec. "Data types" (a
 * micro-kernel is re-targeted by changing the type of its operands only); same
 * arguments, layouts, alignment rules and error codes as gemm_f16. */
int gemm_bf16(int layout, int64_t M, int64_t N, int64_t K,
              float alpha, const uint16_t *A, int64_t lda,
              const uint16_t *B, int64_t ldb,
              float beta, float *C, int64_t ldc,
              void *workspace, size_t workspace_bytes, void *stream);

/* The same two with C kept in the 16-bit format of the inputs (bit patterns), in and out: the product
 * is accumulated in fp32, alpha*acc + beta*C_old is evaluated in fp32 and rounded once, to nearest
 * even, when it is stored (overflow gives infinity).  The storage type of C is one more of the
 * type parameters the paper's Sec. "Data types" changes.  ldc counts 16-bit elements; the K-split
 * workspace still holds fp32 partial tiles.  Everything else as gemm_f16 / gemm_bf16. */
int gemm_f16_c16(int layout, int64_t M, int64_t N, int64_t K,
                 float alpha, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb,
                 float beta, uint16_t *C, int64_t ldc,
                 void *workspace, size_t workspace_bytes, void *stream);
int gemm_bf16_c16(int layout, int64_t M, int64_t N, int64_t K,
                  float alpha, const uint16_t *A, int64_t lda,
                  const uint16_t *B, int64_t ldb,
                  float beta, uint16_t *C, int64_t ldc,
                  void *workspace, size_t workspace_bytes, void *stream);

/* int8 inputs, int32 accumulation, int32 C in and out, int32 alpha and beta.
 * The result is exact (bit-for-bit) as long as the true value of every
 * intermediate fits in int32, which holds for K <= 131071 at alpha = 1,
 * beta = 0; beyond that the arithmetic wraps modulo 2^32. */
int gemm_i8(int layout, int64_t M, int64_t N, int64_t K,
            int32_t alpha, const int8_t *A, int64_t lda,
            const int8_t *B, int64_t ldb,
            int32_t beta, int32_t *C, int64_t ldc,
            void *workspace, size_t workspace_bytes, void *stream);

/* The general form C = alpha*op(A)*op(B) + beta*C for any data type, op(X) = X
 * (trans = 0) or X^T (trans = 1): op(A) is M x K and op(B) is K x N, so a
 * transposed A is stored as a K x M matrix and a transposed B as N x K, in the
 * layout given (column-major: X(i,j) at X[i + j*ldx], row-major: X[i*ldx + j]),
 * with lda / ldb at least the contiguous extent of the stored matrix.  This is
 * the transposed-operand case the paper's Sec. "Micro-kernel Generation" sets
 * aside when it fixes row-major C code with C^T = B^T A^T.  alpha and beta are
 * host pointers to a float (fp32, fp16, bf16) or an int32 (int8).  With
 * transa = transb = 0 the call is gemm_f32 / gemm_f16 / gemm_i8 / gemm_bf16;
 * every combination runs on the direct kernels at about their normal speed when the rows of the
 * operands are 16-byte aligned (a K-contiguous A is staged like B, an N-contiguous B like A; for
 * fp16 / bf16 / int8 the latter on the square tiles); fp32 operands whose rows are not 16-byte
 * aligned go through the staged kernels or the guarded path of the direct ones.  Same ownership, stream and
 * workspace rules; status -k names the k-th argument of this list
 * (gemm_ex_status_string gives the text). */
int gemm_ex(int dtype, int layout, int transa, int transb, int64_t M, int64_t N, int64_t K,
            const void *alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
            const void *beta, void *C, int64_t ldc,
            void *workspace, size_t workspace_bytes, void *stream);
const char *gemm_ex_status_string(int status);

/* gemm_ex for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation): the same operation, arguments
 * (without workspace and workspace_bytes; stream is the 16th) and status codes, and bit-for-bit the
 * result of gemm_ex with a workspace of gemm_workspace_bytes(dtype, M, N, K) bytes.  The partial tiles
 * of a split K loop are kept in a fixed array of MI_GEMM_STATIC_WS_BYTES that is part of the library's
 * code object (one copy per GPU, held until the process ends) instead of a caller's workspace.  The
 * call allocates and frees nothing.  A problem whose gemm_workspace_bytes exceeds the array is
 * rejected with MI_GEMM_STATUS_STATIC_WS_TOO_SMALL and nothing is launched (use gemm_ex with a
 * workspace).  All calls on one GPU share that GPU's array: calls that may overlap on one GPU
 * (different streams, or threads) race on it and must be ordered by the caller; calls on one stream
 * are ordered.  The array keeps the last call's partial tiles; no call reads what it has not
 * written first.  The first call on each GPU looks the array's address up and should be made outside
 * graph capture. */
#define MI_GEMM_STATIC_WS_BYTES (16u << 20)
#define MI_GEMM_STATUS_STATIC_WS_TOO_SMALL (-100)
int gemm_ex_static_ws(int dtype, int layout, int transa, int transb, int64_t M, int64_t N, int64_t K,
                      const void *alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                      const void *beta, void *C, int64_t ldc, void *stream);

/* Convolution through the im2row GEMM, fp32.  The paper's Sec. "Rectangular Matrices" takes the GEMM
 * sizes of its Tables "resnet50" and "vgg16" from the im2row transform of convolution layers
 * (m = Hout*Wout at batch 1, n = Cout, k = kh*kw*Cin) and its conclusions name convolutions as the next
 * code to generate; it cites the transform without writing it out, so this is the usual channels-last one:
 *   image  [batch][H][W][Cin], filter [kh][kw][Cin][Cout] (the K x N matrix B, row-major),
 *   output [batch][Hout][Wout][Cout] (the M x N matrix C, row-major), all device pointers, dense,
 *   Hout = (H + 2*pad_h - kh)/stride_h + 1, Wout likewise (integer division),
 *   output[b][oh][ow][co] = alpha * sum over r < kh, s < kw, c < Cin of
 *       image[b][oh*stride_h - pad_h + r][ow*stride_w - pad_w + s][c] * filter[r][s][c][co]
 *       + beta * output[b][oh][ow][co]
 *   with zeros for image positions outside [0,H) x [0,W), no filter flip; beta == 0: output is not read.
 * When the image is smaller than 2 GiB (and, unless Cin is a multiple of 16, kh*kw*Cin < 2^22) the
 * GEMM kernels read the im2row matrix from the image in place (it is never formed); with Cin a
 * multiple of 32 and a 16-byte aligned image also the kernels that stage tiles in LDS do.  Otherwise, or
 * when the timing model expects it to be faster and the workspace has room, the matrix is written
 * into the workspace (M*K floats) and the GEMM runs on it.  conv2d_im2row_workspace_bytes gives a workspace
 * that suffices for either; a smaller one (or none) restricts the call to the in-place path and
 * its K split.  Same stream, ownership and error conventions as gemm_f32: -k names the k-th argument
 * of this list (conv2d_im2row_status_string), -18 = this geometry needs the im2row matrix and the
 * workspace is too small for it.  Asynchronous on `stream`. */
int conv2d_im2row_f32(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                      int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                      float alpha, const float *image, const float *filter,
                      float beta, float *output,
                      void *workspace, size_t workspace_bytes, void *stream);
size_t conv2d_im2row_workspace_bytes(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh,
                                     int64_t kw, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w);
const char *conv2d_im2row_status_string(int status);

/* The same convolution for any data type, as gemm_ex is to gemm_f32 (the data-type retargeting of the paper's
 * Sec. "Data types" applied to the im2row GEMMs of its Sec. "Rectangular Matrices"): image and filter hold fp32,
 * binary16 or bfloat16 bit patterns, or int8; the sum is accumulated in fp32 (int32 for int8) and the output is
 * fp32 (int32), in and out; alpha and beta are host pointers to a float (an int32 for int8).  Same layouts,
 * zero padding, stream, ownership and workspace rules as conv2d_im2row_f32.  For the 16- and 8-bit types the
 * kernels read the im2row matrix from the image in place when Cin is a multiple of their K step (32 elements
 * of 16 bits, 64 of 8 bits), the image is smaller than 2 GiB and Cout is at least 2 (4 for int8); otherwise the
 * matrix is written into the workspace (M*K elements of the input type) and the GEMM runs on it.
 * conv2d_im2row_ex_workspace_bytes gives a workspace that suffices for either.  Status -k names the k-th
 * argument of this list (conv2d_im2row_ex_status_string); -19 = the geometry needs the im2row matrix and the
 * workspace is too small for it. */
int conv2d_im2row_ex(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                     int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                     const void *alpha, const void *image, const void *filter,
                     const void *beta, void *output,
                     void *workspace, size_t workspace_bytes, void *stream);
size_t conv2d_im2row_ex_workspace_bytes(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                        int64_t kh, int64_t kw, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                        int64_t pad_w);
const char *conv2d_im2row_ex_status_string(int status);

/* Output extent and GEMM sizes of that convolution (pure host computation); any output pointer may be
 * NULL.  Returns 0 or the -k of conv2d_im2row_f32's geometry arguments. */
int conv2d_im2row_shape(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                        int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                        int64_t *Hout, int64_t *Wout, int64_t *M, int64_t *N, int64_t *K);

/* The im2row transform on its own: matrix[M][K] (row-major, dense, device memory of M*K floats owned by
 * the caller), row (b, oh, ow), column (r, s, c), from the same image and geometry as above.
 * Returns 0, -k for the k-th argument of this list, or a HIP error. */
int im2row_f32(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t kh, int64_t kw,
               int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
               const float *image, float *matrix, void *stream);

/* For tests and reports: restrict later conv2d_im2row_f32 calls of the calling thread to one path
 * (0 automatic, 1 in place when the geometry allows it, 2 through the im2row matrix); which path the
 * last call on this thread took (0 none, 1 in place, 2 through the matrix).  gemm_force_kernel(F32, ...)
 * and gemm_last_kernel_id / gemm_last_split apply to the GEMM inside. */
int conv2d_im2row_force_path(int path);
int conv2d_im2row_last_path(void);

/* Upper bound of the workspace any split of the K loop may use for this
 * problem (dtype is one of MI_GEMM_F32/F16/I8/BF16); 0 if M, N or K is not positive. */
size_t gemm_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K);

/* Text for a status returned by the entry points (static storage). */
const char *gemm_status_string(int status);

/*
 * Kernel table introspection, for tests, tuning and reports.  Each dtype has
 * gemm_kernel_count(dtype) tile configurations ("per-shape micro-kernels" in
 * the paper's terms, Sec. "Edge Cases"), numbered from 0.
 * gemm_kernel_name() returns a static string such as "f32_128x128_w64x64".
 * gemm_force_kernel(dtype, id, split) overrides the selector for later calls
 * made by the calling thread (other threads keep their own setting; meant for
 * tests and tuning): id = -1 restores automatic selection; split <= 0 lets the
 * selector choose the K split, split >= 1 fixes it (clamped to what the
 * workspace allows).  Returns 0, or -1 for an unknown dtype / id.
 * gemm_last_kernel_id() / gemm_last_split() report what the most recent call
 * on this thread launched (-1 / 0 if it launched no MFMA kernel).
 */
int gemm_kernel_count(int dtype);
const char *gemm_kernel_name(int dtype, int id);
int gemm_force_kernel(int dtype, int id, int split);
int gemm_last_kernel_id(void);
int gemm_last_split(void);

/* What a call with these arguments would launch (pure host computation, nothing
 * runs; the answer for a problem is remembered per thread, so a repeated question
 * - and the selection inside a repeated GEMM call - costs a table lookup, not an
 * evaluation of the timing model): the tile configuration and the K split chosen by the selector - or the
 * forced ones - for a workspace of `workspace_bytes`, operands with tight leading
 * dimensions and 16-byte aligned base addresses.  Either output pointer may
 * be NULL.  Returns 0, or -1 unknown dtype, -2 unknown layout, -3/-4/-5 M/N/K
 * not positive or too large. */
int gemm_select(int dtype, int layout, int64_t M, int64_t N, int64_t K, size_t workspace_bytes, int *kernel_id,
                int *split);

/* The selector's timing model (the counterpart of the analytical blocking model
 * the paper cites in Sec. "Blocked algorithms for GEMM"): the time in
 * microseconds it predicts for tile configuration `id` with K split `split` on
 * the canonical (column-major) problem M x N x K with tight leading dimensions
 * and 16-byte aligned base addresses (as gemm_select assumes), launch included.
 * Pure host computation.  Returns a negative value for an unknown dtype or id, or M, N, K
 * or split that are not positive. */
double gemm_predict_us(int dtype, int id, int64_t M, int64_t N, int64_t K, int split);

/* Tile of configuration `id`: BM x BN of C per workgroup, BK elements of K per
 * step, and how many workgroups the kernel is built to keep resident per CU.
 * Any output pointer may be NULL.  Returns 0, or -1 for an unknown dtype / id. */
int gemm_kernel_tile(int dtype, int id, int *bm, int *bn, int *bk, int *workgroups_per_cu);

/*
 * Solo mode (paper Sec. "Solo Mode": the micro-kernel run on its own).  Launches
 * `workgroups` workgroups of configuration `id`; each fills one LDS stage with
 * operands (fill = 0: zeros, 1: pseudo-random finite values) and repeats the
 * fragment reads and MFMAs of one K step `ksteps` times on it - no global
 * memory traffic, no barriers, no output.  The work is
 * workgroups * ksteps * 2*BM*BN*BK flop (ops); the caller times it on `stream`
 * (asynchronous, like the GEMM calls).  The rate reached is the measured
 * ceiling for that tile on this machine at the clock it sustains under the
 * load.  Returns 0; -1/-2 unknown dtype/id, -3 workgroups outside [1, 2^20],
 * -4 negative ksteps, -5 fill not 0 or 1; positive = HIP error code.
 */
int gemm_solo(int dtype, int id, int workgroups, int ksteps, int fill, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MI_GEMM_H */
