/*
 * CPU oracle for C = alpha*A*B + beta*C.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker the GPU library is compared against.  It shares no
 * code with the GPU path and must never be called from it: only the tests, the
 * smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * What it computes is the plain definition of the product (paper Sec. II-A:
 * A is m x k, B is k x n, C is m x n) in the alpha/beta form of the paper's
 * reference micro-kernel (Fig. "Exo code for GEMM micro-kernel"): every
 * C(i,j) is a sum over p of A(i,p)*B(p,j), scaled by alpha, plus beta times
 * the old C(i,j).  Blocking, packing and the micro-kernel of the paper only
 * reorder that sum, so the definition itself is the oracle.
 *
 * Arithmetic: every product and the running sum are held in double (fp32 and
 * binary16 inputs convert to double exactly, and a product of two of them is
 * exact in double) or in int64 (int8 inputs).  alpha and beta are applied in
 * the wide type.  beta == 0 means the old C is not read at all, so NaN or Inf
 * stored there cannot leak into the result (reference-BLAS convention).
 *
 * All pointers are host pointers.  layout: 0 = column-major, X(i,j) at
 * X[i + j*ldx]; 1 = row-major, X(i,j) at X[i*ldx + j].  The result goes to a
 * separate wide buffer D with its own leading dimension ldd in the same layout.
 * Return value: 0, or -1 for an unknown layout.
 *
 * Pins (tests/test_oracle_pins.py): exact rational brute force on 7x5x3,
 * identity and permutation operands, all-ones and rank-1 closed forms,
 * small-integer exactness, int8 extremes, all 65536 binary16 patterns against
 * numpy's float16, all 65536 bfloat16 patterns against the fp32 whose upper
 * half they are, and torch.matmul in float64/int64 on random inputs.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static inline size_t at(int layout, int64_t i, int64_t j, int64_t ld)
{
    return layout == 0 ? (size_t)i + (size_t)j * (size_t)ld
                       : (size_t)i * (size_t)ld + (size_t)j;
}

/* IEEE 754 binary16 bit pattern -> double, exactly (1 sign, 5 exponent, 10 fraction bits). */
double ref_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = (double)f * (1.0 / 16777216.0);            /* subnormal: f * 2^-24 */
    } else if (e == 31) {
        if (f == 0) {
            v = 1.0 / 0.0;
        } else {
            v = 0.0 / 0.0;
        }
    } else {
        v = ldexp((double)(1024 + f), e - 25);          /* (1024+f) * 2^(e-25) */
    }
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exactly (1 sign, 8 exponent, 7 fraction bits; the exponent
 * range and bias of IEEE binary32). */
double ref_bfloat16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xff;
    int f = h & 0x7f;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -133);                     /* subnormal: f * 2^-7 * 2^-126 */
    } else if (e == 255) {
        v = (f == 0) ? 1.0 / 0.0 : 0.0 / 0.0;
    } else {
        v = ldexp((double)(128 + f), e - 134);          /* (1 + f/128) * 2^(e-127) */
    }
    return sign ? -v : v;
}

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* fp32 inputs, double accumulation, double result. */
int ref_gemm_f32(int layout, int64_t M, int64_t N, int64_t K,
                 float alpha, const float *A, int64_t lda,
                 const float *B, int64_t ldb,
                 float beta, const float *C, int64_t ldc,
                 double *D, int64_t ldd)
{
    if (layout != 0 && layout != 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        for (int64_t i = 0; i < M; ++i) {
            double acc = 0.0;
            for (int64_t p = 0; p < K; ++p)
                acc += (double)A[at(layout, i, p, lda)] * (double)B[at(layout, p, j, ldb)];
            double r = (double)alpha * acc;
            if (beta != 0.0f) r += (double)beta * (double)C[at(layout, i, j, ldc)];
            D[at(layout, i, j, ldd)] = r;
        }
    }
    return 0;
}

/* binary16 inputs (bit patterns), double accumulation, fp32 C in, double result. */
int ref_gemm_f16(int layout, int64_t M, int64_t N, int64_t K,
                 float alpha, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb,
                 float beta, const float *C, int64_t ldc,
                 double *D, int64_t ldd)
{
    if (layout != 0 && layout != 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        for (int64_t i = 0; i < M; ++i) {
            double acc = 0.0;
            for (int64_t p = 0; p < K; ++p)
                acc += ref_half_to_double(A[at(layout, i, p, lda)]) *
                       ref_half_to_double(B[at(layout, p, j, ldb)]);
            double r = (double)alpha * acc;
            if (beta != 0.0f) r += (double)beta * (double)C[at(layout, i, j, ldc)];
            D[at(layout, i, j, ldd)] = r;
        }
    }
    return 0;
}

/* bfloat16 inputs (bit patterns), double accumulation, fp32 C in, double result. */
int ref_gemm_bf16(int layout, int64_t M, int64_t N, int64_t K,
                  float alpha, const uint16_t *A, int64_t lda,
                  const uint16_t *B, int64_t ldb,
                  float beta, const float *C, int64_t ldc,
                  double *D, int64_t ldd)
{
    if (layout != 0 && layout != 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        for (int64_t i = 0; i < M; ++i) {
            double acc = 0.0;
            for (int64_t p = 0; p < K; ++p)
                acc += ref_bfloat16_to_double(A[at(layout, i, p, lda)]) *
                       ref_bfloat16_to_double(B[at(layout, p, j, ldb)]);
            double r = (double)alpha * acc;
            if (beta != 0.0f) r += (double)beta * (double)C[at(layout, i, j, ldc)];
            D[at(layout, i, j, ldd)] = r;
        }
    }
    return 0;
}

/* int8 inputs, int64 accumulation; D holds the exact int64 value of
 * alpha*sum + beta*C (the caller wraps it to int32 where it wants to). */
int ref_gemm_i8(int layout, int64_t M, int64_t N, int64_t K,
                int32_t alpha, const int8_t *A, int64_t lda,
                const int8_t *B, int64_t ldb,
                int32_t beta, const int32_t *C, int64_t ldc,
                int64_t *D, int64_t ldd)
{
    if (layout != 0 && layout != 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        for (int64_t i = 0; i < M; ++i) {
            int64_t acc = 0;
            for (int64_t p = 0; p < K; ++p)
                acc += (int64_t)A[at(layout, i, p, lda)] * (int64_t)B[at(layout, p, j, ldb)];
            int64_t r = (int64_t)alpha * acc;
            if (beta != 0) r += (int64_t)beta * (int64_t)C[at(layout, i, j, ldc)];
            D[at(layout, i, j, ldd)] = r;
        }
    }
    return 0;
}

/*
 * The general form C = alpha*op(A)*op(B) + beta*C, op(X) = X or X^T (BLAS
 * convention: op(A) is M x K, op(B) is K x N; a transposed operand is stored
 * as the K x M, respectively N x K, matrix in the given layout).  Element
 * (i,j) of op(X) is element (j,i) of the stored X when X is transposed.
 * dtype: 0 = fp32, 1 = binary16, 3 = bfloat16 (D is double), 2 = int8 (D is
 * int64, alpha and beta are converted to int64).
 */
static inline size_t at_op(int layout, int trans, int64_t i, int64_t j, int64_t ld)
{
    return trans ? at(layout, j, i, ld) : at(layout, i, j, ld);
}

static inline double wide_elem(int dtype, const void *X, size_t idx)
{
    switch (dtype) {
    case 0: return (double)((const float *)X)[idx];
    case 1: return ref_half_to_double(((const uint16_t *)X)[idx]);
    case 3: return ref_bfloat16_to_double(((const uint16_t *)X)[idx]);
    default: return (double)((const int8_t *)X)[idx];
    }
}

int ref_gemm_ex(int dtype, int layout, int transa, int transb, int64_t M, int64_t N, int64_t K,
                double alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                double beta, const void *C, int64_t ldc, void *D, int64_t ldd)
{
    if (layout != 0 && layout != 1) return -1;
    if (dtype < 0 || dtype > 3) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        for (int64_t i = 0; i < M; ++i) {
            if (dtype == 2) {
                const int8_t *a = (const int8_t *)A, *b = (const int8_t *)B;
                int64_t acc = 0;
                for (int64_t p = 0; p < K; ++p)
                    acc += (int64_t)a[at_op(layout, transa, i, p, lda)] * (int64_t)b[at_op(layout, transb, p, j, ldb)];
                int64_t r = (int64_t)alpha * acc;
                if (beta != 0.0) r += (int64_t)beta * (int64_t)((const int32_t *)C)[at(layout, i, j, ldc)];
                ((int64_t *)D)[at(layout, i, j, ldd)] = r;
            } else {
                double acc = 0.0;
                for (int64_t p = 0; p < K; ++p)
                    acc += wide_elem(dtype, A, at_op(layout, transa, i, p, lda)) *
                           wide_elem(dtype, B, at_op(layout, transb, p, j, ldb));
                double r = alpha * acc;
                if (beta != 0.0) r += beta * (double)((const float *)C)[at(layout, i, j, ldc)];
                ((double *)D)[at(layout, i, j, ldd)] = r;
            }
        }
    }
    return 0;
}

/*
 * The same definition evaluated only at listed positions (is[s], js[s]), for
 * sizes where the full triple loop would take hours: out[s] = the wide value
 * of C(is[s], js[s]).  dtype: 0 = fp32, 1 = binary16, 2 = int8 (out then holds
 * the int64 result converted to double, exact below 2^53), 3 = bfloat16.
 */
int ref_gemm_sample(int dtype, int layout, int64_t K,
                    double alpha, const void *A, int64_t lda,
                    const void *B, int64_t ldb,
                    double beta, const void *C, int64_t ldc,
                    int64_t nsamp, const int64_t *is, const int64_t *js, double *out)
{
    if (layout != 0 && layout != 1) return -1;
    if (dtype < 0 || dtype > 3) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < nsamp; ++s) {
        int64_t i = is[s], j = js[s];
        double r;
        if (dtype == 2) {
            const int8_t *a = (const int8_t *)A, *b = (const int8_t *)B;
            int64_t acc = 0;
            for (int64_t p = 0; p < K; ++p)
                acc += (int64_t)a[at(layout, i, p, lda)] * (int64_t)b[at(layout, p, j, ldb)];
            int64_t v = (int64_t)alpha * acc;
            if (beta != 0.0) v += (int64_t)beta * (int64_t)((const int32_t *)C)[at(layout, i, j, ldc)];
            r = (double)v;
        } else {
            double acc = 0.0;
            if (dtype == 0) {
                const float *a = (const float *)A, *b = (const float *)B;
                for (int64_t p = 0; p < K; ++p)
                    acc += (double)a[at(layout, i, p, lda)] * (double)b[at(layout, p, j, ldb)];
            } else if (dtype == 1) {
                const uint16_t *a = (const uint16_t *)A, *b = (const uint16_t *)B;
                for (int64_t p = 0; p < K; ++p)
                    acc += ref_half_to_double(a[at(layout, i, p, lda)]) *
                           ref_half_to_double(b[at(layout, p, j, ldb)]);
            } else {
                const uint16_t *a = (const uint16_t *)A, *b = (const uint16_t *)B;
                for (int64_t p = 0; p < K; ++p)
                    acc += ref_bfloat16_to_double(a[at(layout, i, p, lda)]) *
                           ref_bfloat16_to_double(b[at(layout, p, j, ldb)]);
            }
            r = alpha * acc;
            if (beta != 0.0) r += beta * (double)((const float *)C)[at(layout, i, j, ldc)];
        }
        out[s] = r;
    }
    return 0;
}

/*
 * Narrowing of a wide result to a 16-bit storage format, for the entry points that keep C in 16 bits
 * (paper Sec. "Data types": the type of the operands of a micro-kernel is a parameter).  One rounding
 * to nearest, ties to even, of the value given; overflow gives infinity, NaN stays NaN (quiet).
 * frac_bits = 10, min_exp = -14, max_exp = 15 is IEEE binary16; 7, -126, 127 is bfloat16.
 * The scaling by a power of two and nearbyint() (default rounding mode: to nearest even) are exact
 * steps, so this is the definition written out.  Pinned against numpy's float16 conversion, against
 * round trips of all 65536 patterns of both formats and against hand-picked ties.
 */
static uint16_t narrow16(double x, int frac_bits, int min_exp, int max_exp)
{
    const int exp_bits = 15 - frac_bits;
    const uint16_t sign = signbit(x) ? 0x8000u : 0u;
    const uint16_t exp_all = (uint16_t)(((1u << exp_bits) - 1u) << frac_bits);
    if (isnan(x)) return (uint16_t)(sign | exp_all | (1u << (frac_bits - 1)));
    const double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | exp_all);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                       /* a in [2^(e-1), 2^e) */
    int exp = e - 1;
    if (exp < min_exp) exp = min_exp;         /* subnormal range: fixed quantum */
    const double quantum = ldexp(1.0, exp - frac_bits);
    const double r = nearbyint(a / quantum) * quantum;
    const double largest = (2.0 - ldexp(1.0, -frac_bits)) * ldexp(1.0, max_exp);
    if (r > largest) return (uint16_t)(sign | exp_all);
    if (r < ldexp(1.0, min_exp)) return (uint16_t)(sign | (uint16_t)(r / ldexp(1.0, min_exp - frac_bits)));
    (void)frexp(r, &e);
    exp = e - 1;
    const double frac = r / ldexp(1.0, exp) - 1.0;
    return (uint16_t)(sign | (uint16_t)((exp - min_exp + 1) << frac_bits) | (uint16_t)(frac * (double)(1 << frac_bits)));
}

void ref_narrow_f16(const double *x, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = narrow16(x[i], 10, -14, 15);
}

void ref_narrow_bf16(const double *x, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = narrow16(x[i], 7, -126, 127);
}
