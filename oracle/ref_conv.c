/*
 * CPU oracle for the convolution that the paper's rectangular GEMMs come from.  TEST INFRASTRUCTURE ONLY
 * (same rules as ref_gemm.c: never called from the GPU path, shares no code with it).
 *
 * The paper (Sec. "Rectangular Matrices", Tables "resnet50" and "vgg16") takes its GEMM sizes from the
 * im2row transform of convolution layers at batch 1: m = Hout*Wout, n = Cout, k = kh*kw*Cin.  It cites
 * the transform without writing it out, so the definition below is a reading (the usual one for a
 * channels-last tensor), fixed by those three sizes:
 *
 *   input   [batch][H][W][Cin]            (channels last)
 *   filter  [kh][kw][Cin][Cout]           = the K x N matrix B of the GEMM, row-major
 *   output  [batch][Hout][Wout][Cout]     = the M x N matrix C of the GEMM, row-major
 *   Hout = (H + 2*pad_h - kh) / stride_h + 1,  Wout likewise (integer division)
 *
 *   im2row: row (b, oh, ow), column (r, s, c) of the M x K matrix A holds
 *           input[b][oh*stride_h - pad_h + r][ow*stride_w - pad_w + s][c], or 0 where that lies outside
 *           the image (zero padding);
 *   convolution (cross-correlation, no filter flip):
 *           output[b][oh][ow][co] = alpha * sum_{r,s,c} A[(b,oh,ow)][(r,s,c)] * filter[r][s][c][co]
 *                                   + beta * output_old[b][oh][ow][co]      (beta == 0: old output not read)
 *
 * ref_conv2d_nhwc_f32 evaluates the sum directly over the image (it never forms A); ref_im2row_f32
 * forms A.  Products and sums are held in double.  Pins (tests/test_oracle_pins.py): a worked 3x3
 * example, a single-one input (gives the filter back, mirrored through the stride/pad rule), all-ones
 * operands (counts of taps inside the image), 1x1 filters (a plain GEMM), the identity
 * conv == ref_gemm(im2row, filter), and torch.nn.functional.conv2d in float64.
 * ref_im2row_ex / ref_conv2d_nhwc_ex are the same two definitions for every data type of the GEMM oracle
 * (dtype 0 = fp32, 1 = binary16 bit patterns, 2 = int8, 3 = bfloat16 bit patterns; inputs and filter in
 * that type): each input value is converted exactly to double (int8: to int64) with the converters of
 * ref_gemm.c, the sum is held in double (int64), the old and the new output are fp32 / double (int32 /
 * int64).  Pins: the same worked examples, single-one, all-ones and torch checks on values every type
 * holds exactly, and conv == ref_gemm_<type>(im2row, filter) on random values.
 * Return value: 0, or -1 for a geometry with no output, -2 for an unknown dtype.
 */
#include <stdint.h>
#include <stddef.h>

static int out_extent(int64_t in, int64_t k, int64_t stride, int64_t pad, int64_t *out)
{
    if (in <= 0 || k <= 0 || stride <= 0 || pad < 0 || in + 2 * pad < k) return -1;
    *out = (in + 2 * pad - k) / stride + 1;
    return 0;
}

int ref_im2row_f32(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t kh, int64_t kw,
                   int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                   const float *input, float *matrix)
{
    int64_t Hout, Wout;
    if (batch <= 0 || Cin <= 0 || out_extent(H, kh, stride_h, pad_h, &Hout) || out_extent(W, kw, stride_w, pad_w, &Wout))
        return -1;
    const int64_t K = kh * kw * Cin;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < batch * Hout * Wout; ++row) {
        const int64_t b = row / (Hout * Wout), oh = (row / Wout) % Hout, ow = row % Wout;
        for (int64_t r = 0; r < kh; ++r)
            for (int64_t s = 0; s < kw; ++s)
                for (int64_t c = 0; c < Cin; ++c) {
                    const int64_t ih = oh * stride_h - pad_h + r, iw = ow * stride_w - pad_w + s;
                    float v = 0.0f;
                    if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = input[((b * H + ih) * W + iw) * Cin + c];
                    matrix[row * K + (r * kw + s) * Cin + c] = v;
                }
    }
    return 0;
}

int ref_conv2d_nhwc_f32(int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                        int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                        float alpha, const float *input, const float *filter,
                        float beta, const float *output_old, double *output)
{
    int64_t Hout, Wout;
    if (batch <= 0 || Cin <= 0 || Cout <= 0 || out_extent(H, kh, stride_h, pad_h, &Hout) ||
        out_extent(W, kw, stride_w, pad_w, &Wout))
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < batch * Hout * Wout; ++pix) {
        const int64_t b = pix / (Hout * Wout), oh = (pix / Wout) % Hout, ow = pix % Wout;
        for (int64_t co = 0; co < Cout; ++co) {
            double acc = 0.0;
            for (int64_t r = 0; r < kh; ++r) {
                const int64_t ih = oh * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int64_t s = 0; s < kw; ++s) {
                    const int64_t iw = ow * stride_w - pad_w + s;
                    if (iw < 0 || iw >= W) continue;
                    for (int64_t c = 0; c < Cin; ++c)
                        acc += (double)input[((b * H + ih) * W + iw) * Cin + c] *
                               (double)filter[((r * kw + s) * Cin + c) * Cout + co];
                }
            }
            double v = (double)alpha * acc;
            if (beta != 0.0f) v += (double)beta * (double)output_old[pix * Cout + co];
            output[pix * Cout + co] = v;
        }
    }
    return 0;
}

/* ---- the same for every data type ---------------------------------------------------------------- */
double ref_half_to_double(uint16_t h);            /* ref_gemm.c */
double ref_bfloat16_to_double(uint16_t h);

static size_t elem_size(int dtype) { return dtype == 0 ? 4 : (dtype == 2 ? 1 : 2); }

static double elem_to_double(int dtype, const void *X, int64_t idx)
{
    switch (dtype) {
    case 0: return (double)((const float *)X)[idx];
    case 1: return ref_half_to_double(((const uint16_t *)X)[idx]);
    case 3: return ref_bfloat16_to_double(((const uint16_t *)X)[idx]);
    default: return (double)((const int8_t *)X)[idx];
    }
}

int ref_im2row_ex(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t kh, int64_t kw,
                  int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                  const void *input, void *matrix)
{
    int64_t Hout, Wout;
    if (dtype < 0 || dtype > 3) return -2;
    if (batch <= 0 || Cin <= 0 || out_extent(H, kh, stride_h, pad_h, &Hout) || out_extent(W, kw, stride_w, pad_w, &Wout))
        return -1;
    const int64_t K = kh * kw * Cin;
    const size_t es = elem_size(dtype);
    const unsigned char *in = (const unsigned char *)input;
    unsigned char *out = (unsigned char *)matrix;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < batch * Hout * Wout; ++row) {
        const int64_t b = row / (Hout * Wout), oh = (row / Wout) % Hout, ow = row % Wout;
        for (int64_t r = 0; r < kh; ++r)
            for (int64_t s = 0; s < kw; ++s)
                for (int64_t c = 0; c < Cin; ++c) {
                    const int64_t ih = oh * stride_h - pad_h + r, iw = ow * stride_w - pad_w + s;
                    unsigned char *dst = out + (size_t)(row * K + (r * kw + s) * Cin + c) * es;
                    for (size_t q = 0; q < es; ++q)           /* all-zero bytes are the value 0 in every type */
                        dst[q] = (ih >= 0 && ih < H && iw >= 0 && iw < W) ? in[(size_t)(((b * H + ih) * W + iw) * Cin + c) * es + q] : 0;
                }
    }
    return 0;
}

int ref_conv2d_nhwc_ex(int dtype, int64_t batch, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t kh, int64_t kw,
                       int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                       double alpha, const void *input, const void *filter,
                       double beta, const void *output_old, void *output)
{
    int64_t Hout, Wout;
    if (dtype < 0 || dtype > 3) return -2;
    if (batch <= 0 || Cin <= 0 || Cout <= 0 || out_extent(H, kh, stride_h, pad_h, &Hout) ||
        out_extent(W, kw, stride_w, pad_w, &Wout))
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < batch * Hout * Wout; ++pix) {
        const int64_t b = pix / (Hout * Wout), oh = (pix / Wout) % Hout, ow = pix % Wout;
        for (int64_t co = 0; co < Cout; ++co) {
            double acc = 0.0;
            int64_t iacc = 0;
            for (int64_t r = 0; r < kh; ++r) {
                const int64_t ih = oh * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int64_t s = 0; s < kw; ++s) {
                    const int64_t iw = ow * stride_w - pad_w + s;
                    if (iw < 0 || iw >= W) continue;
                    for (int64_t c = 0; c < Cin; ++c) {
                        const int64_t xi = ((b * H + ih) * W + iw) * Cin + c, wi = ((r * kw + s) * Cin + c) * Cout + co;
                        if (dtype == 2) iacc += (int64_t)((const int8_t *)input)[xi] * (int64_t)((const int8_t *)filter)[wi];
                        else acc += elem_to_double(dtype, input, xi) * elem_to_double(dtype, filter, wi);
                    }
                }
            }
            if (dtype == 2) {
                int64_t v = (int64_t)alpha * iacc;
                if (beta != 0.0) v += (int64_t)beta * (int64_t)((const int32_t *)output_old)[pix * Cout + co];
                ((int64_t *)output)[pix * Cout + co] = v;
            } else {
                double v = alpha * acc;
                if (beta != 0.0) v += beta * (double)((const float *)output_old)[pix * Cout + co];
                ((double *)output)[pix * Cout + co] = v;
            }
        }
    }
    return 0;
}
