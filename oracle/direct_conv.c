/*
 * CPU oracle for 2-D convolution in NHWC layout -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is checked against.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the product path never does, and this file shares no code with it.
 *
 * What it computes is the direct convolution of the paper's Listing 1, seven
 * nested loops:
 *
 *   out[n][oy][ox][oc] = sum over ky<R, kx<S, ic<C of
 *                        in[n][iy][ix][ic] * filt[oc][ky][kx][ic]
 *   iy = oy*SY + ky*DY - pad_top,   ix = ox*SX + kx*DX - pad_left,
 *
 * where a term is left out when (iy, ix) falls outside the input, which is
 * what implicit zero padding means (section 2.3, second paragraph).  The loop
 * nest keeps the listing's order n, oy, ox, oc, ky, kx, ic; nothing is
 * blocked, fused or reordered.
 *
 * Readings of the paper taken here:
 *  - the listing subtracts "PL" in the y formula and "PT" in the x formula;
 *    this is taken as a slip: y uses the top padding, x the left padding;
 *  - "0 <= ix < Win" is read as the two-sided range test it stands for;
 *  - the listing accumulates with += into an output whose start value it does
 *    not state; with alpha = 1, beta = 0 (section 2.1) the output starts at 0;
 *  - the output extent is never defined in the paper; the usual floor formula
 *    Hout = floor((Hin + pad_top + pad_bottom - DY*(R-1) - 1) / SY) + 1 is
 *    used (bottom / right padding only enter here);
 *  - the paper says nothing on quantised arithmetic.  The uint8 x int8 path
 *    computes sum (x - zero_point) * w in int32 over the in-bounds taps; a
 *    padding tap holds the zero point and so adds exactly 0.  The "raw"
 *    variant sums x * w over all taps with x = zero_point in the padding.
 *
 * Floating-point inputs are accumulated in double, integer ones in int32.
 * OpenMP splits the (n, oy) loops only, which leaves every output element's
 * own summation order untouched.
 */
#include <stdint.h>
#include <stddef.h>

typedef struct {
    int32_t N, Hin, Win, C, K, R, S;
    int32_t SY, SX, DY, DX;
    int32_t PT, PL, PB, PR;
} oracle_shape;

/* Output extent along one axis; returns <= 0 when the dilated kernel does not fit. */
int32_t oracle_out_extent(int32_t in, int32_t pad_lo, int32_t pad_hi, int32_t dil, int32_t ksize,
                          int32_t stride)
{
    int64_t span = (int64_t)in + pad_lo + pad_hi - (int64_t)dil * (ksize - 1) - 1;
    if (span < 0) return 0;
    return (int32_t)(span / stride) + 1;
}

/*
 * Direct convolution, double accumulation.
 *   in   : [N][Hin][Win] pixels, each `in_pixel_stride` doubles apart, C used
 *   filt : [K][R][S][C]
 *   out  : [N][Hout][Wout][K]
 *   abs_out (may be NULL): same shape, sum of |in * filt| per output element
 *          (the magnitude a rounding-error bound scales with)
 */
void oracle_conv2d_f64(const oracle_shape *p, const double *in, int64_t in_pixel_stride,
                       const double *filt, double *out, double *abs_out)
{
    const int32_t Hout = oracle_out_extent(p->Hin, p->PT, p->PB, p->DY, p->R, p->SY);
    const int32_t Wout = oracle_out_extent(p->Win, p->PL, p->PR, p->DX, p->S, p->SX);
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t n = 0; n < p->N; n++)
        for (int32_t oy = 0; oy < Hout; oy++)
            for (int32_t ox = 0; ox < Wout; ox++)
                for (int32_t oc = 0; oc < p->K; oc++) {
                    double acc = 0.0, mag = 0.0;
                    for (int32_t ky = 0; ky < p->R; ky++)
                        for (int32_t kx = 0; kx < p->S; kx++)
                            for (int32_t ic = 0; ic < p->C; ic++) {
                                const int32_t iy = oy * p->SY + ky * p->DY - p->PT;
                                const int32_t ix = ox * p->SX + kx * p->DX - p->PL;
                                if (0 <= ix && ix < p->Win && 0 <= iy && iy < p->Hin) {
                                    const double a =
                                        in[(((int64_t)n * p->Hin + iy) * p->Win + ix) * in_pixel_stride + ic];
                                    const double b = filt[(((int64_t)oc * p->R + ky) * p->S + kx) * p->C + ic];
                                    acc += a * b;
                                    if (abs_out) mag += (a * b < 0 ? -(a * b) : a * b);
                                }
                            }
                    const int64_t o = ((((int64_t)n * Hout + oy) * Wout + ox) * p->K) + oc;
                    out[o] = acc;
                    if (abs_out) abs_out[o] = mag;
                }
}

/*
 * Quantised direct convolution: uint8 input with a zero point, int8 filter,
 * int32 accumulation.  centred != 0: sum (x - zp) * w over in-bounds taps.
 * centred == 0 ("raw"): sum x * w over all taps, padding taps reading x = zp.
 */
void oracle_conv2d_u8i8(const oracle_shape *p, const uint8_t *in, int64_t in_pixel_stride,
                        const int8_t *filt, int32_t zero_point, int32_t centred, int32_t *out)
{
    const int32_t Hout = oracle_out_extent(p->Hin, p->PT, p->PB, p->DY, p->R, p->SY);
    const int32_t Wout = oracle_out_extent(p->Win, p->PL, p->PR, p->DX, p->S, p->SX);
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t n = 0; n < p->N; n++)
        for (int32_t oy = 0; oy < Hout; oy++)
            for (int32_t ox = 0; ox < Wout; ox++)
                for (int32_t oc = 0; oc < p->K; oc++) {
                    int32_t acc = 0;
                    for (int32_t ky = 0; ky < p->R; ky++)
                        for (int32_t kx = 0; kx < p->S; kx++)
                            for (int32_t ic = 0; ic < p->C; ic++) {
                                const int32_t iy = oy * p->SY + ky * p->DY - p->PT;
                                const int32_t ix = ox * p->SX + kx * p->DX - p->PL;
                                const int32_t b = filt[(((int64_t)oc * p->R + ky) * p->S + kx) * p->C + ic];
                                if (0 <= ix && ix < p->Win && 0 <= iy && iy < p->Hin) {
                                    const int32_t a =
                                        in[(((int64_t)n * p->Hin + iy) * p->Win + ix) * in_pixel_stride + ic];
                                    acc += (centred ? a - zero_point : a) * b;
                                } else if (!centred) {
                                    acc += zero_point * b;
                                }
                            }
                    out[((((int64_t)n * Hout + oy) * Wout + ox) * p->K) + oc] = acc;
                }
}

/*
 * Logical content of the indirection buffer (section 2.3, first two
 * paragraphs): one entry per output pixel m = (n, oy, ox) and kernel element
 * t = ky*S + kx.  The paper stores a pointer to the input pixel's row of C
 * values, or to the explicit zero vector when the tap is outside the input;
 * here the entry is the pixel's index (n*Hin + iy)*Win + ix, and -1 stands
 * for the zero vector.
 *   entries : [N*Hout*Wout][R*S]
 */
void oracle_indirection(const oracle_shape *p, int32_t *entries)
{
    const int32_t Hout = oracle_out_extent(p->Hin, p->PT, p->PB, p->DY, p->R, p->SY);
    const int32_t Wout = oracle_out_extent(p->Win, p->PL, p->PR, p->DX, p->S, p->SX);
    for (int32_t n = 0; n < p->N; n++)
        for (int32_t oy = 0; oy < Hout; oy++)
            for (int32_t ox = 0; ox < Wout; ox++)
                for (int32_t ky = 0; ky < p->R; ky++)
                    for (int32_t kx = 0; kx < p->S; kx++) {
                        const int32_t iy = oy * p->SY + ky * p->DY - p->PT;
                        const int32_t ix = ox * p->SX + kx * p->DX - p->PL;
                        const int64_t m = ((int64_t)n * Hout + oy) * Wout + ox;
                        const int64_t t = (int64_t)ky * p->S + kx;
                        int32_t e = -1;
                        if (0 <= ix && ix < p->Win && 0 <= iy && iy < p->Hin)
                            e = (n * p->Hin + iy) * p->Win + ix;
                        entries[m * ((int64_t)p->R * p->S) + t] = e;
                    }
}

/*
 * The indirect GEMM of Listing 3 read as a whole-matrix reference: for every
 * output pixel, walk its R*S entries, and for each take the dot product of the
 * C values the entry designates (the zero vector for -1) with the filter row
 * of that kernel element.  Used to check that entries + zero vector reproduce
 * the direct convolution; double accumulation.
 */
void oracle_indirect_gemm_f64(const oracle_shape *p, const int32_t *entries, const double *in,
                              int64_t in_pixel_stride, const double *zero_vec, const double *filt,
                              double *out)
{
    const int32_t Hout = oracle_out_extent(p->Hin, p->PT, p->PB, p->DY, p->R, p->SY);
    const int32_t Wout = oracle_out_extent(p->Win, p->PL, p->PR, p->DX, p->S, p->SX);
    const int64_t M = (int64_t)p->N * Hout * Wout;
    const int64_t T = (int64_t)p->R * p->S;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; m++)
        for (int32_t oc = 0; oc < p->K; oc++) {
            double acc = 0.0;
            for (int64_t t = 0; t < T; t++) {
                const int32_t e = entries[m * T + t];
                const double *row = e < 0 ? zero_vec : in + (int64_t)e * in_pixel_stride;
                const double *w = filt + ((int64_t)oc * T + t) * p->C;
                for (int32_t ic = 0; ic < p->C; ic++) acc += row[ic] * w[ic];
            }
            out[m * p->K + oc] = acc;
        }
}

/*
 * Output stage applied to the accumulators of the convolution above (an extension beyond the paper, which only
 * names a bias tensor among the operands of its benchmark protocol, section 3.1): per output channel oc
 *
 *   float  : y = acc + bias[oc];  relu: y = max(y, 0)                      (all in double)
 *   int32  : y = acc + bias[oc];  relu: y = max(y, 0)
 *   requantised uint8 (from the int32 result y):
 *            q = clamp( rint( (float)y * scale ) + out_zero_point, 0, 255 )
 *            with the product and the rounding (to nearest, ties to even) in IEEE single precision, the rounded
 *            value limited to +-1e9 before it becomes an integer.
 *
 * bias may be NULL (no bias).  `count` elements, channel = index % K.
 */
void oracle_epilogue_f64(double *y, int64_t count, int32_t K, const double *bias, int32_t relu)
{
    for (int64_t i = 0; i < count; i++) {
        double v = y[i] + (bias ? bias[i % K] : 0.0);
        if (relu && v < 0.0) v = 0.0;
        y[i] = v;
    }
}

void oracle_epilogue_i32(int32_t *y, int64_t count, int32_t K, const int32_t *bias, int32_t relu)
{
    for (int64_t i = 0; i < count; i++) {
        int32_t v = y[i] + (bias ? bias[i % K] : 0);
        if (relu && v < 0) v = 0;
        y[i] = v;
    }
}

void oracle_requantise_u8(const int32_t *y, int64_t count, float scale, int32_t out_zero_point, uint8_t *q)
{
    for (int64_t i = 0; i < count; i++) {
        volatile float prod = (float)y[i] * scale;      /* volatile: one correctly rounded single-precision product */
        float r = __builtin_rintf(prod);
        if (r > 1e9f) r = 1e9f;
        if (r < -1e9f) r = -1e9f;
        int64_t v = (int64_t)r + out_zero_point;
        if (v < 0) v = 0;
        if (v > 255) v = 255;
        q[i] = (uint8_t)v;
    }
}
