/*
 * conv_oracle.c -- CPU reference for a 2-D convolution layer (cross-correlation with zero
 * padding, as deep-learning libraries define "Conv2d"), accumulated in IEEE fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  The yardstick for the correctness leg of the validation gate
 * (paper Sec. 3.1; Sec. 4.1 "Workloads": Conv2d with N=8, C=64, H=W=56, F=128, 3x3, stride 1,
 * padding 1, FP16; correctness at three random seeds) applied to the convolution kernels of
 * the HIP library.  It shares no code with that library and is never linked, imported or
 * called from it.  Built into the same shared object as gemm_oracle.c, whose oracle_decode()
 * (bit pattern -> real value) it calls.
 *
 * What it computes.  Activations x[n][h][w][c] (N x H x W x C, channels fastest), filters
 * w[f][r][s][c] (F x R x S x C, channels fastest), output y[n][p][q][f] (N x P x Q x F) with
 * P = (H + 2 pad_h - R) / stride_h + 1, Q = (W + 2 pad_w - S) / stride_w + 1 (integer division):
 *
 *     y_ref[n,p,q,f] = sum_{r<R} sum_{s<S} sum_{c<C} X(n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c) * dec(w[f,r,s,c])
 *     X(n,h,w,c)     = dec(x[n,h,w,c]) if 0 <= h < H and 0 <= w < W, else 0
 *     D[n,p,q,f]     = the same sum over |X| * |dec w|
 *
 * The filter is NOT flipped (cross-correlation).  Every product and sum is an fp64 operation
 * taken in increasing (r, s, c); products of two <= 24-bit significands are exact.  D is the
 * denominator of the normalised error max |y - y_ref| / D used as the acceptance metric.  The
 * paper does not define the oracle (it says "correctness" only): this is the layer's textbook
 * definition as nested loops; nothing is blocked, lowered to a matrix product or reordered.
 * Threads split independent output pixels only.
 *
 * Pins (tests/test_conv_oracle_pins.py): centre-tap identity filter, single-tap shifts (which
 * fix the direction of r, s and of the padding), all-ones closed form (C x number of taps inside
 * the image: 9C / 6C / 4C for 3x3, pad 1), 1x1 filters against an int64 matrix product,
 * integer-valued inputs against scipy.signal.correlate2d and against torch's fp64 conv2d with
 * strides and paddings, exact rational brute force on tiny shapes, linearity in x and w.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { CONV_ORACLE_OK = 0, CONV_ORACLE_BAD_ARG = 1, CONV_ORACLE_NO_MEMORY = 2 };

double oracle_decode(int dtype, uint32_t code);   /* gemm_oracle.c */

static int conv_elem_bytes(int dtype)
{
    return dtype == 0 ? 4 : (dtype == 1 || dtype == 2) ? 2 : dtype == 3 ? 1 : 0;
}

static double conv_load(int dtype, const void *base, int64_t idx)
{
    const unsigned char *p = (const unsigned char *)base;
    if (dtype == 0) { uint32_t c; memcpy(&c, p + 4 * idx, 4); return oracle_decode(dtype, c); }
    if (dtype == 1 || dtype == 2) { uint16_t c; memcpy(&c, p + 2 * idx, 2); return oracle_decode(dtype, c); }
    return oracle_decode(dtype, p[idx]);
}

static int conv_check(int dtype, int64_t N, int64_t H, int64_t W, int64_t C, int64_t F, int64_t R, int64_t S,
                      int64_t sh, int64_t sw, int64_t ph, int64_t pw, const void *x, const void *w)
{
    if (conv_elem_bytes(dtype) == 0) return CONV_ORACLE_BAD_ARG;
    if (N < 0 || H < 1 || W < 1 || C < 0 || F < 0 || R < 1 || S < 1) return CONV_ORACLE_BAD_ARG;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0) return CONV_ORACLE_BAD_ARG;
    if (H + 2 * ph < R || W + 2 * pw < S) return CONV_ORACLE_BAD_ARG;
    if (N > 0 && C > 0 && !x) return CONV_ORACLE_BAD_ARG;
    if (F > 0 && C > 0 && !w) return CONV_ORACLE_BAD_ARG;
    return CONV_ORACLE_OK;
}

/* Output extent along one axis: the number of filter positions, `stride` apart, that fit into
 * the padded extent. */
static int64_t conv_out(int64_t extent, int64_t pad, int64_t filt, int64_t stride)
{
    return (extent + 2 * pad - filt) / stride + 1;
}

void oracle_conv2d_output_size(int64_t H, int64_t W, int64_t R, int64_t S, int64_t stride_h, int64_t stride_w,
                               int64_t pad_h, int64_t pad_w, int64_t *P, int64_t *Q)
{
    *P = conv_out(H, pad_h, R, stride_h);
    *Q = conv_out(W, pad_w, S, stride_w);
}

/* One output from decoded copies (xd, wd hold fp64 values in the storage order of x and w). */
static void conv_point(const double *xd, const double *wd, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S,
                       int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                       int64_t n, int64_t p, int64_t q, int64_t f, double *y, double *d)
{
    double acc = 0.0, mag = 0.0;
    for (int64_t r = 0; r < R; ++r) {
        const int64_t h = p * sh - ph + r;
        for (int64_t s = 0; s < S; ++s) {
            const int64_t ww = q * sw - pw + s;
            if (h < 0 || h >= H || ww < 0 || ww >= W) continue;          /* zero padding: the term is 0 */
            for (int64_t c = 0; c < C; ++c) {
                const double pr = xd[((n * H + h) * W + ww) * C + c] * wd[((f * R + r) * S + s) * C + c];
                acc += pr;
                mag += fabs(pr);
            }
        }
    }
    *y = acc;
    *d = mag;
}

static int conv_decode_copies(int dtype, int64_t nx, int64_t nw, const void *x, const void *w, double **xd, double **wd)
{
    *xd = (double *)malloc((size_t)(nx ? nx : 1) * sizeof(double));
    *wd = (double *)malloc((size_t)(nw ? nw : 1) * sizeof(double));
    if (!*xd || !*wd) { free(*xd); free(*wd); return CONV_ORACLE_NO_MEMORY; }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nx; ++i) (*xd)[i] = conv_load(dtype, x, i);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nw; ++i) (*wd)[i] = conv_load(dtype, w, i);
    return CONV_ORACLE_OK;
}

/*
 * Whole layer.  x, w: host memory in the stored format `dtype` (0 fp32, 1 bf16, 2 fp16, 3 e4m3),
 * dense in the layouts above.  y_ref, D: fp64, N x P x Q x F, either may be NULL.  Returns
 * CONV_ORACLE_OK or an error code; nothing is written on error.
 */
int oracle_conv2d(int dtype, int64_t N, int64_t H, int64_t W, int64_t C, int64_t F, int64_t R, int64_t S,
                  int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                  const void *x, const void *w, double *y_ref, double *D)
{
    int rc = conv_check(dtype, N, H, W, C, F, R, S, stride_h, stride_w, pad_h, pad_w, x, w);
    if (rc != CONV_ORACLE_OK) return rc;
    int64_t P, Q;
    oracle_conv2d_output_size(H, W, R, S, stride_h, stride_w, pad_h, pad_w, &P, &Q);
    if (N == 0 || F == 0) return CONV_ORACLE_OK;
    double *xd, *wd;
    rc = conv_decode_copies(dtype, N * H * W * C, F * R * S * C, x, w, &xd, &wd);
    if (rc != CONV_ORACLE_OK) return rc;
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < N * P * Q; ++pix) {
        const int64_t n = pix / (P * Q), p = (pix / Q) % P, q = pix % Q;
        for (int64_t f = 0; f < F; ++f) {
            double y, d;
            conv_point(xd, wd, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, n, p, q, f, &y, &d);
            if (y_ref) y_ref[pix * F + f] = y;
            if (D) D[pix * F + f] = d;
        }
    }
    free(xd);
    free(wd);
    return CONV_ORACLE_OK;
}

/* Selected outputs (pn[i], pp[i], pq[i], pf[i]), i < npts, by the same loop. */
int oracle_conv2d_points(int dtype, int64_t N, int64_t H, int64_t W, int64_t C, int64_t F, int64_t R, int64_t S,
                         int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                         const void *x, const void *w, int64_t npts,
                         const int64_t *pn, const int64_t *pp, const int64_t *pq, const int64_t *pf,
                         double *y_ref, double *D)
{
    int rc = conv_check(dtype, N, H, W, C, F, R, S, stride_h, stride_w, pad_h, pad_w, x, w);
    if (rc != CONV_ORACLE_OK) return rc;
    int64_t P, Q;
    oracle_conv2d_output_size(H, W, R, S, stride_h, stride_w, pad_h, pad_w, &P, &Q);
    if (npts < 0 || (npts > 0 && (!pn || !pp || !pq || !pf))) return CONV_ORACLE_BAD_ARG;
    for (int64_t i = 0; i < npts; ++i)
        if (pn[i] < 0 || pn[i] >= N || pp[i] < 0 || pp[i] >= P || pq[i] < 0 || pq[i] >= Q || pf[i] < 0 || pf[i] >= F)
            return CONV_ORACLE_BAD_ARG;
    double *xd, *wd;
    rc = conv_decode_copies(dtype, N * H * W * C, F * R * S * C, x, w, &xd, &wd);
    if (rc != CONV_ORACLE_OK) return rc;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < npts; ++i) {
        double y, d;
        conv_point(xd, wd, H, W, C, R, S, stride_h, stride_w, pad_h, pad_w, pn[i], pp[i], pq[i], pf[i], &y, &d);
        if (y_ref) y_ref[i] = y;
        if (D) D[i] = d;
    }
    free(xd);
    free(wd);
    return CONV_ORACLE_OK;
}
