/*
 * gemm_oracle.c -- CPU reference for C = s * (A . B), accumulated in IEEE fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the validation gate's
 * correctness leg compares GPU kernels against (paper Sec. 3.1: a candidate is
 * accepted only after compile / correctness / profile; Sec. 4.1 "Platforms and
 * protocol": correctness is verified at three random seeds).  It shares no code
 * with the HIP library and must never be linked, imported or called from it.
 *
 * What it computes, for each batch item b and each output (i, j):
 *
 *     C_ref[b,i,j] = s_b * sum_{k=0..K-1} dec(A[b,i,k]) * dec(B[b,k,j])
 *     D[b,i,j]     = |s_b| * sum_k |dec(A[b,i,k])| * |dec(B[b,k,j])|
 *
 * where dec() maps a stored bit pattern (fp32, bf16, fp16, OCP e4m3) to the
 * real number it encodes, s_b = scale_a[b]*scale_b[b] (1 when absent) and every
 * product and sum is an fp64 operation taken in increasing k.  Products of two
 * <=24-bit significands are exact in fp64.  D is the denominator of the
 * normalised error  max |C - C_ref| / D  used as the acceptance metric.
 *
 * The paper never defines a GEMM oracle (it says "correctness" only), so this
 * is the textbook definition of the matrix product written out as a triple
 * loop; nothing is blocked, fused or reordered.  Threads split independent
 * output rows only.
 *
 * Pins (tests/test_oracle_pins.py): decode tables against numpy/torch dtype
 * conversions and the OCP FP8 spec's named values; identity, all-ones == K,
 * rank-1 outer products, integer-valued exactness, exact rational brute force
 * on tiny shapes, transpose/permutation/power-of-two-scaling identities.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2, ORACLE_E4M3 = 3 };
enum { ORACLE_ROW_MAJOR = 0, ORACLE_COL_MAJOR = 1 };
enum { ORACLE_OK = 0, ORACLE_BAD_ARG = 1, ORACLE_NO_MEMORY = 2 };

/* Generic IEEE-style binary decode: 1 sign bit, ebits exponent bits with the
 * given bias, mbits fraction bits.  Normal: (-1)^s 2^(e-bias) (1 + m/2^mbits);
 * subnormal (e==0): (-1)^s 2^(1-bias) m/2^mbits.  The caller handles the
 * format's special codes (Inf/NaN) before calling. */
static double decode_fields(uint32_t sign, uint32_t e, uint32_t m, int bias, int mbits)
{
    double mag;
    if (e == 0)
        mag = ldexp((double)m, 1 - bias - mbits);
    else
        mag = ldexp((double)((1u << mbits) + m), (int)e - bias - mbits);
    return sign ? -mag : mag;
}

/* Bit pattern -> real value.  Non-finite codes decode to NaN / +-Inf. */
double oracle_decode(int dtype, uint32_t code)
{
    switch (dtype) {
    case ORACLE_F32: {
        uint32_t s = code >> 31, e = (code >> 23) & 0xFFu, m = code & 0x7FFFFFu;
        if (e == 0xFFu) return m ? NAN : (s ? -INFINITY : INFINITY);
        return decode_fields(s, e, m, 127, 23);
    }
    case ORACLE_BF16: {
        uint32_t c = code & 0xFFFFu;
        uint32_t s = c >> 15, e = (c >> 7) & 0xFFu, m = c & 0x7Fu;
        if (e == 0xFFu) return m ? NAN : (s ? -INFINITY : INFINITY);
        return decode_fields(s, e, m, 127, 7);
    }
    case ORACLE_F16: {
        uint32_t c = code & 0xFFFFu;
        uint32_t s = c >> 15, e = (c >> 10) & 0x1Fu, m = c & 0x3FFu;
        if (e == 0x1Fu) return m ? NAN : (s ? -INFINITY : INFINITY);
        return decode_fields(s, e, m, 15, 10);
    }
    case ORACLE_E4M3: {
        /* OCP 8-bit float E4M3: bias 7, no infinities, the all-ones magnitude
         * (S.1111.111) is NaN, every other code is finite; max finite 448. */
        uint32_t c = code & 0xFFu;
        uint32_t s = c >> 7, e = (c >> 3) & 0xFu, m = c & 0x7u;
        if (e == 0xFu && m == 0x7u) return NAN;
        return decode_fields(s, e, m, 7, 3);
    }
    default:
        return NAN;
    }
}

static int elem_bytes(int dtype)
{
    switch (dtype) {
    case ORACLE_F32: return 4;
    case ORACLE_BF16: return 2;
    case ORACLE_F16: return 2;
    case ORACLE_E4M3: return 1;
    default: return 0;
    }
}

static double load_elem(int dtype, const void *base, int64_t idx)
{
    switch (dtype) {
    case ORACLE_F32: {
        uint32_t c; memcpy(&c, (const unsigned char *)base + 4 * idx, 4);
        return oracle_decode(dtype, c);
    }
    case ORACLE_BF16:
    case ORACLE_F16: {
        uint16_t c; memcpy(&c, (const unsigned char *)base + 2 * idx, 2);
        return oracle_decode(dtype, c);
    }
    default:
        return oracle_decode(dtype, ((const unsigned char *)base)[idx]);
    }
}

/* Element (r, c) of a matrix with leading dimension ld: row-major stores row r
 * contiguously, column-major stores column c contiguously. */
static int64_t mat_index(int layout, int64_t r, int64_t c, int64_t ld)
{
    return layout == ORACLE_ROW_MAJOR ? r * ld + c : c * ld + r;
}

static int check_args(int dtype, int layout_a, int layout_b, int64_t M, int64_t N, int64_t K,
                      int64_t batch, const void *A, int64_t lda, const void *B, int64_t ldb)
{
    if (elem_bytes(dtype) == 0) return ORACLE_BAD_ARG;
    if ((layout_a != 0 && layout_a != 1) || (layout_b != 0 && layout_b != 1)) return ORACLE_BAD_ARG;
    if (M < 0 || N < 0 || K < 0 || batch < 0) return ORACLE_BAD_ARG;
    if (M > 0 && K > 0 && !A) return ORACLE_BAD_ARG;
    if (N > 0 && K > 0 && !B) return ORACLE_BAD_ARG;
    if (lda < (layout_a == ORACLE_ROW_MAJOR ? K : M)) return ORACLE_BAD_ARG;
    if (ldb < (layout_b == ORACLE_ROW_MAJOR ? N : K)) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

static double batch_scale(const float *scale_a, const float *scale_b, int64_t b)
{
    double s = 1.0;
    if (scale_a) s *= (double)scale_a[b];
    if (scale_b) s *= (double)scale_b[b];
    return s;
}

/*
 * Full product.  A is M x K, B is K x N (logical shapes; storage per layout
 * flag and leading dimension, in elements; batch items stride_* elements
 * apart).  C_ref and D are row-major fp64 with leading dimension ldc and batch
 * stride stride_c; either may be NULL.  All pointers are host memory owned by
 * the caller.  Returns ORACLE_OK or an error code; nothing is written on error.
 */
int oracle_gemm(int dtype, int layout_a, int layout_b,
                int64_t M, int64_t N, int64_t K, int64_t batch,
                const void *A, int64_t lda, int64_t stride_a,
                const void *B, int64_t ldb, int64_t stride_b,
                const float *scale_a, const float *scale_b,
                double *C_ref, double *D, int64_t ldc, int64_t stride_c)
{
    int rc = check_args(dtype, layout_a, layout_b, M, N, K, batch, A, lda, B, ldb);
    if (rc != ORACLE_OK) return rc;
    if (ldc < N) return ORACLE_BAD_ARG;
    if (M == 0 || N == 0 || batch == 0) return ORACLE_OK;

    /* Decoded copies: Ad[i][k] and Bd[j][k], both with k contiguous.  This is a
     * change of storage only; the arithmetic below is the definition. */
    size_t na = (size_t)M * (size_t)(K ? K : 1), nb = (size_t)N * (size_t)(K ? K : 1);
    double *Ad = (double *)malloc(na * sizeof(double));
    double *Bd = (double *)malloc(nb * sizeof(double));
    if (!Ad || !Bd) { free(Ad); free(Bd); return ORACLE_NO_MEMORY; }

    for (int64_t b = 0; b < batch; ++b) {
        const unsigned char *Ab = (const unsigned char *)A + (size_t)elem_bytes(dtype) * (size_t)(b * stride_a);
        const unsigned char *Bb = (const unsigned char *)B + (size_t)elem_bytes(dtype) * (size_t)(b * stride_b);
        const double s = batch_scale(scale_a, scale_b, b);

#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t k = 0; k < K; ++k)
                Ad[i * K + k] = load_elem(dtype, Ab, mat_index(layout_a, i, k, lda));
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < N; ++j)
            for (int64_t k = 0; k < K; ++k)
                Bd[j * K + k] = load_elem(dtype, Bb, mat_index(layout_b, k, j, ldb));

#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < M; ++i) {
            for (int64_t j = 0; j < N; ++j) {
                double acc = 0.0, mag = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double p = Ad[i * K + k] * Bd[j * K + k];
                    acc += p;
                    mag += fabs(p);
                }
                if (C_ref) C_ref[b * stride_c + i * ldc + j] = s * acc;
                if (D) D[b * stride_c + i * ldc + j] = fabs(s) * mag;
            }
        }
    }
    free(Ad);
    free(Bd);
    return ORACLE_OK;
}

/*
 * Selected outputs of the same product: for p in [0, n) the entry
 * (pb[p], pi[p], pj[p]) is evaluated straight from the stored inputs with the
 * same fp64 loop.  Used where the full product is too large to finish in
 * seconds.  C_ref[p], D[p] are written per point.
 */
int oracle_gemm_points(int dtype, int layout_a, int layout_b,
                       int64_t M, int64_t N, int64_t K, int64_t batch,
                       const void *A, int64_t lda, int64_t stride_a,
                       const void *B, int64_t ldb, int64_t stride_b,
                       const float *scale_a, const float *scale_b,
                       int64_t n, const int64_t *pb, const int64_t *pi, const int64_t *pj,
                       double *C_ref, double *D)
{
    int rc = check_args(dtype, layout_a, layout_b, M, N, K, batch, A, lda, B, ldb);
    if (rc != ORACLE_OK) return rc;
    if (n < 0 || (n > 0 && (!pb || !pi || !pj))) return ORACLE_BAD_ARG;
    for (int64_t p = 0; p < n; ++p)
        if (pb[p] < 0 || pb[p] >= batch || pi[p] < 0 || pi[p] >= M || pj[p] < 0 || pj[p] >= N)
            return ORACLE_BAD_ARG;

#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t p = 0; p < n; ++p) {
        const int64_t b = pb[p], i = pi[p], j = pj[p];
        const unsigned char *Ab = (const unsigned char *)A + (size_t)elem_bytes(dtype) * (size_t)(b * stride_a);
        const unsigned char *Bb = (const unsigned char *)B + (size_t)elem_bytes(dtype) * (size_t)(b * stride_b);
        const double s = batch_scale(scale_a, scale_b, b);
        double acc = 0.0, mag = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = load_elem(dtype, Ab, mat_index(layout_a, i, k, lda));
            double bv = load_elem(dtype, Bb, mat_index(layout_b, k, j, ldb));
            double pr = a * bv;
            acc += pr;
            mag += fabs(pr);
        }
        if (C_ref) C_ref[p] = s * acc;
        if (D) D[p] = fabs(s) * mag;
    }
    return ORACLE_OK;
}

/* Number of threads the loops above will use (1 without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
