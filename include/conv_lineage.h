/*
 * conv_lineage.h -- C ABI of the convolution layer built on the GEMM lineage's expert state
 * (AMD Instinct MI355X, gfx950).
 *
 * The paper's second workload (Sec. 4.1, workload table: Conv2d, N=8, C=64, H=W=56, F=128, 3x3,
 * stride 1, padding 1, FP16) reaches its expert state along "im2col + tensor core" (Sec. 4.2); a
 * matrix intrinsic without staging, swizzle and pipelining stays 5-14x behind (Sec. 4.4, generated-only
 * ablation).  Here the layer is a short lineage of three states, the last two on the GEMM lineage's
 * K4 kernel:
 *
 *     C0 direct          one thread per output, seven nested loops
 *     C1 im2col + MFMA   the patches are written out as a matrix (caller-lent scratch), then K4's
 *                        direct-to-LDS MFMA kernel multiplies it with the filters
 *     C2 implicit MFMA   the same kernel gathers the patches itself: K slab s of output pixel m is the
 *                        128 contiguous bytes of channels at input pixel (p*stride - pad + r, q*stride
 *                        - pad + s); taps that fall into the padding are fetched out of range of the
 *                        buffer resource and arrive in LDS as zeros.  No scratch, no extra pass.
 *
 * Definition (cross-correlation, filter not flipped, zero padding):
 *     y[n,p,q,f] = round_out( sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] * w[f,r,s,c] + bias[f] )
 *     P = (H + 2 pad_h - R) / stride_h + 1,  Q = (W + 2 pad_w - S) / stride_w + 1,  fp32 accumulation.
 * Layouts (dense, channels fastest): x is N x H x W x C, w is F x R x S x C, y is N x P x Q x F.
 *
 * Conventions as in gemm_lineage.h: x, w, y, bias and workspace are DEVICE pointers owned by the
 * caller; descriptors and query results are HOST memory; the library allocates nothing and keeps no
 * state; launches are asynchronous on the given stream; errors are gemm_status_t values; on any
 * status other than GEMM_OK nothing was launched and y is untouched; no state substitutes another:
 * a state whose conditions do not hold is refused with GEMM_ERR_PRECONDITION (C2) or
 * GEMM_ERR_WORKSPACE (C1 without scratch).
 */
#ifndef CONV_LINEAGE_H
#define CONV_LINEAGE_H

#include "gemm_lineage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CONV_C0_DIRECT = 0,        /* any dtype of gemm_dtype_t */
    CONV_C1_IM2COL_MFMA = 1,   /* + "im2col" and the GEMM lineage's expert state; bf16, fp16, e4m3 */
    CONV_C2_IMPLICIT_MFMA = 2, /* + gather fused into the direct-to-LDS loader; bf16, fp16, e4m3 */
    CONV_VARIANT_COUNT = 3
} conv2d_variant_t;

/* Conditions a state may rely on. */
enum {
    CONV_COND_ALIGN16_X      = 1u << 0, /* x is 16-byte aligned */
    CONV_COND_ALIGN16_W      = 1u << 1,
    CONV_COND_ALIGN16_Y      = 1u << 2,
    CONV_COND_C_WHOLE_SLABS  = 1u << 3, /* C * element size is a multiple of 128 bytes: a K slab never straddles two taps */
    CONV_COND_DTYPE_ON_FAST_KERNEL = 1u << 4, /* bf16, fp16 or e4m3: the types K4's direct-to-LDS kernel is built for (fp32 runs on C0 only) */
    CONV_COND_X_BELOW_2GIB   = 1u << 5, /* x spans less than 2^31 bytes: the gather uses 32-bit byte offsets */
    CONV_COND_SCRATCH_LENT   = 1u << 6  /* workspace of at least conv2d_query's workspace_bytes, 16-byte aligned */
};

typedef struct {
    int64_t N, H, W, C;              /* activations: images, height, width, channels; N >= 0, others >= 1 */
    int64_t F, R, S;                 /* filters: count (>= 0), height, width (>= 1) */
    int32_t stride_h, stride_w;      /* >= 1 */
    int32_t pad_h, pad_w;            /* >= 0, zero padding on both sides; H + 2 pad_h >= R, W + 2 pad_w >= S */
    int32_t in_dtype, out_dtype;     /* gemm_dtype_t; pairs as in gemm_desc_t; accumulation is fp32 */
    const float *bias;               /* device: F fp32 values or NULL */
    void *workspace;                 /* device scratch lent by the caller (C1 only), or NULL */
    size_t workspace_bytes;
    void *stream;                    /* hipStream_t; NULL = the default stream */
    uint32_t flags;                  /* must be 0 */
    uint32_t reserved;               /* must be 0 */
} conv2d_desc_t;

typedef struct {
    uint32_t required;        /* conditions the state relies on */
    uint32_t violated;        /* subset of `required` that does not hold for this call */
    uint32_t holds;           /* every CONV_COND_* bit that holds for this call */
    int64_t  P, Q;            /* output height and width */
    int64_t  gemm_m, gemm_n, gemm_k; /* the matrix product the layer is lowered to: N*P*Q x F x R*S*C */
    int32_t  bm, bn, bk;      /* workgroup tile of the kernel that multiplies (0 for C0) */
    int32_t  threads;
    int32_t  lds_bytes;
    int64_t  grid;            /* workgroups of the multiplying kernel (of the only kernel for C0) */
    size_t   workspace_bytes; /* scratch C1 needs for this call (0 for the other states) */
    char     path[64];
} conv2d_query_t;

/* conv2d_run: validates, checks the state's conditions, launches on d->stream. */
int conv2d_run(int variant, const conv2d_desc_t *d, const void *x, const void *w, void *y);

/* conv2d_query: host only, launches nothing; x, w, y may be NULL (then the ALIGN16 conditions are
 * reported as holding).  Returns the status conv2d_run would return before launching. */
int conv2d_query(int variant, const conv2d_desc_t *d, const void *x, const void *w, const void *y,
                 conv2d_query_t *out);

/* conv2d_default_desc: the paper's layer geometry for the given sizes (stride 1, padding R/2, S/2,
 * out dtype = in dtype, bf16 for e4m3). */
int conv2d_default_desc(conv2d_desc_t *d, int64_t N, int64_t H, int64_t W, int64_t C, int64_t F,
                        int64_t R, int64_t S, int dtype);

/* The HIP runtime's message for the calling thread's most recent GEMM_ERR_LAUNCH from conv2d_run. */
const char *conv2d_last_launch_error(void);
const char *conv2d_variant_name(int variant);
const char *conv2d_variant_intent(int variant);
const char *conv2d_cond_name(uint32_t single_bit);
int conv2d_variant_count(void);

#ifdef __cplusplus
}
#endif
#endif /* CONV_LINEAGE_H */
