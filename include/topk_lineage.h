/*
 * topk_lineage.h -- C ABI of row-wise top-k selection (AMD Instinct MI355X, gfx950).
 *
 * The paper's selection workload (Sec. 4.1, workload table: Top-K, batch 64, sequence 4096, k = 512,
 * FP32) reaches its expert state by one algorithmic step, from selection sort to radix select
 * (Sec. 4.2; Table 1 lists `radix_select` with the carrier "coarse + refine pass").  Three states:
 *
 *     T0 selection        k rounds of a workgroup-wide arg-max over the not yet taken elements
 *     T1 radix select     the k-th largest key by four 8-bit histogram passes over the row (most
 *                         significant digit first), then one ordered compaction pass
 *     T2 resident coarse + refine   the row's keys stay in registers (one load); an 11-bit coarse
 *                         histogram finds the threshold's bin, two refine passes (11 + 10 bits) over
 *                         the candidates in that bin finish it; compaction from the registers
 *
 * Definition.  Element i precedes element j when x[i] > x[j], or x[i] == x[j] and i < j (-0.0 and
 * +0.0 tie).  The selection of a row is the set of the k elements that fewer than k others precede:
 * the k largest, ties at the threshold resolved towards lower indices.  idx[b][0..k) lists it in
 * increasing index order and val[b][t] = x[b][idx[b][t]] bit for bit.  Rows holding NaN give an
 * unspecified (but memory-safe) selection.
 *
 * Conventions as in gemm_lineage.h: x, idx, val are DEVICE pointers owned by the caller; descriptors
 * and query results are HOST memory; nothing is allocated, no state is kept; launches are asynchronous
 * on the given stream; errors are gemm_status_t values; on any status other than GEMM_OK nothing was
 * launched; a state whose conditions do not hold is refused with GEMM_ERR_PRECONDITION.
 */
#ifndef TOPK_LINEAGE_H
#define TOPK_LINEAGE_H

#include "gemm_lineage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TOPK_T0_SELECTION = 0,
    TOPK_T1_RADIX_SELECT = 1,
    TOPK_T2_RESIDENT = 2,
    TOPK_VARIANT_COUNT = 3
} topk_variant_t;

enum {
    TOPK_COND_ROW_IN_LDS       = 1u << 0, /* n <= 65536: T0 keeps one "taken" byte per element in LDS */
    TOPK_COND_ROW_IN_REGISTERS = 1u << 1, /* n <= 16384: T2 holds 4 or 16 keys per lane of a 1024-lane workgroup */
    TOPK_COND_ALIGN16          = 1u << 2  /* x 16-byte aligned and ld a multiple of 4: T2 loads 16 bytes per lane */
};

typedef struct {
    int64_t batch;      /* rows, >= 0 */
    int64_t n;          /* elements per row, 0 <= n < 2^31 */
    int64_t k;          /* 0 <= k <= n */
    int64_t ld;         /* elements between consecutive rows, >= n */
    void *stream;       /* hipStream_t; NULL = the default stream */
    uint32_t flags;     /* must be 0 */
    uint32_t reserved;  /* must be 0 */
} topk_desc_t;

typedef struct {
    uint32_t required, violated, holds; /* TOPK_COND_* */
    int32_t  threads;                   /* workgroup size; one workgroup per row */
    int32_t  passes;                    /* passes over the row's keys (histogram passes + compaction; k rounds for T0) */
    int32_t  lds_bytes;
    int64_t  grid;
    char     path[64];
} topk_query_t;

/* topk_run: idx is batch x k int32, val is batch x k fp32, both dense. */
int topk_run(int variant, const topk_desc_t *d, const float *x, int32_t *idx, float *val);

/* topk_query: host only, launches nothing; x may be NULL (then ALIGN16 is reported as holding for the
 * pointer).  Returns the status topk_run would return before launching. */
int topk_query(int variant, const topk_desc_t *d, const float *x, topk_query_t *out);

const char *topk_last_launch_error(void);
const char *topk_variant_name(int variant);
const char *topk_variant_intent(int variant);
const char *topk_cond_name(uint32_t single_bit);
int topk_variant_count(void);

#ifdef __cplusplus
}
#endif
#endif /* TOPK_LINEAGE_H */
