/*
 * gemm_lineage.h -- C ABI of the GEMM kernel lineage for AMD Instinct MI355X (gfx950).
 *
 * The library holds one workload, the dense product C = s * (A . B) with fp32
 * accumulation, as an ordered lineage of hand-written kernel states
 *
 *     L = (K0, tau_1, K1, ..., tau_n, K_n = K*)            (paper Sec. 3.1)
 *
 * from a naive kernel to the expert one.  Each state adds one optimisation
 * intent of the paper's Table 1 ("tile / sm_stage", "vectorize_global",
 * "cp.async + pipeline", "mma" + "ldmatrix.swizzle", "templatize"), realised
 * for CDNA4: LDS staging, 16-byte global loads with masked tails, a
 * double-buffered LDS pipeline, wave64 MFMA with a conflict-free LDS operand
 * layout.  Every state can be launched on its own so that the validation gate
 * (compile -> correctness -> profile, Sec. 3.1 / Sec. 4.1) can be applied at
 * every step of the lineage.
 *
 * Conventions for every entry point
 *   - A, B, C, scale_a, scale_b and workspace are DEVICE pointers owned by the
 *     caller; descriptors and query results are HOST memory owned by the caller.
 *   - The library allocates and frees nothing and keeps no state between calls.
 *   - Launches are asynchronous on the given stream; nothing synchronises.
 *   - Errors are returned as gemm_status_t values; no exception crosses the ABI.
 *     Argument, variant, dtype, precondition and workspace errors are found before
 *     anything is launched: C and the workspace are untouched.  GEMM_ERR_LAUNCH comes
 *     from the HIP runtime in the middle of a call that may consist of several
 *     launches (pack + product, product + row remainder, K ranges + their sum):
 *     after it, C and the workspace are unspecified.
 *   - A variant never substitutes another variant (App. B audits submissions for
 *     wrappers around a reference; a state of this lineage is always its own kernel).  When the
 *     fast path of a variant does not apply, either its own documented slow
 *     path runs (and gemm_query names it) or, with GEMM_FLAG_STRICT, the call
 *     is refused with GEMM_ERR_PRECONDITION.
 */
#ifndef GEMM_LINEAGE_H
#define GEMM_LINEAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GEMM_OK = 0,
    GEMM_ERR_BAD_ARG = 1,           /* null pointer, negative size, ld smaller than the extent ... */
    GEMM_ERR_BAD_VARIANT = 2,       /* variant id outside [0, GEMM_VARIANT_COUNT) */
    GEMM_ERR_UNSUPPORTED_DTYPE = 3, /* in/out dtype pair the library does not implement */
    GEMM_ERR_PRECONDITION = 4,      /* a condition the variant relies on does not hold (see gemm_query) */
    GEMM_ERR_WORKSPACE = 5,         /* workspace was lent but is smaller than gemm_query reports, or misaligned */
    GEMM_ERR_LAUNCH = 6             /* the HIP runtime refused the launch */
} gemm_status_t;

/* Storage formats.  bf16/fp16 are 2-byte IEEE-style patterns, GEMM_FP8_E4M3 is the
 * OCP 8-bit E4M3 format (bias 7, max 448, no infinities). */
typedef enum { GEMM_F32 = 0, GEMM_BF16 = 1, GEMM_F16 = 2, GEMM_FP8_E4M3 = 3 } gemm_dtype_t;

/* Row-major: element (r, c) at r*ld + c.  Column-major: at c*ld + r. */
typedef enum { GEMM_ROW_MAJOR = 0, GEMM_COL_MAJOR = 1 } gemm_layout_t;

/* The lineage, in forward order (Sec. 3.1, Table 1). */
typedef enum {
    GEMM_K0_NAIVE = 0,      /* one thread per output element, operands read from global memory */
    GEMM_K1_LDS_TILED = 1,  /* + "tile / sm_stage": workgroup output tiles, K slabs staged through LDS */
    GEMM_K2_VECTORIZED = 2, /* + "vectorize_global": 16-byte global loads, element-masked tails */
    GEMM_K3_PIPELINED = 3,  /* + "cp.async + pipeline": slabs travel global -> LDS without registers, three stages deep
                               (operands kept in storage format, decoded on read); where that form's conditions
                               fail, two LDS buffers with the next slab fetched through registers */
    GEMM_K4_MFMA = 4,       /* + "mma" / "swizzle": wave64 MFMA, swizzled LDS operand layout (fp32: its masked kernel only) */
    GEMM_VARIANT_COUNT = 5
} gemm_variant_t;

/* Conditions a variant may rely on: one bit per entry of Table 1's precondition column as it
 * applies to this product on gfx950 (Sec. 1 names the same three families: access width,
 * staging, matrix-instruction shape). */
enum {
    GEMM_COND_ALIGN16_A      = 1u << 0,  /* base pointer of A (incl. batch stride) is 16-byte aligned */
    GEMM_COND_ALIGN16_B      = 1u << 1,
    GEMM_COND_ALIGN16_C      = 1u << 2,
    GEMM_COND_LD16_A         = 1u << 3,  /* lda * element size is a multiple of 16 bytes */
    GEMM_COND_LD16_B         = 1u << 4,
    GEMM_COND_LD16_C         = 1u << 5,
    GEMM_COND_TILE_DIV_M     = 1u << 6,  /* M is a multiple of the variant's BM */
    GEMM_COND_TILE_DIV_N     = 1u << 7,
    GEMM_COND_TILE_DIV_K     = 1u << 8,
    GEMM_COND_K_CONTIG_A     = 1u << 9,  /* A stored with K contiguous (row-major) */
    GEMM_COND_K_CONTIG_B     = 1u << 10, /* B stored with K contiguous (column-major) */
    GEMM_COND_DTYPE_HAS_MFMA = 1u << 11, /* the input dtype has a matrix instruction on gfx950 (all four do) */
    GEMM_COND_LDS_STAGED     = 1u << 12, /* operands pass through LDS (holds from K1 on) */
    GEMM_COND_SMALL_M        = 1u << 13  /* M <= 96: few enough rows for K4's streaming (bandwidth-bound) kernel */
};

enum {
    GEMM_FLAG_STRICT = 1u << 0, /* refuse (GEMM_ERR_PRECONDITION) instead of taking a variant's slow path */
    /* Edges of the backward walk from the expert state (Sec. 3.2): each switches one optimisation of
     * K4's fast kernel off, and the result goes through the gate like any state.  On any other variant
     * or path they are refused with GEMM_ERR_BAD_ARG.  Same result, slower: the latency difference is
     * the evidence for what the optimisation buys. */
    GEMM_FLAG_DEOPT_NO_SWIZZLE = 1u << 1, /* LDS operand rows unswizzled: fragment reads conflict on banks */
    GEMM_FLAG_DEOPT_NO_OVERLAP = 1u << 2, /* loads waited for at once: nothing in flight under the MFMAs */
    /* Tile override for K4's fast kernel (Table 1 "autotune": the sweep that froze the default choice
     * needs both).  Default: 256 x 256 tiles, 128 x 128 when 256-tiles would not fill the CUs once.
     * At most one of the two; refused with GEMM_ERR_BAD_ARG on other variants or paths. */
    GEMM_FLAG_TILE_256 = 1u << 3,
    GEMM_FLAG_TILE_128 = 1u << 4,
    /* Two more validated simplifications, so that the backward walk from the expert state (Sec. 3.2;
     * the paper's deoptimisation traces remove "L2 raster", "swizzle", "vec. load" one at a time) has an
     * edge for each of them. */
    GEMM_FLAG_DEOPT_NO_RASTER = 1u << 5, /* K4's fast kernel only: workgroup i takes tile i in row-major order
                                            instead of the XCD-aware banded walk */
    GEMM_FLAG_DEOPT_NO_VECTOR = 1u << 6, /* K2 and K3 only: slabs fetched element by element (K3 with it is
                                            "pipeline without vectorised loads", an order the lineage skips) */
    GEMM_FLAG_DEOPT_NO_PERSISTENT = 1u << 7, /* K4's fast kernel only: one workgroup per tile (ring filled from a cold
                                            start and drained per tile) where the default would keep one workgroup per
                                            CU walking several tiles with the ring running across their boundaries */
    /* Configuration override for K4's streaming kernel (Table 1 "autotune" over the "templatize"d configuration:
     * waves per workgroup x columns per strip x K tile x row groups).  Bits 8..10 hold 1 + the form:
     *   0: 1 wave x 16 columns x 512-byte runs, 16 rows     1: 4 waves x 16 x 512 B, 16 rows (K tiles dealt to the waves)
     *   2: 2 waves x 32 x 512 B, 32 rows    3 / 4 / 5: 4 waves x 64 columns x 256-byte runs, 48 / 64 / 96 rows
     * Only on the streaming path and only a form with at least the product's rows (of the transposed product on the
     * small-N path); otherwise GEMM_ERR_BAD_ARG.  0 in these bits: the frozen rule chooses. */
    GEMM_FLAG_STREAM_FORM_SHIFT = 8,
    GEMM_FLAG_STREAM_FORM_MASK = 7u << 8,
    /* Instruction override for K4's fast kernel (a sweep point of Table 1 "autotune", and an edge of the backward
     * walk): bf16 / fp16 products on 256 x 256 tiles with one tile per workgroup multiply with v_mfma_f32_16x16x32
     * (8 x 8 accumulator tiles per wave: less accumulator traffic per flop, a higher clock under the power limit);
     * with this bit they use v_mfma_f32_32x32x16 (4 x 4 tiles), as every other form of the kernel does.  Accepted
     * where the other fast-kernel switches are; no effect on forms that use 32x32 already. */
    GEMM_FLAG_MFMA_32X32 = 1u << 11
};
#define GEMM_FLAG_STREAM_FORM(form) ((uint32_t)((form) + 1) << GEMM_FLAG_STREAM_FORM_SHIFT)

typedef struct {
    int64_t M, N, K;                 /* logical sizes: A is M x K, B is K x N, C is M x N; >= 0 */
    int64_t batch;                   /* number of independent problems, >= 1 */
    int32_t in_dtype, out_dtype;     /* gemm_dtype_t; accumulation is always fp32 */
    int32_t layout_a, layout_b;      /* gemm_layout_t; C is always row-major */
    int64_t lda, ldb, ldc;           /* leading dimensions, in elements */
    int64_t stride_a, stride_b, stride_c; /* elements between consecutive batch items */
    const float *scale_a, *scale_b;  /* device: one fp32 per batch item each, or NULL (= 1).  The
                                        epilogue multiplies the fp32 accumulator by scale_a[b]*scale_b[b]
                                        before rounding to out_dtype (round to nearest even). */
    const float *bias;               /* device: N fp32 values or NULL.  C[b,i,j] = round(s_b * acc + bias[j]):
                                        the "AddMM" shape of the paper's held-out GEMM family (App. D),
                                        fused into every state's epilogue; shared by all batch items. */
    void *workspace;                 /* optional device scratch lent by the caller (16-byte aligned), or NULL.
                                        Only K4 uses it, in two cases.  (1) Its fast path's conditions fail:
                                        with scratch of at least gemm_query's workspace_bytes it packs the
                                        operands (K contiguous, aligned, zero-padded K; an operand that meets
                                        the conditions by itself is used in place when K is whole slabs) and
                                        runs the fast kernel on the copies; without scratch a product with A and
                                        B row-major and at least 256 tiles of 256 x 256 (bf16, fp16) is multiplied
                                        in place by the persistent kernel (gemm_query names the path), any other
                                        by the masked kernel.  (2) The
                                        fast path applies but the product has too few tiles to fill the chip
                                        and a long K (batch 1, 17 or more rows): with scratch it splits K into
                                        ranges that run side by side and adds their fp32 partial products in a
                                        second pass; without scratch the unsplit kernel runs.  Scratch that is
                                        lent but too small or misaligned is an error (GEMM_ERR_WORKSPACE), never
                                        a silent slow path.  Contents after the call are unspecified. */
    size_t workspace_bytes;
    void *stream;                    /* hipStream_t; NULL = the default stream */
    uint32_t flags;                  /* GEMM_FLAG_* */
    uint32_t reserved;               /* must be 0 */
} gemm_desc_t;

typedef struct {
    uint32_t required;        /* conditions the variant's fast path relies on for this dtype */
    uint32_t violated;        /* subset of `required` that does not hold for this call */
    uint32_t holds;           /* every GEMM_COND_* bit that holds for this call */
    int32_t  bm, bn, bk;      /* workgroup tile (0 where meaningless) */
    int32_t  threads;         /* workgroup size */
    int32_t  stages;          /* LDS buffers in flight */
    int32_t  lds_bytes;       /* static + dynamic LDS per workgroup */
    int64_t  grid;            /* workgroups launched */
    size_t   workspace_bytes; /* scratch the packed or split-K path of K4 uses for this call (0: no path would use any) */
    char     path[64];        /* name of the code path gemm_run_ex would take */
} gemm_query_t;

/*
 * gemm_run: one validated state of the lineage L = (K0, ..., K*) of Sec. 3.1 applied to one product,
 * short form.  Batch 1, tight
 * leading dimensions, output dtype = input dtype (bf16 for fp8 input), no scales, default
 * stream, layouts A row-major and B row-major for GEMM_F32/GEMM_F16, A row-major and B
 * column-major (K contiguous) for GEMM_BF16/GEMM_FP8_E4M3.
 */
int gemm_run(int variant, int64_t M, int64_t N, int64_t K, int dtype,
             const void *A, const void *B, void *C);

/* gemm_run_ex: full form of the same (Sec. 3.1: the state the gate compiles, checks and profiles; Table 1:
 * the conditions it checks).  Validates, checks the variant's conditions, launches on d->stream. */
int gemm_run_ex(int variant, const gemm_desc_t *d, const void *A, const void *B, void *C);

/*
 * gemm_run_static: gemm_run_ex for callers that cannot allocate device memory and have none to lend:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * checks, paths, kernels and results as gemm_run_ex, except that d->workspace must be NULL and
 * d->workspace_bytes 0 (else GEMM_ERR_BAD_ARG): where K4's packed or split-K path wants scratch, it
 * uses a fixed array of GEMM_STATIC_SCRATCH_BYTES that is part of the loaded library (each GPU the
 * library runs on holds its own copy until the process ends).  A call whose path wants more than
 * that is refused with GEMM_ERR_WORKSPACE before anything is launched (gemm_query with a non-NULL
 * workspace reports the size a call wants).  The call allocates and frees nothing.  Its very first
 * call on a device looks the array's address up (once; outside graph capture).  All calls on one GPU
 * share the array, whose contents are unspecified between calls (every path writes what it reads, so
 * nothing needs clearing): calls that use it and overlap on one GPU -- different streams, or threads
 * -- race; order them on one stream.
 */
#define GEMM_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int gemm_run_static(int variant, const gemm_desc_t *d, const void *A, const void *B, void *C);
size_t gemm_static_scratch_bytes(void);

/* gemm_query: host only, launches nothing.  The deterministic part of a skill record's `pre` field
 * (Sec. 3.1) for this call.  Reports which conditions the variant relies on,
 * which of them this call violates, the path that would run and its launch geometry.  A, B, C
 * may be NULL (then the ALIGN16 conditions are reported as holding).  Returns the status
 * gemm_run_ex would return before launching. */
int gemm_query(int variant, const gemm_desc_t *d, const void *A, const void *B, const void *C,
               gemm_query_t *out);

/* gemm_default_desc: fills *d with the defaults gemm_run uses for (M, N, K, dtype). */
int gemm_default_desc(gemm_desc_t *d, int64_t M, int64_t N, int64_t K, int dtype);

/*
 * Measurement probes (not part of the lineage, never used by gemm_run*).  The gate's profile leg
 * (Sec. 3.1) reads a kernel's time against a ceiling; these three plain kernels measure, on the GPU at
 * hand, the ceilings the published peaks only bound from above.  All pointers are device pointers,
 * 16-byte aligned; byte counts are multiples of 16; launches are asynchronous on `stream`.
 *   gemm_probe_copy         dst[0..bytes) = src[0..bytes): reads and writes exactly `bytes` each; the
 *                           unit for calibrating HBM byte counters
 *   gemm_probe_stream_read  reads src[0..bytes) once with 16-byte loads; sink: >= 4 bytes
 *   gemm_probe_mfma         `workgroups` x 4 waves each issue iters x 32 matrix instructions of the
 *                           expert kernel (bf16/fp16: 32x32x16; e4m3: scaled 32x32x64) on fragments
 *                           read once from `operands` (>= gemm_probe_mfma_operand_bytes bytes, any
 *                           finite values of the dtype); *flops receives the flop count of the launch;
 *                           sink: workgroups*256 floats.  Errors: GEMM_ERR_BAD_ARG,
 *                           GEMM_ERR_UNSUPPORTED_DTYPE (fp32), GEMM_ERR_LAUNCH.
 *   gemm_probe_mfma16       the same for the 16x16x32 instruction the expert kernel uses for bf16 / fp16 on
 *                           256 x 256 tiles: iters x 128 instructions per wave (the flops of 2 x iters of
 *                           the loop above) on 2 x gemm_probe_mfma_operand_bytes bytes; bf16 and fp16 only.
 */
int gemm_probe_copy(void *dst, const void *src, size_t bytes, void *stream);
int gemm_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream);
size_t gemm_probe_mfma_operand_bytes(int dtype, int workgroups);
int gemm_probe_mfma(int dtype, const void *operands, size_t operand_bytes, int workgroups, int iters,
                    void *sink, size_t sink_bytes, double *flops, void *stream);
int gemm_probe_mfma16(int dtype, const void *operands, size_t operand_bytes, int workgroups, int iters,
                      void *sink, size_t sink_bytes, double *flops, void *stream);

const char *gemm_status_string(int status);
/* The HIP runtime's message for the calling thread's most recent GEMM_ERR_LAUNCH ("no error" if none). */
const char *gemm_last_launch_error(void);
const char *gemm_variant_name(int variant);
const char *gemm_variant_intent(int variant); /* Table 1 intent the transition into this state adds */
const char *gemm_cond_name(uint32_t single_bit);
int gemm_variant_count(void);
int gemm_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_LINEAGE_H */
