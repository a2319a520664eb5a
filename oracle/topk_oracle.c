/*
 * topk_oracle.c -- CPU reference for row-wise top-k selection of fp32 values.
 *
 * TEST INFRASTRUCTURE ONLY.  The yardstick for the correctness leg of the validation gate (paper
 * Sec. 3.1; Sec. 4.1 workload table: Top-K, batch 64, sequence 4096, k = 512, FP32) applied to the
 * selection kernels of the HIP library.  Shares no code with that library.
 *
 * Definition.  For a row x[0..n) and 0 <= k <= n, element i "precedes" element j when
 * x[i] > x[j], or x[i] == x[j] and i < j (so -0.0 and +0.0 tie and the lower index wins).  The
 * rank of i is the number of elements that precede it; the selection is { i : rank(i) < k }: the k
 * largest values, ties at the threshold resolved towards lower indices.  That set is unique.  The
 * output lists it in increasing index order: idx[0..k) and val[t] = x[idx[t]].
 *
 * The paper says "top-k" and names the shape only; ordering of the output and the tie rule are
 * this repository's reading (a set has no order; increasing index is the order a stable compaction
 * produces).  The implementation is the definition itself, a rank count per element in O(n^2): no
 * sort, no partition, no histogram, nothing a selection algorithm could get wrong in the same way.
 * Inputs must be free of NaN (rejected).
 *
 * Pins (tests/test_topk_oracle_pins.py): ramps and constant rows in closed form, k = 0 / 1 / n,
 * signed zeros, numpy's stable argsort, torch.topk's values, exhaustive comparison against a
 * sort-based brute force on all short rows over a small alphabet.
 */
#include <math.h>
#include <stdint.h>

enum { TOPK_ORACLE_OK = 0, TOPK_ORACLE_BAD_ARG = 1 };

/*
 * x: batch rows of n fp32 values, `ld` elements apart (ld >= n).  idx: batch x k int32,
 * val: batch x k fp32, dense.  Host memory owned by the caller.
 */
int oracle_topk(int64_t batch, int64_t n, int64_t k, const float *x, int64_t ld, int32_t *idx, float *val)
{
    if (batch < 0 || n < 0 || k < 0 || k > n || ld < n || n > 2147483647) return TOPK_ORACLE_BAD_ARG;
    if (batch > 0 && n > 0 && !x) return TOPK_ORACLE_BAD_ARG;
    if (batch > 0 && k > 0 && (!idx || !val)) return TOPK_ORACLE_BAD_ARG;
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t i = 0; i < n; ++i)
            if (isnan(x[b * ld + i])) return TOPK_ORACLE_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < batch; ++b) {
        const float *row = x + b * ld;
        int64_t out = 0;
        for (int64_t i = 0; i < n; ++i) {
            int64_t rank = 0;
            for (int64_t j = 0; j < n; ++j)
                if (row[j] > row[i] || (row[j] == row[i] && j < i)) ++rank;
            if (rank < k && out < k) {    /* i increases, so the output is in index order; exactly k ranks are below k */
                idx[b * k + out] = (int32_t)i;
                val[b * k + out] = row[i];
                ++out;
            }
        }
    }
    return TOPK_ORACLE_OK;
}
