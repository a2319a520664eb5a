// Row-wise top-k selection (paper Sec. 4.1 workload table: Top-K; Sec. 4.2: selection sort -> radix
// select; Table 1: `radix_select`, "coarse + refine pass"): the kernels of its three states and the C ABI.
// One workgroup per row.  A value's key is its bit pattern made monotone (sign bit flipped for
// non-negative values, all bits for negative ones; -0.0 takes +0.0's key), so "k-th largest value" is
// "k-th largest unsigned key" and can be found digit by digit from histograms.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/topk_lineage.h"

namespace {

struct TopkArgs {
    const float* x;
    int32_t* idx;
    float* val;
    int64_t n, k, ld;
};

__device__ __forceinline__ uint32_t key_of(float v)
{
    uint32_t b = __float_as_uint(v);
    if (b == 0x80000000u) b = 0;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Inclusive prefix sum of v over the workgroup's T threads; *total receives the sum over all of them.
// `wsum` is T/64 ints of LDS.  Two barriers; safe to call back to back.
template <int T>
__device__ __forceinline__ int block_scan(int v, int* wsum, int* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int s = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(s, o, 64);
        if (lane >= o) s += u;
    }
    __syncthreads();                      // the previous call's readers are done with wsum
    if (lane == 63) wsum[wave] = s;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < T / 64; ++w) {
        const int ws = wsum[w];
        if (w < wave) base += ws;
        tot += ws;
    }
    *total = tot;
    return s + base;
}

// Ordered compaction shared by all states.  Each thread owns a contiguous run of elements [lo, hi) and
// classifies element i through `cls(i)`: 2 = above the threshold, 1 = equal to it, 0 = below.  Selected
// are all of class 2 and the first `take_equal` of class 1 in index order; they are written in index
// order, values taken from `value(i)`.  Rows shorter than 65536 elements need one scan (both counts
// packed into one word), longer ones two.
template <int T, typename CLS, typename VAL>
__device__ __forceinline__ void compact(const TopkArgs& a, int64_t lo, int64_t hi, int take_equal, int* wsum, CLS cls, VAL value)
{
    int gt = 0, eq = 0;
    for (int64_t i = lo; i < hi; ++i) {
        const int c = cls(i);
        gt += c == 2;
        eq += c == 1;
    }
    int total, g, e;
    if (a.n < 65536) {
        const int both = block_scan<T>(gt | (eq << 16), wsum, &total) - (gt | (eq << 16));
        g = both & 0xFFFF;                             // class-2 elements before this thread's run
        e = (int)((uint32_t)both >> 16);               // class-1 elements before it
    } else {
        g = block_scan<T>(gt, wsum, &total) - gt;
        e = block_scan<T>(eq, wsum, &total) - eq;
    }
    int32_t* idx = a.idx + (int64_t)blockIdx.x * a.k;
    float* val = a.val + (int64_t)blockIdx.x * a.k;
    for (int64_t i = lo; i < hi; ++i) {
        const int c = cls(i);
        if (c == 2 || (c == 1 && e < take_equal)) {
            const int64_t pos = g + (e < take_equal ? e : take_equal);
            if (pos < a.k) {                            // always true for NaN-free rows
                idx[pos] = (int32_t)i;
                val[pos] = value(i);
            }
        }
        g += c == 2;
        e += c == 1;
    }
}

// ---- T0: selection ------------------------------------------------------------------------------
constexpr int SEL_T = 256;
constexpr int SEL_MAX_N = 65536;

__global__ __launch_bounds__(SEL_T) void topk_selection(TopkArgs a)
{
    __shared__ unsigned char taken[SEL_MAX_N];
    __shared__ float wv[SEL_T / 64];
    __shared__ int wi[SEL_T / 64];
    __shared__ int wsum[SEL_T / 64];
    const float* row = a.x + (int64_t)blockIdx.x * a.ld;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = (int)a.n;
    constexpr int NONE = 0x7FFFFFFF;
    for (int i = tid; i < n; i += SEL_T) taken[i] = 0;
    __syncthreads();
    // a candidate (v, i) beats the best so far when there is none, when it is larger, or equal and earlier
    auto beats = [](float v, int i, float bv, int bi) { return i != NONE && (bi == NONE || v > bv || (v == bv && i < bi)); };
    for (int64_t round = 0; round < a.k; ++round) {
        float bv = 0.0f;
        int bi = NONE;
        for (int i = tid; i < n; i += SEL_T) {
            if (taken[i]) continue;
            const float v = row[i];
            if (beats(v, i, bv, bi)) { bv = v; bi = i; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (beats(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { wv[wave] = bv; wi[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < SEL_T / 64; ++w)
                if (beats(wv[w], wi[w], bv, bi)) { bv = wv[w]; bi = wi[w]; }
            if (bi != NONE) taken[bi] = 1;
        }
        __syncthreads();
    }
    const int64_t seg = (a.n + SEL_T - 1) / SEL_T;
    const int64_t lo = tid * seg < a.n ? tid * seg : a.n, hi = lo + seg < a.n ? lo + seg : a.n;
    compact<SEL_T>(a, lo, hi, 0, wsum, [&](int64_t i) { return taken[i] ? 2 : 0; }, [&](int64_t i) { return row[i]; });
}

// ---- T1 / T2: radix select ----------------------------------------------------------------------
// NPASS histogram passes over digits of B0, B1, ... bits, most significant first (they add up to 32).
// RESIDENT: the thread's ITEMS consecutive keys are loaded once (16 bytes at a time) and every pass
// runs from registers; otherwise every pass reads the row again (any n).
template <int T, int ITEMS, bool RESIDENT, int NPASS, int B0, int B1, int B2, int B3>
__global__ __launch_bounds__(T) void topk_radix(TopkArgs a)
{
    static_assert(B0 + B1 + B2 + B3 == 32 && NPASS >= 1 && NPASS <= 4, "the digits cover the key");
    constexpr int MAXB = B0 > B1 ? (B0 > B2 ? (B0 > B3 ? B0 : B3) : (B2 > B3 ? B2 : B3)) : (B1 > B2 ? (B1 > B3 ? B1 : B3) : (B2 > B3 ? B2 : B3));
    constexpr int BITS[4] = {B0, B1, B2, B3};
    __shared__ int hist[1 << MAXB];
    __shared__ int wsum[T / 64];
    __shared__ int found_digit, found_remaining;
    const float* row = a.x + (int64_t)blockIdx.x * a.ld;
    const int tid = threadIdx.x;
    const int64_t n = a.n;

    // resident form: the thread's values as loaded (bit patterns; the key is three ALU operations away).
    // Elements past n are held as the pattern whose key is 0, below every non-NaN key.
    constexpr uint32_t PAD_BITS = 0xFFFFFFFFu;
    uint32_t held[RESIDENT ? ITEMS : 1];
    if constexpr (RESIDENT) {
        static_assert(ITEMS % 4 == 0, "16-byte loads");
#pragma unroll
        for (int j = 0; j < ITEMS; j += 4) {
            const int64_t i = (int64_t)tid * ITEMS + j;
            if (i + 3 < n) {
                const float4 v = *(const float4*)(row + i);
                held[j] = __float_as_uint(v.x); held[j + 1] = __float_as_uint(v.y); held[j + 2] = __float_as_uint(v.z); held[j + 3] = __float_as_uint(v.w);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) held[j + e] = i + e < n ? __float_as_uint(row[i + e]) : PAD_BITS;
            }
        }
    }

    uint32_t prefix = 0, mask = 0;
    int remaining = (int)a.k, shift = 32;
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
        const int bits = BITS[p], nb = 1 << bits;
        shift -= bits;
        for (int i = tid; i < nb; i += T) hist[i] = 0;
        __syncthreads();
        if constexpr (RESIDENT) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const uint32_t key = key_of(__uint_as_float(held[j]));
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (nb - 1)], 1);
            }
        } else {
            for (int64_t i = tid; i < n; i += T) {
                const uint32_t key = key_of(row[i]);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (nb - 1)], 1);
            }
        }
        __syncthreads();
        // the digit d with  #(candidates with a larger digit) < remaining <= #(candidates with digit >= d)
        const int ch = nb >= T ? nb / T : 1;               // bins per thread, a contiguous chunk
        const bool active = tid * ch < nb;
        int s = 0;
        if (active)
            for (int c = 0; c < ch; ++c) s += hist[tid * ch + c];
        int total;
        const int incl = block_scan<T>(s, wsum, &total);
        const int above = total - incl;                     // candidates in the chunks above this thread's
        if (active && above < remaining && remaining <= above + s) {
            int acc = above;
            for (int d = tid * ch + ch - 1; d >= tid * ch; --d) {
                if (acc + hist[d] >= remaining) {
                    found_digit = d;
                    found_remaining = remaining - acc;
                    break;
                }
                acc += hist[d];
            }
        }
        __syncthreads();
        prefix |= (uint32_t)found_digit << shift;
        mask |= (uint32_t)(nb - 1) << shift;
        remaining = found_remaining;
    }
    // prefix is now the k-th largest key; `remaining` of the elements equal to it are taken
    const uint32_t thr = prefix;
    if constexpr (RESIDENT) {
        const int64_t lo = (int64_t)tid * ITEMS < n ? (int64_t)tid * ITEMS : n, hi = lo + ITEMS < n ? lo + ITEMS : n;
        const int64_t base = (int64_t)tid * ITEMS;
        auto bits_of = [&](int64_t i) {
            uint32_t b = PAD_BITS;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) b = (i - base == j) ? held[j] : b;       // register select, no scratch
            return b;
        };
        compact<T>(a, lo, hi, remaining, wsum,
                   [&](int64_t i) { const uint32_t key = key_of(__uint_as_float(bits_of(i))); return key > thr ? 2 : key == thr ? 1 : 0; },
                   [&](int64_t i) { return __uint_as_float(bits_of(i)); });
    } else {
        const int64_t seg = (n + T - 1) / T;
        const int64_t lo = tid * seg < n ? tid * seg : n, hi = lo + seg < n ? lo + seg : n;
        compact<T>(a, lo, hi, remaining, wsum,
                   [&](int64_t i) { const uint32_t key = key_of(row[i]); return key > thr ? 2 : key == thr ? 1 : 0; },
                   [&](int64_t i) { return row[i]; });
    }
}

constexpr int RES_ITEMS = 16;

struct Plan {
    int status = GEMM_OK;
    bool empty = false;
    TopkArgs a{};
    int threads = 0;
    int items = 0;          // T2: keys per lane
    hipStream_t stream = nullptr;
    topk_query_t q{};
};

Plan make_plan(int variant, const topk_desc_t* d, const float* x, const void* idx, const void* val, bool need_ptrs)
{
    Plan p;
    auto fail = [&](int s) { p.status = s; return p; };
    if (variant < 0 || variant >= TOPK_VARIANT_COUNT) return fail(GEMM_ERR_BAD_VARIANT);
    if (!d) return fail(GEMM_ERR_BAD_ARG);
    if (d->batch < 0 || d->n < 0 || d->k < 0 || d->k > d->n || d->ld < d->n || d->flags != 0 || d->reserved != 0) return fail(GEMM_ERR_BAD_ARG);
    if (d->n >= ((int64_t)1 << 31) || d->batch >= ((int64_t)1 << 31)) return fail(GEMM_ERR_BAD_ARG);
    p.empty = d->batch == 0 || d->k == 0;
    if (need_ptrs && !p.empty && (!x || !idx || !val)) return fail(GEMM_ERR_BAD_ARG);
    p.a = TopkArgs{x, (int32_t*)idx, (float*)val, d->n, d->k, d->ld};
    p.stream = (hipStream_t)d->stream;

    uint32_t holds = 0, required = 0;
    if (d->n <= SEL_MAX_N) holds |= TOPK_COND_ROW_IN_LDS;
    if (d->n <= 1024 * RES_ITEMS) holds |= TOPK_COND_ROW_IN_REGISTERS;
    if ((!x || ((uintptr_t)x & 15u) == 0) && d->ld % 4 == 0) holds |= TOPK_COND_ALIGN16;
    const char* path = "";
    topk_query_t& q = p.q;
    switch (variant) {
    case TOPK_T0_SELECTION:
        required = TOPK_COND_ROW_IN_LDS;
        path = "selection(k arg-max rounds)";
        p.threads = SEL_T; q.passes = (int32_t)(d->k < 0x7FFFFFFF ? d->k : 0x7FFFFFFF); q.lds_bytes = SEL_MAX_N + 48;
        break;
    case TOPK_T1_RADIX_SELECT:
        path = "radix-select(8+8+8+8, streaming)";
        p.threads = 256; q.passes = 5; q.lds_bytes = 256 * 4 + 24;
        break;
    default:
        required = TOPK_COND_ROW_IN_REGISTERS | TOPK_COND_ALIGN16;
        // 1024 lanes per row: 64 rows keep a quarter of the CUs busy, so the work per lane is what counts
        // (batch 64, n 4096, k 512: 15.5 us with 256 lanes x 16 keys, 10.2 us with 1024 lanes x 4 keys)
        p.threads = 1024;
        p.items = d->n <= 1024 * 4 ? 4 : RES_ITEMS;
        path = p.items == 4 ? "radix-select(11+11+10, 4 keys/lane x 1024)" : "radix-select(11+11+10, 16 keys/lane x 1024)";
        q.passes = 4; q.lds_bytes = 2048 * 4 + 72;
        break;
    }
    q.required = required; q.holds = holds; q.violated = required & ~holds;
    q.threads = p.threads;
    q.grid = p.empty ? 0 : d->batch;
    strncpy(q.path, path, sizeof(q.path) - 1);
    if (q.violated) p.status = GEMM_ERR_PRECONDITION;
    return p;
}

thread_local hipError_t last_topk_launch_error = hipSuccess;

}  // namespace

extern "C" {

int topk_query(int variant, const topk_desc_t* d, const float* x, topk_query_t* out)
{
    if (!out) return GEMM_ERR_BAD_ARG;
    Plan p = make_plan(variant, d, x, nullptr, nullptr, /*need_ptrs=*/false);
    memset(out, 0, sizeof(*out));
    if (p.status == GEMM_OK || p.status == GEMM_ERR_PRECONDITION) *out = p.q;
    return p.status;
}

int topk_run(int variant, const topk_desc_t* d, const float* x, int32_t* idx, float* val)
{
    Plan p = make_plan(variant, d, x, idx, val, /*need_ptrs=*/true);
    if (p.status != GEMM_OK) return p.status;
    if (p.empty) return GEMM_OK;
    (void)hipGetLastError();
    const dim3 grid((unsigned)d->batch);
    if (variant == TOPK_T0_SELECTION)
        hipLaunchKernelGGL(topk_selection, grid, dim3(SEL_T), 0, p.stream, p.a);
    else if (variant == TOPK_T1_RADIX_SELECT)
        hipLaunchKernelGGL((topk_radix<256, 1, false, 4, 8, 8, 8, 8>), grid, dim3(256), 0, p.stream, p.a);
    else if (p.items == 4)
        hipLaunchKernelGGL((topk_radix<1024, 4, true, 3, 11, 11, 10, 0>), grid, dim3(1024), 0, p.stream, p.a);
    else
        hipLaunchKernelGGL((topk_radix<1024, RES_ITEMS, true, 3, 11, 11, 10, 0>), grid, dim3(1024), 0, p.stream, p.a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) last_topk_launch_error = e;
    return e == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

const char* topk_last_launch_error(void) { return hipGetErrorString(last_topk_launch_error); }

const char* topk_variant_name(int v)
{
    static const char* names[] = {"T0_selection", "T1_radix_select", "T2_resident_coarse_refine"};
    return (v >= 0 && v < TOPK_VARIANT_COUNT) ? names[v] : "?";
}

const char* topk_variant_intent(int v)
{
    static const char* intents[] = {"(start of lineage)", "radix_select", "keys resident in registers; coarse + refine pass"};
    return (v >= 0 && v < TOPK_VARIANT_COUNT) ? intents[v] : "?";
}

const char* topk_cond_name(uint32_t bit)
{
    switch (bit) {
    case TOPK_COND_ROW_IN_LDS: return "ROW_IN_LDS";
    case TOPK_COND_ROW_IN_REGISTERS: return "ROW_IN_REGISTERS";
    case TOPK_COND_ALIGN16: return "ALIGN16";
    default: return "?";
    }
}

int topk_variant_count(void) { return TOPK_VARIANT_COUNT; }

}  // extern "C"
