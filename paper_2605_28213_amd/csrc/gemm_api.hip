// C ABI of the GEMM lineage: argument validation, the per-variant precondition check and the
// dispatch to the kernel of exactly the requested lineage state.  Host code only.
//
// The precondition bookkeeping is the deterministic part of what the paper calls a skill's
// `pre` and `risk` fields (Sec. 3.1): for every state it names the conditions the fast path
// relies on, which of them a given call violates, and what happens then (the state's own
// masked path, or a refusal under GEMM_FLAG_STRICT).  No state ever runs another state's kernel.
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "common.hpp"

using namespace gl;

// Scratch of gemm_run_static: device memory that belongs to the loaded code object, one copy per GPU,
// held until the process ends.  In host code the array's name only stands for the symbol; the address a
// kernel can use is looked up once per device (static_scratch_of) and passed on like a lent workspace.
static __device__ __align__(256) unsigned char scratch[GEMM_STATIC_SCRATCH_BYTES];

namespace {

constexpr int ABI_VERSION = 3;
thread_local hipError_t last_launch_error = hipSuccess;   // of the calling thread's most recent GEMM_ERR_LAUNCH

constexpr int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES];       // per device, filled on the first call with that device current
std::mutex scratch_lock;

hipError_t static_scratch_of(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

bool aligned16(const void* p, int64_t batch, int64_t stride, int es)
{
    if (p && ((uintptr_t)p & 15u)) return false;
    return batch <= 1 || (stride * es) % 16 == 0;
}

struct Plan {
    int status = GEMM_OK;
    bool empty = false;     // nothing to compute (M, N or batch extent 0)
    int path = 0;           // launcher-specific
    Args args{};
    gemm_query_t q{};
};

int validate(int variant, const gemm_desc_t* d, const void* A, const void* B, const void* C, bool need_ptrs)
{
    if (variant < 0 || variant >= GEMM_VARIANT_COUNT) return GEMM_ERR_BAD_VARIANT;
    if (!d) return GEMM_ERR_BAD_ARG;
    if (d->M < 0 || d->N < 0 || d->K < 0 || d->batch < 1 || d->reserved != 0) return GEMM_ERR_BAD_ARG;
    if (d->M > (int64_t)1 << 30 || d->N > (int64_t)1 << 30 || d->K > (int64_t)1 << 30 || d->batch > 65535) return GEMM_ERR_BAD_ARG;
    if (d->in_dtype < 0 || d->in_dtype > GEMM_FP8_E4M3 || d->out_dtype < 0 || d->out_dtype > GEMM_FP8_E4M3)
        return GEMM_ERR_UNSUPPORTED_DTYPE;
    if (!dtype_pair_supported(d->in_dtype, d->out_dtype)) return GEMM_ERR_UNSUPPORTED_DTYPE;
    if ((d->layout_a != GEMM_ROW_MAJOR && d->layout_a != GEMM_COL_MAJOR) ||
        (d->layout_b != GEMM_ROW_MAJOR && d->layout_b != GEMM_COL_MAJOR))
        return GEMM_ERR_BAD_ARG;
    constexpr uint32_t K4_FLAGS = GEMM_FLAG_DEOPT_NO_SWIZZLE | GEMM_FLAG_DEOPT_NO_OVERLAP | GEMM_FLAG_TILE_256 | GEMM_FLAG_TILE_128 |
                                  GEMM_FLAG_DEOPT_NO_RASTER | GEMM_FLAG_DEOPT_NO_PERSISTENT | GEMM_FLAG_STREAM_FORM_MASK | GEMM_FLAG_MFMA_32X32;
    if (d->flags & ~(uint32_t)(GEMM_FLAG_STRICT | K4_FLAGS | GEMM_FLAG_DEOPT_NO_VECTOR)) return GEMM_ERR_BAD_ARG;
    if (((d->flags & GEMM_FLAG_STREAM_FORM_MASK) >> GEMM_FLAG_STREAM_FORM_SHIFT) > 6) return GEMM_ERR_BAD_ARG;
    if ((d->flags & GEMM_FLAG_TILE_256) && (d->flags & GEMM_FLAG_TILE_128)) return GEMM_ERR_BAD_ARG;
    const int64_t min_lda = d->layout_a == GEMM_ROW_MAJOR ? d->K : d->M;
    const int64_t min_ldb = d->layout_b == GEMM_ROW_MAJOR ? d->N : d->K;
    if (d->lda < 1 || d->ldb < 1 || d->ldc < 1) return GEMM_ERR_BAD_ARG;
    if (d->lda < min_lda || d->ldb < min_ldb || d->ldc < d->N) return GEMM_ERR_BAD_ARG;
    if (d->stride_a < 0 || d->stride_b < 0 || d->stride_c < 0) return GEMM_ERR_BAD_ARG;
    if (d->batch > 1 && d->M > 0 && d->N > 0 && d->stride_c < (d->M - 1) * d->ldc + d->N) return GEMM_ERR_BAD_ARG;
    if (need_ptrs && d->M > 0 && d->N > 0) {
        if (!C) return GEMM_ERR_BAD_ARG;
        if (d->K > 0 && (!A || !B)) return GEMM_ERR_BAD_ARG;
    }
    return GEMM_OK;
}

// Grid limits of the launchers (65535 workgroups along y/z, 2^31-1 along x).
bool grid_fits(int variant, const gemm_desc_t* d)
{
    const int64_t lim = 65535;
    if (variant == GEMM_K0_NAIVE) return (d->M + 15) / 16 <= lim;
    if (variant == GEMM_K1_LDS_TILED) return (d->M + 63) / 64 <= lim;
    if (variant == GEMM_K2_VECTORIZED || variant == GEMM_K3_PIPELINED) return (d->M + 127) / 128 <= lim;
    // K4: one-dimensional grid over (batch, tile); the smallest tile of its paths is 128 x 128
    return ((d->M + 127) / 128) * ((d->N + 127) / 128) * d->batch < ((int64_t)1 << 31);
}

Plan make_plan(int variant, const gemm_desc_t* d, const void* A, const void* B, const void* C, bool need_ptrs)
{
    Plan p;
    p.status = validate(variant, d, A, B, C, need_ptrs);
    if (p.status != GEMM_OK) return p;
    if (!grid_fits(variant, d)) { p.status = GEMM_ERR_BAD_ARG; return p; }

    Args& a = p.args;
    a.A = A; a.B = B; a.C = (void*)C;
    a.scale_a = d->scale_a; a.scale_b = d->scale_b; a.bias = d->bias;
    a.workspace = d->workspace;
    a.M = d->M; a.N = d->N; a.K = d->K; a.batch = d->batch;
    a.a_si = d->layout_a == GEMM_ROW_MAJOR ? d->lda : 1;
    a.a_sk = d->layout_a == GEMM_ROW_MAJOR ? 1 : d->lda;
    a.b_sk = d->layout_b == GEMM_ROW_MAJOR ? d->ldb : 1;
    a.b_sj = d->layout_b == GEMM_ROW_MAJOR ? 1 : d->ldb;
    a.ldc = d->ldc;
    a.stride_a = d->stride_a; a.stride_b = d->stride_b; a.stride_c = d->stride_c;
    a.in_dtype = d->in_dtype; a.out_dtype = d->out_dtype;
    a.flags = d->flags & ~(uint32_t)GEMM_FLAG_STRICT;
    a.stream = (hipStream_t)d->stream;
    p.empty = d->M == 0 || d->N == 0;

    const int es = elem_size(d->in_dtype), eo = elem_size(d->out_dtype);
    uint32_t holds = 0;
    if (aligned16(A, d->batch, d->stride_a, es)) holds |= GEMM_COND_ALIGN16_A;
    if (aligned16(B, d->batch, d->stride_b, es)) holds |= GEMM_COND_ALIGN16_B;
    if (aligned16(C, d->batch, d->stride_c, eo)) holds |= GEMM_COND_ALIGN16_C;
    if ((d->lda * es) % 16 == 0) holds |= GEMM_COND_LD16_A;
    if ((d->ldb * es) % 16 == 0) holds |= GEMM_COND_LD16_B;
    if ((d->ldc * eo) % 16 == 0) holds |= GEMM_COND_LD16_C;
    if (d->layout_a == GEMM_ROW_MAJOR) holds |= GEMM_COND_K_CONTIG_A;
    if (d->layout_b == GEMM_COL_MAJOR) holds |= GEMM_COND_K_CONTIG_B;
    holds |= GEMM_COND_DTYPE_HAS_MFMA;   // all four input types have one on gfx950 (fp32: v_mfma_f32_32x32x2_f32)
    if (variant >= GEMM_K1_LDS_TILED) holds |= GEMM_COND_LDS_STAGED;
    if (d->M <= 96) holds |= GEMM_COND_SMALL_M;

    const uint32_t vecA = GEMM_COND_ALIGN16_A | GEMM_COND_LD16_A, vecB = GEMM_COND_ALIGN16_B | GEMM_COND_LD16_B;
    uint32_t required = 0;
    size_t pack_bytes = 0;     // K4 only: scratch of the packed or split-K path (used when lent, advertised otherwise)
    char splitk_path[64];
    Geometry g{};
    const char* path = "";
    switch (variant) {
    case GEMM_K0_NAIVE:
        g = geometry_k0(a);
        path = "naive";
        break;
    case GEMM_K1_LDS_TILED:
        required = GEMM_COND_LDS_STAGED;
        g = geometry_valu_tiled(variant, 0, a);
        path = "lds-tiled";
        break;
    case GEMM_K2_VECTORIZED:
    case GEMM_K3_PIPELINED: {
        required = vecA | vecB | (variant == GEMM_K3_PIPELINED ? (uint32_t)GEMM_COND_LDS_STAGED : 0u);
        const bool va = (holds & vecA) == vecA, vb = (holds & vecB) == vecB;
        p.path = (va ? 1 : 0) | (vb ? 2 : 0);
        path = va && vb ? "vec16" : va ? "vec16(A)+elementwise-masked(B)" : vb ? "elementwise-masked(A)+vec16(B)"
                                                                              : "elementwise-masked";
        if (variant == GEMM_K3_PIPELINED) {
            // the pipelined state's asynchronous form (slabs travel global -> LDS without registers, three stages)
            // also wants K contiguous in both operands and K whole 64-byte slabs; where that fails, or on small
            // problems, the state runs its register-staged form
            required |= GEMM_COND_K_CONTIG_A | GEMM_COND_K_CONTIG_B | GEMM_COND_TILE_DIV_K;
            if (va && vb && k3_async_applies(a)) {
                p.path = VALU_ASYNC;
                path = "vec16-direct-to-lds(3 stages)";
                g = geometry_k3_async(a);
                break;
            }
        }
        g = geometry_valu_tiled(variant, p.path, a);
        break;
    }
    default: {  // GEMM_K4_MFMA
        required = GEMM_COND_DTYPE_HAS_MFMA | GEMM_COND_LDS_STAGED | vecA | vecB | GEMM_COND_K_CONTIG_A | GEMM_COND_K_CONTIG_B |
                   GEMM_COND_TILE_DIV_K;
        const bool va = (holds & (vecA | GEMM_COND_K_CONTIG_A)) == (vecA | GEMM_COND_K_CONTIG_A);
        const bool vb = (holds & (vecB | GEMM_COND_K_CONTIG_B)) == (vecB | GEMM_COND_K_CONTIG_B);
        const int64_t kvec = 16 / es;
        // the streaming kernel addresses a strip of columns and the rows of A with 32-bit byte offsets
        const bool skinny = (holds & GEMM_COND_SMALL_M) && va && vb && d->K % kvec == 0 && d->K > 0 &&
                            d->in_dtype != GEMM_F32 && d->ldb <= ((int64_t)1 << 24) &&
                            d->lda <= ((int64_t)1 << 24) && k4_streams_rows(a);
        // few columns instead of few rows: the same kernel on the transposed product (C^T = B^T A^T)
        const bool skinny_n = !skinny && d->M > d->N && d->N <= 96 && va && vb && d->K % kvec == 0 && d->K > 0 &&
                              d->in_dtype != GEMM_F32 && d->ldb <= ((int64_t)1 << 24) && d->lda <= ((int64_t)1 << 24) &&
                              k4_streams_rows(k4_transposed(a));
        // fp32 has its matrix instruction in the masked kernel only: no direct-to-LDS, packed or streaming form
        const bool f32 = d->in_dtype == GEMM_F32;
        if (f32) required = GEMM_COND_DTYPE_HAS_MFMA | GEMM_COND_LDS_STAGED;
        const bool kdiv = d->K % (128 / es) == 0;   // whole 128-byte slabs: the direct-to-LDS kernel masks nothing along K
        // that kernel addresses a 256-row tile with 32-bit byte offsets: rows are bounded to 4 MiB
        const bool rows_fit = d->lda * es <= ((int64_t)1 << 22) && d->ldb * es <= ((int64_t)1 << 22);
        // packing both operands into lent scratch turns any layout/alignment/K into the fast kernel's case
        // (and the pack kernels' one-dimensional grids, one workgroup per 2048..7936 packed elements, stay below 2^31)
        // an operand that meets the fast kernel's conditions by itself is used in place (K whole slabs: no padding needed)
        const int keep = (va && kdiv && d->lda * es <= ((int64_t)1 << 22) ? 1 : 0) | (vb && kdiv && d->ldb * es <= ((int64_t)1 << 22) ? 2 : 0);
        const bool can_pack = !f32 && d->K > 0 && k4_packed_k(a) * es <= ((int64_t)1 << 22) &&
                              (d->M + d->N) * k4_packed_k(a) < ((int64_t)1 << 40);
        if (skinny) {
            p.path = MFMA_SKINNY;
            path = "mfma16-stream(small-M)";
            required &= ~(uint32_t)GEMM_COND_TILE_DIV_K;
        } else if (skinny_n) {
            p.path = MFMA_SKINNY_N;
            path = "mfma16-stream(small-N)";
            required &= ~(uint32_t)GEMM_COND_TILE_DIV_K;
        } else if (!f32 && va && vb && kdiv && rows_fit) {
            p.path = MFMA_VEC16 | (3 << 8);
            snprintf(splitk_path, sizeof(splitk_path), "mfma32-direct-to-lds%s%s", k4_fast_is_persistent(MFMA_VEC16, a) ? "(persistent)" : "",
                     k4_splits_m_tail(a) ? "+stream(M-tail)" : "");
            path = splitk_path;
            // too few tiles for the chip and a long K: with scratch for the partial products, K is split
            const int splits = k4_splitk_factor(a);
            if (splits > 1) {
                pack_bytes = k4_splitk_workspace_bytes(a, splits);
                if (d->workspace != nullptr) {
                    p.path = MFMA_SPLITK;
                    snprintf(splitk_path, sizeof(splitk_path), "mfma32-direct-to-lds%s+splitK(%d)",
                             k4_fast_is_persistent(MFMA_SPLITK, a) ? "(persistent)" : "", splits);
                    path = splitk_path;
                }
            }
        } else if (!f32 && d->layout_a == GEMM_ROW_MAJOR && d->layout_b == GEMM_ROW_MAJOR && k4_ring_takes_row_major_b(a)) {
            // A and B row-major, enough tiles for the persistent kernel: it reads B in place (transposing LDS reads),
            // rows aligned to an element only with under-aligned loads, a ragged K cleared in LDS: no scratch, no
            // packing pass, and none of the alignment, K-layout and K-divisibility conditions is relied on.  A thin
            // remainder of rows that would cost a whole round of tiles goes to the thin kernel, which reads B in place
            // as well; lent scratch is not used (ragged fp16 workload: 150 us in place, 157 us packed).
            p.path = MFMA_VEC16_BROW | (3 << 8);
            static const char* const BROW_PATHS[8] = {
                "mfma32-direct-to-lds(persistent,B-row-major)", "mfma32-direct-to-lds(persistent,B-row-major)+masked(last col)",
                "mfma32-direct-to-lds(persistent,B-row-major)+thin(last row)", "mfma32-direct-to-lds(persistent,B-row-major)+split(row,col)",
                "mfma32-direct-to-lds(persistent,B-row-major)+thin(M-tail)", "mfma32-direct-to-lds(persistent,B-row-major)+split(M-tail,col)",
                "", ""};
            path = BROW_PATHS[k4_brow_splits(a) & 7];
            required = GEMM_COND_DTYPE_HAS_MFMA | GEMM_COND_LDS_STAGED | GEMM_COND_K_CONTIG_A;
        } else if (!f32 && d->layout_a == GEMM_ROW_MAJOR && d->layout_b == GEMM_ROW_MAJOR && k4_thin_takes_row_major_b(a)) {
            // at most 64 rows, A and B row-major: B is read once, in place, by the thin kernel (no scratch)
            p.path = MFMA_THIN_BROW | (3 << 8);
            path = "mfma16-thin(B-row-major)";
            required = GEMM_COND_DTYPE_HAS_MFMA | GEMM_COND_LDS_STAGED | GEMM_COND_K_CONTIG_A | GEMM_COND_SMALL_M;
        } else if (can_pack && d->workspace != nullptr) {
            // the caller lent scratch: repair the violated conditions by packing, then run the fast kernel
            p.path = MFMA_PACKED | (keep << 8);
            snprintf(splitk_path, sizeof(splitk_path), "mfma32-packed%s+direct-to-lds%s%s", keep == 1 ? "(B)" : keep == 2 ? "(A)" : "",
                     k4_fast_is_persistent(MFMA_PACKED, a) ? "(persistent)" : "",
                     k4_splits_m_tail(a) ? "+stream(M-tail)" : "");
            path = splitk_path;
            pack_bytes = k4_packed_workspace_bytes(a, keep);
        } else {
            if (can_pack) pack_bytes = k4_packed_workspace_bytes(a, keep);   // what lending scratch would buy
            p.path = MFMA_ELEMENTWISE | (((va ? 1 : 0) | (vb ? 2 : 0)) << 8);
            path = va && vb ? "mfma32-vec16-masked" : va ? "mfma32-vec16(A)+elementwise-masked(B)"
                            : vb ? "mfma32-elementwise-masked(A)+vec16(B)" : "mfma32-elementwise-masked";
        }
        g = geometry_k4(p.path & 0xFF, a);
        break;
    }
    }
    if (g.bm > 0 && d->M % g.bm == 0) holds |= GEMM_COND_TILE_DIV_M;
    if (g.bn > 0 && d->N % g.bn == 0) holds |= GEMM_COND_TILE_DIV_N;
    // (K3 relies on whole 64-byte slabs, the K tile of its asynchronous form, whichever of its forms runs)
    const int64_t ktile = variant == GEMM_K3_PIPELINED ? 64 / es : g.bk;
    if (ktile > 0 && d->K % ktile == 0) holds |= GEMM_COND_TILE_DIV_K;

    gemm_query_t& q = p.q;
    q.required = required;
    q.holds = holds;
    q.violated = required & ~holds;
    q.bm = g.bm; q.bn = g.bn; q.bk = g.bk;
    q.threads = g.threads; q.stages = g.stages; q.lds_bytes = g.lds_bytes;
    q.grid = p.empty ? 0 : g.grid;
    q.workspace_bytes = pack_bytes;
    strncpy(q.path, path, sizeof(q.path) - 1);

    if (a.flags & GEMM_FLAG_DEOPT_NO_VECTOR) {   // the vector-load simplification belongs to K2 and K3
        if ((variant != GEMM_K2_VECTORIZED && variant != GEMM_K3_PIPELINED) || (a.flags & ~(uint32_t)GEMM_FLAG_DEOPT_NO_VECTOR)) {
            p.status = GEMM_ERR_BAD_ARG;
            return p;
        }
        p.path = 0;
        strncpy(q.path, "elementwise-masked(-novec)", sizeof(q.path) - 1);
    } else if (a.flags & GEMM_FLAG_STREAM_FORM_MASK) {   // the configuration override of K4's streaming kernel
        const int kind = p.path & 0xFF;
        const bool streams = variant == GEMM_K4_MFMA && (kind == MFMA_SKINNY || kind == MFMA_SKINNY_N);
        if (!streams || (a.flags & ~(uint32_t)GEMM_FLAG_STREAM_FORM_MASK) || !k4_stream_form_fits(kind == MFMA_SKINNY_N ? k4_transposed(a) : a)) {
            p.status = GEMM_ERR_BAD_ARG;
            return p;
        }
        const size_t n = strlen(q.path);
        snprintf(q.path + n, sizeof(q.path) - n, "-form%u", ((a.flags & GEMM_FLAG_STREAM_FORM_MASK) >> GEMM_FLAG_STREAM_FORM_SHIFT) - 1);
    } else if (a.flags) {   // the other simplifications and the tile overrides exist for K4's fast kernel only (also on packed operands)
        const int kind = p.path & 0xFF;
        const bool split_ok = kind == MFMA_SPLITK && (a.flags & ~K4_NEUTRAL_FLAGS) == 0;   // (the split form keeps its ranges' kernel choice)
        if (variant != GEMM_K4_MFMA || (kind != MFMA_VEC16 && kind != MFMA_PACKED && !split_ok)) { p.status = GEMM_ERR_BAD_ARG; return p; }
        const size_t n = strlen(q.path);
        snprintf(q.path + n, sizeof(q.path) - n, "%s%s%s%s%s", (a.flags & GEMM_FLAG_DEOPT_NO_SWIZZLE) ? "-noswz" : "",
                 (a.flags & GEMM_FLAG_DEOPT_NO_OVERLAP) ? "-noovl" : "", (a.flags & GEMM_FLAG_DEOPT_NO_RASTER) ? "-noraster" : "",
                 (a.flags & GEMM_FLAG_DEOPT_NO_PERSISTENT) ? "-nopersist" : "", (a.flags & GEMM_FLAG_MFMA_32X32) ? "-mfma32x32" : "");
    }
    const bool hard = (q.violated & GEMM_COND_DTYPE_HAS_MFMA) != 0;   // no slow path exists for this one
    if (hard || (q.violated && (d->flags & GEMM_FLAG_STRICT))) p.status = GEMM_ERR_PRECONDITION;
    else if (((p.path & 0xFF) == MFMA_PACKED || (p.path & 0xFF) == MFMA_SPLITK) && variant == GEMM_K4_MFMA &&
             (d->workspace_bytes < q.workspace_bytes || ((uintptr_t)d->workspace & 15u)))
        p.status = GEMM_ERR_WORKSPACE;   // scratch was lent but is too small or misaligned: say so rather than run slow
    return p;
}

// Launches the kernel(s) of a plan that make_plan accepted.
int run_plan(int variant, const Plan& p)
{
    (void)hipGetLastError();   // the thread's last-error slot may hold someone else's stale error: GEMM_ERR_LAUNCH must mean this launch
    hipError_t e;
    switch (variant) {
    case GEMM_K0_NAIVE: e = launch_k0(p.args); break;
    case GEMM_K1_LDS_TILED:
    case GEMM_K2_VECTORIZED:
    case GEMM_K3_PIPELINED: e = (variant == GEMM_K3_PIPELINED && p.path == VALU_ASYNC) ? launch_k3_async(p.args) : launch_valu_tiled(variant, p.path, p.args); break;
    default: e = launch_k4(p.path, p.args); break;
    }
    if (e != hipSuccess) last_launch_error = e;
    return e == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int gemm_default_desc(gemm_desc_t* d, int64_t M, int64_t N, int64_t K, int dtype)
{
    if (!d) return GEMM_ERR_BAD_ARG;
    if (dtype < 0 || dtype > GEMM_FP8_E4M3) return GEMM_ERR_UNSUPPORTED_DTYPE;
    if (M < 0 || N < 0 || K < 0) return GEMM_ERR_BAD_ARG;
    memset(d, 0, sizeof(*d));
    d->M = M; d->N = N; d->K = K; d->batch = 1;
    d->in_dtype = dtype;
    d->out_dtype = dtype == GEMM_FP8_E4M3 ? GEMM_BF16 : dtype;
    d->layout_a = GEMM_ROW_MAJOR;
    d->layout_b = (dtype == GEMM_F32 || dtype == GEMM_F16) ? GEMM_ROW_MAJOR : GEMM_COL_MAJOR;
    d->lda = K > 0 ? K : 1;
    d->ldb = d->layout_b == GEMM_ROW_MAJOR ? (N > 0 ? N : 1) : (K > 0 ? K : 1);
    d->ldc = N > 0 ? N : 1;
    d->stride_a = M * d->lda;
    d->stride_b = (d->layout_b == GEMM_ROW_MAJOR ? K : N) * d->ldb;
    d->stride_c = M * d->ldc;
    return GEMM_OK;
}

int gemm_query(int variant, const gemm_desc_t* d, const void* A, const void* B, const void* C, gemm_query_t* out)
{
    if (!out) return GEMM_ERR_BAD_ARG;
    Plan p = make_plan(variant, d, A, B, C, /*need_ptrs=*/false);
    memset(out, 0, sizeof(*out));
    if (p.status == GEMM_OK || p.status == GEMM_ERR_PRECONDITION || p.status == GEMM_ERR_WORKSPACE) *out = p.q;
    return p.status;
}

int gemm_run_ex(int variant, const gemm_desc_t* d, const void* A, const void* B, void* C)
{
    Plan p = make_plan(variant, d, A, B, C, /*need_ptrs=*/true);
    if (p.status != GEMM_OK) return p.status;
    if (p.empty) return GEMM_OK;
    return run_plan(variant, p);
}

size_t gemm_static_scratch_bytes(void) { return GEMM_STATIC_SCRATCH_BYTES; }

int gemm_run_static(int variant, const gemm_desc_t* d, const void* A, const void* B, void* C)
{
    if (!d) return GEMM_ERR_BAD_ARG;
    if (d->workspace != nullptr || d->workspace_bytes != 0) return GEMM_ERR_BAD_ARG;   // this form brings its own scratch
    void* ws = nullptr;
    const hipError_t e = static_scratch_of(&ws);
    if (e != hipSuccess) { last_launch_error = e; return GEMM_ERR_LAUNCH; }
    gemm_desc_t own = *d;
    own.workspace = ws;
    own.workspace_bytes = GEMM_STATIC_SCRATCH_BYTES;
    // a path that wants more scratch than the array holds comes back as GEMM_ERR_WORKSPACE from the plan
    Plan p = make_plan(variant, &own, A, B, C, /*need_ptrs=*/true);
    if (p.status != GEMM_OK) return p.status;
    if (p.empty) return GEMM_OK;
    return run_plan(variant, p);
}

const char* gemm_last_launch_error(void) { return hipGetErrorString(last_launch_error); }

int gemm_run(int variant, int64_t M, int64_t N, int64_t K, int dtype, const void* A, const void* B, void* C)
{
    gemm_desc_t d;
    int rc = gemm_default_desc(&d, M, N, K, dtype);
    if (rc != GEMM_OK) return rc;
    return gemm_run_ex(variant, &d, A, B, C);
}

const char* gemm_status_string(int s)
{
    switch (s) {
    case GEMM_OK: return "ok";
    case GEMM_ERR_BAD_ARG: return "bad argument";
    case GEMM_ERR_BAD_VARIANT: return "unknown variant";
    case GEMM_ERR_UNSUPPORTED_DTYPE: return "unsupported dtype";
    case GEMM_ERR_PRECONDITION: return "precondition of the variant violated";
    case GEMM_ERR_WORKSPACE: return "workspace missing or too small";
    case GEMM_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
    }
}

const char* gemm_variant_name(int v)
{
    static const char* names[] = {"K0_naive", "K1_lds_tiled", "K2_vectorized", "K3_pipelined", "K4_mfma"};
    return (v >= 0 && v < GEMM_VARIANT_COUNT) ? names[v] : "?";
}

const char* gemm_variant_intent(int v)
{
    static const char* intents[] = {"(start of lineage)", "tile / sm_stage", "vectorize_global", "cp.async + pipeline (direct-to-LDS loads, three stages)",
                                    "mma + operand-layout swizzle"};
    return (v >= 0 && v < GEMM_VARIANT_COUNT) ? intents[v] : "?";
}

const char* gemm_cond_name(uint32_t bit)
{
    switch (bit) {
    case GEMM_COND_ALIGN16_A: return "ALIGN16_A";
    case GEMM_COND_ALIGN16_B: return "ALIGN16_B";
    case GEMM_COND_ALIGN16_C: return "ALIGN16_C";
    case GEMM_COND_LD16_A: return "LD16_A";
    case GEMM_COND_LD16_B: return "LD16_B";
    case GEMM_COND_LD16_C: return "LD16_C";
    case GEMM_COND_TILE_DIV_M: return "TILE_DIV_M";
    case GEMM_COND_TILE_DIV_N: return "TILE_DIV_N";
    case GEMM_COND_TILE_DIV_K: return "TILE_DIV_K";
    case GEMM_COND_K_CONTIG_A: return "K_CONTIG_A";
    case GEMM_COND_K_CONTIG_B: return "K_CONTIG_B";
    case GEMM_COND_DTYPE_HAS_MFMA: return "DTYPE_HAS_MFMA";
    case GEMM_COND_LDS_STAGED: return "LDS_STAGED";
    case GEMM_COND_SMALL_M: return "SMALL_M";
    default: return "?";
    }
}

int gemm_variant_count(void) { return GEMM_VARIANT_COUNT; }
int gemm_abi_version(void) { return ABI_VERSION; }

}  // extern "C"
