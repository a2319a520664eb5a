// Launcher of the persistent form of K4's direct-to-LDS kernel (a translation unit of its own: it is compiled
// without the machine-code sinking pass, see the build script).
#include "k4_ring.hpp"

namespace gl {

static_assert(RING_WORKGROUPS == K4_RING_WORKGROUPS, "the planner reports the grid the launcher uses");

// The persistent form of the 256-tile kernel takes a product that gives every one of its workgroups at least
// one tile and whose K is at least three slabs (the slab kinds first / last-but-one / last of a tile are
// distinct) and at most 48: what it saves is per tile (the ring's cold start, and loads that stop during the
// epilogue), so it pays on short K (same box, one-tile form against this one: e4m3 64 x 1024^3, 8 slabs, 95 -> 84 us;
// bf16 32 x 1024^3, 16 slabs, 85 -> 70 us; bf16 16 x 2048^3, 32 slabs, 243 -> 230 us), and loses 2 % at 64 slabs
// (bf16 4096^3: 106 -> 108 us) and at 128 (bf16 8192^3: 779 -> 793 us), where the package is at its power limit either
// way and the loads issued outside the steady-state loop carry their wait states.  The simplified states and the
// 128-tile configuration stay with k4_mfma_fast.
bool k4_uses_ring(const Args& a)
{
    constexpr uint32_t DEOPT = GEMM_FLAG_DEOPT_NO_SWIZZLE | GEMM_FLAG_DEOPT_NO_OVERLAP | GEMM_FLAG_DEOPT_NO_RASTER | GEMM_FLAG_DEOPT_NO_PERSISTENT;
    if ((a.flags & DEOPT) || k4_small_tiles(a)) return false;
    const int64_t ke = ROW_BYTES / elem_size(a.in_dtype);
    const int64_t tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256) * a.batch;
    return a.K / ke >= 3 && a.K / ke <= 48 && tiles >= K4_RING_WORKGROUPS && tiles < ((int64_t)1 << 31);
}

// Row-major B read in place (transposing LDS reads): two-byte types, A row-major; any leading dimensions and any K
// (rows aligned to an element only are loaded with under-aligned 16-byte loads, a ragged last slab is cleared in
// LDS), at least three slabs, at least 256 tiles of 256 x 256, rows of A up to 4 MiB, B below 2 GiB (its k rows are
// addressed with 32-bit byte offsets from the tile's first column).  No upper limit on K: this is the only kernel
// that reads such a B without a packing pass.  When the last row of an operand has an odd number of elements
// (K odd for A, N odd for B) the kernel's loads reach the one element after the operand (RING_BROW_SLACK): with the
// pointers known, such a product is only taken when that element lies in the same 4 KiB page as the operand's last
// byte, so that it is mapped whatever follows the operand, or the row (of A) or column (of C) that needs that element is
// left to a kernel that does not reach past the operand: k4_brow_splits_last_row, k4_brow_splits_last_col.
static bool brow_shape_fits(const Args& a)
{
    if (a.flags != 0 || a.in_dtype == GEMM_FP8_E4M3 || a.in_dtype == GEMM_F32) return false;
    if (a.a_sk != 1 || a.b_sj != 1 || a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
    const int es = elem_size(a.in_dtype);
    const int64_t ke = ROW_BYTES / es;
    const int64_t tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256) * a.batch;
    if ((a.K + ke - 1) / ke < 3 || tiles < K4_RING_WORKGROUPS || tiles >= ((int64_t)1 << 31)) return false;
    return a.a_si * es <= ((int64_t)1 << 22) && a.K * a.b_sk * es < ((int64_t)1 << 31);
}
static bool brow_a_tail_mapped(const Args& a) { return tail_element_in_last_page(a.A, (a.batch - 1) * a.stride_a + (a.M - 1) * a.a_si + a.K, a.K, elem_size(a.in_dtype)); }
static bool brow_b_tail_mapped(const Args& a) { return tail_element_in_last_page(a.B, (a.batch - 1) * a.stride_b + (a.K - 1) * a.b_sk + a.N, a.N, elem_size(a.in_dtype)); }

// A ends with an odd-length row at the very end of a page: the element after it, which the persistent kernel's loads
// of that row would touch, may not be mapped.  The row is then left to the thin kernel (which loads aligned dwords
// of A whenever a row starts off a dword, and so never reaches past the operand's last dword), and the rows before it,
// whose one element of slack is the next row's first, stay here: instead of the masked kernel for the whole product
// (fp16 4096 x 4093 x 4097 with such an A: 1540 us).
bool k4_brow_splits_last_row(const Args& a)
{
    if (a.M < 2 || brow_a_tail_mapped(a)) return false;
    Args top = a;
    top.M = a.M - 1;
    Args bot = a;
    bot.M = 1;
    return brow_shape_fits(top) && k4_thin_takes_row_major_b(bot);
}

// The same for B (N odd, B's last byte the last of a page): the last column of C is left to the masked kernel, which
// loads element by element, and the columns before it, a B of even row length, stay here.
bool k4_brow_splits_last_col(const Args& a)
{
    if (a.N < 2 || brow_b_tail_mapped(a)) return false;
    Args left = a;
    left.N = a.N - 1;
    return brow_shape_fits(left);
}

// The columns the persistent kernel keeps (all, or all but the last).
static Args brow_kept_columns(const Args& a)
{
    Args inner = a;
    if (k4_brow_splits_last_col(a)) inner.N = a.N - 1;
    return inner;
}

bool k4_ring_takes_row_major_b(const Args& a)
{
    if (!brow_shape_fits(a)) return false;
    if (!brow_b_tail_mapped(a) && !k4_brow_splits_last_col(a)) return false;
    const Args inner = brow_kept_columns(a);            // (B's rows are of even length there, or its tail is mapped)
    return brow_a_tail_mapped(inner) || k4_brow_splits_last_row(inner);
}

// What a product on this path hands to other kernels: 1 = C's last column (masked kernel), 2 = A's last row,
// 4 = a thin remainder of rows (thin kernel both).
int k4_brow_splits(const Args& a)
{
    const Args inner = brow_kept_columns(a);
    int m = inner.N != a.N ? 1 : 0;
    if (k4_brow_splits_last_row(inner)) return m | 2;
    return m | (k4_brow_splits_m_tail(inner) ? 4 : 0);
}

static hipError_t launch_brow_rows(const Args& a);

template <typename IN, bool BROW = false>
static hipError_t launch_ring(const Args& a)
{
    using CFG = RingCfg<IN, 8, BROW>;
    const int tiles_m = (int)((a.M + CFG::BM - 1) / CFG::BM), tiles_n = (int)((a.N + CFG::BN - 1) / CFG::BN);
    const int total = (int)((int64_t)tiles_m * tiles_n * a.batch);
    const int eo = a.out_dtype == GEMM_F32 ? 4 : 2;
    const bool vec_c = ((uintptr_t)a.C % 16 == 0) && (a.ldc * eo) % 16 == 0 && (a.batch <= 1 || (a.stride_c * eo) % 16 == 0);
    hipLaunchKernelGGL(k4_mfma_ring<CFG>, dim3(K4_RING_WORKGROUPS), dim3(CFG::T), 0, a.stream, a, tiles_m, tiles_n, total,
                       vec_c ? (int)FAST_VEC_C : 0);
    return hipGetLastError();
}

hipError_t launch_k4_ring_row_major_b(const Args& a)
{
    if (k4_brow_splits_last_col(a)) {        // the element after B is not known to be mapped: see the rule
        const int es = elem_size(a.in_dtype);
        Args left = a;
        left.N = a.N - 1;
        hipError_t e = launch_k4_ring_row_major_b(left);      // (its B has rows of even length: this branch is not taken again)
        if (e != hipSuccess) return e;
        Args right = a;
        right.N = 1;
        right.B = (const char*)a.B + (a.N - 1) * es;
        right.C = (char*)a.C + (a.N - 1) * (a.out_dtype == GEMM_F32 ? 4 : 2);
        if (a.bias) right.bias = a.bias + (a.N - 1);
        return launch_k4(MFMA_ELEMENTWISE, right);
    }
    if (k4_brow_splits_last_row(a)) {        // the element after A is not known to be mapped: see the rule
        const int es = elem_size(a.in_dtype);
        Args top = a;
        top.M = a.M - 1;
        top.A = (const char*)a.A;            // (its last row's slack element is row M-1's first)
        hipError_t e = launch_brow_rows(top);
        if (e != hipSuccess) return e;
        Args bot = a;
        bot.M = 1;
        bot.A = (const char*)a.A + (a.M - 1) * a.a_si * es;
        bot.C = (char*)a.C + (a.M - 1) * a.ldc * (a.out_dtype == GEMM_F32 ? 4 : 2);
        return launch_k4_thin_row_major_b(bot);
    }
    return launch_brow_rows(a);
}

// (the rows given here end with an element of slack that is mapped)
static hipError_t launch_brow_rows(const Args& a)
{
    if (k4_brow_splits_m_tail(a)) {          // a thin remainder of rows that would cost a round of tiles: see the rule
        const int64_t rem = a.M % 256, top_rows = a.M - rem;
        Args top = a;
        top.M = top_rows;
        hipError_t e = launch_brow_rows(top);
        if (e != hipSuccess) return e;
        Args bot = a;
        bot.M = rem;
        bot.A = (const char*)a.A + top_rows * a.a_si * elem_size(a.in_dtype);
        bot.C = (char*)a.C + top_rows * a.ldc * (a.out_dtype == GEMM_F32 ? 4 : 2);
        return launch_k4_thin_row_major_b(bot);
    }
    switch (a.in_dtype) {
    case GEMM_BF16: return launch_ring<BF16, true>(a);
    case GEMM_F16: return launch_ring<F16, true>(a);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_k4_ring(const Args& a)
{
    switch (a.in_dtype) {
    case GEMM_BF16: return launch_ring<BF16>(a);
    case GEMM_F16: return launch_ring<F16>(a);
    case GEMM_FP8_E4M3: return launch_ring<E4M3>(a);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gl
