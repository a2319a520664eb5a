// Launcher of K4's kernel for thin products with a row-major B (k4_thin.hpp), and the rule by which the
// row-major-B form of the persistent kernel hands it a thin remainder of rows.
#include "k4_thin.hpp"

namespace gl {

// A remainder of 1..64 rows past the last whole 256-row tile costs the persistent kernel a whole extra row of
// tiles.  When that row makes the product need one more round of the chip (fp16 4099 x 4093 x 4097: 17 x 16
// tiles on 256 workgroups, a second round for 3 rows) the remainder goes to the thin kernel, which reads B once
// more; when the extra tiles fit a round that runs anyway they stay.  The tiled part must still give every
// persistent workgroup a tile; up to 16384 columns (beyond, reading B again costs about what the round does);
// the batch is the thin kernel's second grid dimension.
bool k4_brow_splits_m_tail(const Args& a)
{
    const int64_t rem = a.M % 256;
    if (a.M <= 256 || rem < 1 || rem > 64 || a.N > 16384 || a.batch > 65535 || a.flags != 0) return false;
    if ((a.K + 64) * a.b_sk * 2 >= ((int64_t)1 << 31)) return false;      // (the thin kernel's last k tile is addressed past K)
    const int64_t per_row = ((a.N + 255) / 256) * a.batch, rows = a.M / 256;
    if (rows * per_row < K4_RING_WORKGROUPS) return false;
    return (rows * per_row + 255) / 256 < ((rows + 1) * per_row + 255) / 256;
}

// A whole product of at most 64 rows with A and B row-major (two-byte types): B below 2 GiB and A's rows below
// 16 MiB (32-bit byte offsets), the batch within the grid's second dimension, and the element after an odd-length
// last row of B mapped (see tail_element_in_last_page).  Nothing is asked of A's address: its loads are aligned
// dwords (rows that start on one, or the form that rounds them down to one), and an aligned dword that holds an
// element of A lies in A's pages.
bool k4_thin_takes_row_major_b(const Args& a)
{
    if (a.flags != 0 || (a.in_dtype != GEMM_BF16 && a.in_dtype != GEMM_F16)) return false;
    if (a.a_sk != 1 || a.b_sj != 1 || a.M < 1 || a.M > 64 || a.N < 1 || a.K < 1 || a.batch > 65535) return false;
    if ((a.K + 64) * a.b_sk * 2 >= ((int64_t)1 << 31) || a.M * a.a_si * 2 >= ((int64_t)1 << 31)) return false;
    return tail_element_in_last_page(a.B, (a.batch - 1) * a.stride_b + (a.K - 1) * a.b_sk + a.N, a.N, 2);
}

// Strips of 64 columns (128-byte pieces of B's rows).  The kernel also compiles for strips of 32 (twice the workgroups,
// 64-byte pieces, k tiles of 64 rows); measured on fp16 3 / 33 / 64 x 4093 x 4097, where 64-column strips number 64,
// before A's odd rows were loaded as aligned dwords: 17.6 / 38 / 61 us against 18.2 / 43 / 65 us, and with the waits
// fixed for both (every prefetch issued) 18.2 / 41 / 67 against the same: not what bounds it, so the narrow form is
// not instantiated.
int k4_thin_cols(const Args&) { return 64; }

template <typename IN, int MG, int COLS, bool ODD>
static hipError_t launch_thin_cfg(const Args& a)
{
    using CFG = ThinCfg<IN, MG, COLS, ODD>;
    dim3 grid((unsigned)((a.N + CFG::COLS - 1) / CFG::COLS), (unsigned)a.batch, 1), block(CFG::WAVES * 64, 1, 1);
    hipLaunchKernelGGL(k4_thin_brow<CFG>, grid, block, 0, a.stream, a);
    return hipGetLastError();
}

template <typename IN, bool ODD>
static hipError_t launch_thin_rows(const Args& a)
{
    return a.M <= 16 ? launch_thin_cfg<IN, 1, 64, ODD>(a) : a.M <= 32 ? launch_thin_cfg<IN, 2, 64, ODD>(a) : launch_thin_cfg<IN, 4, 64, ODD>(a);
}

// Does any row of A (of any batch item) start 2 bytes off a dword?
static bool k4_thin_rows_off_dword(const Args& a)
{
    return ((uintptr_t)a.A & 2) || (a.M > 1 && (a.a_si & 1)) || (a.batch > 1 && (a.stride_a & 1));
}

template <typename IN>
static hipError_t launch_thin(const Args& a)
{
    return k4_thin_rows_off_dword(a) ? launch_thin_rows<IN, true>(a) : launch_thin_rows<IN, false>(a);
}

// a.M <= 64, A and B row-major, two-byte types, B below 2 GiB, a.batch <= 65535 (checked by the caller's rule)
hipError_t launch_k4_thin_row_major_b(const Args& a)
{
    if (a.M < 1 || a.M > 64 || a.batch > 65535 || a.a_sk != 1 || a.b_sj != 1) return hipErrorInvalidValue;
    switch (a.in_dtype) {
    case GEMM_BF16: return launch_thin<BF16>(a);
    case GEMM_F16: return launch_thin<F16>(a);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace gl
