// K4, thin products with a ROW-MAJOR B: C (R x N, R <= 64) = A (R x K, row-major) . B (K x N, row-major), two-byte
// types, nothing aligned, any K.  Bound by reading B once (the counterpart of k4_stream, which wants B column-major).
//
// A workgroup owns a strip of 64 (or 32) columns of C; its 8 waves split K (wave w takes the k tiles w, w + 8, ...)
// and add their partial sums in LDS at the end.  A k tile is 4 KB: 32 k rows x 128 bytes, or 64 x 64 on the narrow
// strips.  Per tile a wave loads the strip's part of B as it lies in memory (four 16-byte loads per lane,
// under-aligned, through a buffer resource that ends with the matrix: rows past K come back as zeros, columns past N
// are whatever follows and only feed outputs that are never stored), parks it in a wave-private LDS tile and reads
// the fragments of v_mfma_f32_16x16x32 back with the transposing read ds_read_b64_tr_b16 (see RingCfg in
// k4_ring.hpp for its lane layout: a block of 16 lanes turns a 4 k x 16 n patch into 4 consecutive k per lane);
// chunk c of k row r is kept at c ^ swz(r), so that what a block reads with one instruction lies in 16 different
// 8-byte slots.  A's fragments (16 rows x 8 consecutive k per lane) come straight from memory: A is small and stays
// in L2 (rows of A that start 2 bytes off a dword: see ThinCfg::ODD).  K ragged: A's elements past K are masked to zero in registers (B's are zeros already).  The loads of the
// next one or two k tiles are in flight while a tile is multiplied (register sets taken in turn).
//
// Used for the thin remainder of rows that the persistent kernel's row-major-B form would otherwise multiply as
// one more, mostly empty, row of tiles (fp16 4099 x 4093 x 4097: 215 -> 150 us), and for whole products of at most
// 64 rows with both operands row-major (3 / 33 / 64 rows x 4093 x 4097: 18 / 29 / 40 us; 64 workgroups).
// Paper Table 1: "smem_transpose" on the small side of the lineage's expert state.
#pragma once
#include "k4_kernels.hpp"

namespace gl {

template <typename IN, int MG_, int COLS_ = 64, bool ODD_ = false>
struct ThinCfg {
    using In = IN;
    // ODD: some row of A starts on an odd element, i.e. 2 bytes off a dword.  A's fragment loads (16 bytes per lane,
    // 16 rows per instruction) are served at a fraction of the aligned rate from such addresses (64 rows x 4096 x 4096
    // fp16: 26 us with leading dimensions of 4096, 31 with 4098, 67 with 4097, 62 with A's alone 4097), so this
    // form loads the five aligned dwords that hold a lane's 16 bytes and shifts them into place in registers (41 us).
    // B's loads (a row's 128 bytes over 8 consecutive lanes) lose little off a dword (3 rows: 16.9 against 16.2 us)
    // and a fifth dword per load costs them more than that (21 us), so they stay as they are.
    static constexpr bool ODD = ODD_;
    static constexpr int MG = MG_, ROWS = 16 * MG_;      // groups of 16 rows of A (and C)
    static constexpr int WAVES = 8, COLS = COLS_;        // waves per workgroup; columns per strip
    static constexpr int RB = COLS_ * 2;                 // bytes of a k row of the strip
    static constexpr int TK = 4096 / RB;                 // k rows per tile: a tile is 4 KB per wave (32 rows x 128 B or 64 x 64 B)
    static constexpr int KS = TK / 32;                   // matrix-instruction k-steps per tile
    static constexpr int TILE_BYTES = 4096;
    static constexpr int SETS = MG_ <= 2 ? 3 : 2;        // k tiles held in registers per wave (one in hand, the rest landing)
    static constexpr int LDS_BYTES = WAVES * TILE_BYTES > WAVES * 16 * (COLS + 1) * 4 ? WAVES * TILE_BYTES : WAVES * 16 * (COLS + 1) * 4;
    static_assert(IN::BYTES == 2, "two-byte types (the transposing read used here is the 16-bit one)");
    static_assert(MG_ == 1 || MG_ == 2 || MG_ == 4, "16, 32 or 64 rows");
    static_assert(COLS_ == 64 || COLS_ == 32, "strips of 64 or of 32 columns");
    // chunk c (16 bytes) of k row r is parked at c ^ swz(r): the four rows a block of 16 lanes reads with one
    // transposing instruction, and the two chunks of a 16-column patch, then fall into 16 different 8-byte slots
    __device__ static constexpr int swz(int r) { return COLS_ == 64 ? (r & 7) : (r & 2); }
};

template <typename CFG>
__global__ __launch_bounds__(CFG::WAVES * 64) void k4_thin_brow(Args a)
{
    using IN = typename CFG::In;
    constexpr int MG = CFG::MG, WAVES = CFG::WAVES, COLS = CFG::COLS, TK = CFG::TK, RB = CFG::RB, KS = CFG::KS;
    constexpr int LPR = RB / 16, RPL = 64 / LPR;         // lanes per k row of a load; k rows per load instruction
    constexpr int NJB = COLS / 16;                       // 16-column blocks of the strip
    __shared__ __attribute__((aligned(16))) char lds[CFG::LDS_BYTES];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int64_t b = blockIdx.y;
    const int64_t j0 = (int64_t)blockIdx.x * COLS;
    char* tile = lds + wave * CFG::TILE_BYTES;

    // buffer resources over this batch item's A and this strip's part of B (both below 2 GiB: checked by the host)
    // (ODD: A's resource starts at the dword that holds its first element, and a lane's offset carries the two bytes)
    const char* A = (const char*)a.A + b * a.stride_a * 2;
    const char* B = (const char*)a.B + (b * a.stride_b + j0) * 2;
    const int rem_a = CFG::ODD ? (int)((uintptr_t)A & 2) : 0;
    A -= rem_a;
    const int64_t bytes_a = ((a.M - 1) * a.a_si + a.K) * 2 + 2 + rem_a;  // (+ one element: the dword that holds an odd row's last one)
    const int64_t bytes_b = ((a.K - 1) * a.b_sk + (a.N - j0)) * 2 + 2;
    constexpr int RSRC_FLAGS = 0x00020000;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, (int)bytes_a, RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)B, 0, (int)bytes_b, RSRC_FLAGS);

    // B loads: load n (0..3) of a lane covers k row RPL n + lane/LPR of the tile, chunk lane%LPR (8 columns)
    const int brow = lane / LPR, bchunk = lane % LPR;
    const int voff_b = (int)((brow * a.b_sk + bchunk * 8) * 2);
    const int step_b = (int)(RPL * a.b_sk * 2);                            // bytes from load n to load n + 1
    // parked at: row * RB + ((chunk ^ swz(row)) << 4); rows RPL n + lane/LPR: swz(row) = swz(lane/LPR) for every n
    const int park = brow * RB + ((bchunk ^ CFG::swz(brow)) << 4);
    // fragment reads (per k-step ks, 16-column block jb and half h of the lane's 8 k): lane l of a block of 16 points
    // at k row 32 ks + 8 (l/16) + 4 h + (l%16)/4 and columns 16 jb + 4 (l%4) .. +3
    const int l16 = lane & 15, kq = lane >> 4;
    const int fr_row = 8 * kq + (l16 >> 2), fr_col = 4 * (l16 & 3);
    // A fragments: lane holds row l16 of a group, k 8 kq .. 8 kq + 7 of a k-step
    int voff_a[MG], sh_a[MG];
#pragma unroll
    for (int m = 0; m < MG; ++m) {
        const int64_t r = m * 16 + l16 < a.M ? m * 16 + l16 : a.M - 1;      // (rows past M: clamped, never stored)
        // (ODD: the lane's byte offset is rounded down to a dword and sh_a = 0 or 16 bits are shifted out after the
        // load; k tiles are whole dwords apart, so the shift is the same for every load of a lane)
        const int byte_a = (int)((r * a.a_si + 8 * kq) * 2) + rem_a;
        voff_a[m] = CFG::ODD ? byte_a & ~3 : byte_a;
        sh_a[m] = (byte_a & 2) * 8;
    }

    typedef short v4s_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4s_t* tr_ptr;
    f32x4_t acc[MG][NJB];
#pragma unroll
    for (int m = 0; m < MG; ++m)
#pragma unroll
        for (int j = 0; j < NJB; ++j) acc[m][j] = f32x4_t{0, 0, 0, 0};

    const int64_t tiles = (a.K + TK - 1) / TK;
    // One k tile in registers: 4 loads of B, one load of A per row group and k-step (ODD: and the dword after it).
    struct Held { u32x4_t b[4]; u32x4_t a[KS][MG]; uint32_t ax[KS][MG]; };
    auto shifted = [](const u32x4_t v, uint32_t x, int sh) __attribute__((always_inline)) {
        return u32x4_t{__builtin_amdgcn_alignbit(v.y, v.x, sh), __builtin_amdgcn_alignbit(v.z, v.y, sh),
                       __builtin_amdgcn_alignbit(v.w, v.z, sh), __builtin_amdgcn_alignbit(x, v.w, sh)};
    };
    auto fetch = [&](Held& h, int64_t kt) __attribute__((always_inline)) {
        // (the tile number is the same in every lane; said once more, or each load is wrapped in a loop over the
        // lanes' "different" scalar offsets and the waits around it turn conservative)
        const int k0 = __builtin_amdgcn_readfirstlane((int)(kt * TK));
        const int so_b = __builtin_amdgcn_readfirstlane((int)(k0 * a.b_sk * 2));
#pragma unroll
        for (int n = 0; n < 4; ++n)
            h.b[n] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, voff_b + n * step_b, so_b, 0));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int m = 0; m < MG; ++m)
                h.a[ks][m] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, voff_a[m], (k0 + 32 * ks) * 2, 0));
        if constexpr (CFG::ODD) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int m = 0; m < MG; ++m) h.ax[ks][m] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_a, voff_a[m] + 16, (k0 + 32 * ks) * 2, 0);
        }
    };
    auto multiply = [&](Held& h, int64_t kt) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < 4; ++n) *(u32x4_t*)(tile + n * RPL * RB + park) = h.b[n];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if constexpr (CFG::ODD) {
#pragma unroll
                for (int m = 0; m < MG; ++m) h.a[ks][m] = shifted(h.a[ks][m], h.ax[ks][m], sh_a[m]);
            }
            // A's elements beyond K are the next row's first ones (or the slack element): zero them
            const int valid = (int)(a.K - kt * TK) - 32 * ks - 8 * kq;     // this lane's k that lie inside K
            if (valid < 8) {
#pragma unroll
                for (int m = 0; m < MG; ++m)
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const int left = valid - 2 * d;
                        h.a[ks][m][d] = left <= 0 ? 0u : left == 1 ? (h.a[ks][m][d] & 0xFFFFu) : h.a[ks][m][d];
                    }
            }
#pragma unroll
            for (int jb = 0; jb < NJB; ++jb) {
                u32x4_t fb;
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const int row = 32 * ks + fr_row + 4 * hh, chunk = (16 * jb + fr_col) >> 3;
                    const int off = row * RB + ((chunk ^ CFG::swz(row)) << 4) + ((fr_col >> 2) & 1) * 8;
                    const v4s_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(tile + off));
                    const uint32_t lo = (uint32_t)(uint16_t)v[0] | ((uint32_t)(uint16_t)v[1] << 16);
                    const uint32_t hi = (uint32_t)(uint16_t)v[2] | ((uint32_t)(uint16_t)v[3] << 16);
                    if (hh == 0) { fb.x = lo; fb.y = hi; } else { fb.z = lo; fb.w = hi; }
                }
#pragma unroll
                for (int m = 0; m < MG; ++m) mfma16<IN>(h.a[ks][m], fb, acc[m][jb]);
            }
        }
    };
    // Wave w takes k tiles w, w + WAVES, ...  Two tiles' loads are in flight while a third is multiplied (three
    // register sets taken in turn: 8 KB of B per wave on its way beside the tile in hand); with 64 rows the
    // accumulators and A's fragments leave room for two sets.  Every prefetch is issued, also past the last tile
    // (clamped to tile number `tiles`, whose rows all lie past K: the range check answers those loads with zeros
    // without touching memory): were a prefetch conditional, the compiler's wait before each use would have to
    // allow for the path on which it was skipped, i.e. wait for the youngest loads too, and nothing would overlap.
    auto ahead = [&](int64_t k) __attribute__((always_inline)) { return k < tiles ? k : tiles; };
    int64_t kt = wave;
    if constexpr (CFG::SETS == 3) {
        Held h0, h1, h2;
        fetch(h0, ahead(kt));
        fetch(h1, ahead(kt + WAVES));
        while (kt < tiles) {
            fetch(h2, ahead(kt + 2 * WAVES));
            multiply(h0, kt);
            kt += WAVES;
            if (kt >= tiles) break;
            fetch(h0, ahead(kt + 2 * WAVES));
            multiply(h1, kt);
            kt += WAVES;
            if (kt >= tiles) break;
            fetch(h1, ahead(kt + 2 * WAVES));
            multiply(h2, kt);
            kt += WAVES;
        }
    } else {
        Held h0, h1;
        fetch(h0, ahead(kt));
        while (kt < tiles) {
            fetch(h1, ahead(kt + WAVES));
            multiply(h0, kt);
            kt += WAVES;
            if (kt >= tiles) break;
            fetch(h0, ahead(kt + WAVES));
            multiply(h1, kt);
            kt += WAVES;
        }
    }

    // partial sums of the waves meet in LDS, one group of 16 rows at a time.  16 x 16 accumulator: register r of lane
    // l holds row 4 (l/16) + r, column l%16.
    const float sc = batch_scale(a, b);
    float* part = (float*)lds;
#pragma unroll
    for (int m = 0; m < MG; ++m) {
        __syncthreads();
#pragma unroll
        for (int jb = 0; jb < NJB; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[(wave * 16 + 4 * kq + r) * (COLS + 1) + jb * 16 + l16] = acc[m][jb][r];
        __syncthreads();
        for (int o = t; o < 16 * COLS; o += WAVES * 64) {
            const int i = o / COLS, j = o % COLS;
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) v += part[(w * 16 + i) * (COLS + 1) + j];
            const int64_t gi = m * 16 + i, gj = j0 + j;
            if (gi < a.M && gj < a.N) store_out(a.C, b * a.stride_c + gi * a.ldc + gj, v * sc + (a.bias ? a.bias[gj] : 0.0f), a.out_dtype);
        }
    }
}

}  // namespace gl
