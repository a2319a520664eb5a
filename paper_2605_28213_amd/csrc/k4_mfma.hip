// K4 launchers: picks the kernel of the path that gemm_api.hip proved legal and launches it with
// the frozen tile configuration.
#include "k4_kernels.hpp"

namespace gl {

// Frozen configurations ("templatize" + an offline sweep, paper Table 1 expression-level intents).
template <typename IN> using FastK4 = FastCfg<IN, 256>;                    // 256x256 tile, 4 waves, 128x128 per wave, one workgroup per CU
template <typename IN> using FastK4Mi16 = FastCfg<IN, 256, 8, true, true, 0, false, true>;   // the same with 8 x 8 accumulator tiles of v_mfma_f32_16x16x32 per wave (two-byte types)
template <typename IN> using FastK4Mi16Long = FastCfg<IN, 256, 8, true, true, 8, false, true>;   // ... and 8 instructions ahead of the slab barrier (K of 96 slabs or more)
template <typename IN> using FastK4Small = FastCfg<IN, 128>;               // 128x128 tile, 4 waves, 64x64 per wave, two workgroups per CU
template <typename IN> using FastK4SmallDeep = FastCfgDeep<IN>;            // ... with a ring of nine regions, one workgroup per CU
template <typename IN> using StreamK4 = StreamCfg<IN, 1, 1, 256, 19>;      // 16 columns per one-wave workgroup, 512-byte runs, K walk rotated by 19 tiles per workgroup
template <typename IN> using StreamK4Deep = StreamCfg<IN, 4, 1, 256, 19>;  // the same with 4 waves taking K tiles in turn, for strips too few to fill the chip
template <typename IN> using StreamK4Rows32 = StreamCfg<IN, 2, 2, 256, 19, 2>;   // 17..32 rows: 32 columns, two groups of A
template <typename IN> using StreamK4Rows48 = StreamCfg<IN, 4, 4, 128, 19, 3>;   // 33..48 rows: 64 columns, 256-byte runs
template <typename IN> using StreamK4Rows64 = StreamCfg<IN, 4, 4, 128, 19, 4>;   // 49..64 rows
template <typename IN> using StreamK4Rows96 = StreamCfg<IN, 4, 4, 128, 19, 6>;   // 65..96 rows
constexpr int MASKED_BM = 128, MASKED_BN = 128, MASKED_WM = 2, MASKED_WN = 2;   // (64 x 64 for small problems, see masked_tile)

template <typename CFG>
static hipError_t launch_fast(const Args& a)
{
    auto kern = k4_mfma_fast<CFG>;
    const int tiles_m = (int)((a.M + CFG::BM - 1) / CFG::BM), tiles_n = (int)((a.N + CFG::BN - 1) / CFG::BN);
    dim3 grid((unsigned)((int64_t)tiles_m * tiles_n * a.batch), 1, 1), block(CFG::T, 1, 1);
    const int eo = a.out_dtype == GEMM_F32 ? 4 : 2;
    const bool vec_c = ((uintptr_t)a.C % 16 == 0) && (a.ldc * eo) % 16 == 0 && (a.batch <= 1 || (a.stride_c * eo) % 16 == 0);
    // Tile walk: the XCD-aware banded walk unless the caller asks for the row-major one.  (With one operand
    // set resident in the Infinity Cache the row-major order measured 1-5 % faster on single products; with
    // operands rotated, as the benchmark does, it is equal on 8192^3 and 5 % slower on 4096^3.)
    const bool plain = (a.flags & GEMM_FLAG_DEOPT_NO_RASTER) != 0;
    const int kflags = (vec_c ? (int)FAST_VEC_C : 0) | (plain ? (int)FAST_PLAIN_RASTER : 0);
    hipLaunchKernelGGL(kern, grid, block, 0, a.stream, a, tiles_m, tiles_n, kflags);
    return hipGetLastError();
}

// The masked kernel takes 64 x 64 tiles (one 32 x 32 accumulator tile per wave) when 128 x 128 tiles would
// leave most CUs idle (fp32 256^3: 4 workgroups took 37 us).
static int masked_tile(const Args& a)
{
    const int64_t t = ((a.M + MASKED_BM - 1) / MASKED_BM) * ((a.N + MASKED_BN - 1) / MASKED_BN) * a.batch;
    return t < 256 ? 64 : MASKED_BM;
}

template <typename IN, int BT>
static hipError_t launch_masked_tile(const Args& a, int vec_mask)
{
    const int tiles_m = (int)((a.M + BT - 1) / BT), tiles_n = (int)((a.N + BT - 1) / BT);
    dim3 grid((unsigned)((int64_t)tiles_m * tiles_n * a.batch), 1, 1), block(MASKED_WM * MASKED_WN * 64, 1, 1);
    hipLaunchKernelGGL((k4_mfma_masked<IN, BT, BT, MASKED_WM, MASKED_WN>), grid, block, 0, a.stream, a, vec_mask, tiles_m, tiles_n);
    return hipGetLastError();
}

template <typename IN>
static hipError_t launch_masked(const Args& a, int vec_mask)
{
    return masked_tile(a) == 64 ? launch_masked_tile<IN, 64>(a, vec_mask) : launch_masked_tile<IN, MASKED_BM>(a, vec_mask);
}

template <typename CFG>
static hipError_t launch_stream_cfg(const Args& a)
{
    dim3 grid((unsigned)((a.N + CFG::COLS - 1) / CFG::COLS), (unsigned)a.batch, 1), block(CFG::WAVES * 64, 1, 1);
    hipLaunchKernelGGL(k4_stream<CFG>, grid, block, 0, a.stream, a);
    return hipGetLastError();
}

// One wave per strip of 16 columns when that gives every CU work (bf16 16 x 16384 x 16384: 1024 strips,
// 78 us against 85 us for two-wave workgroups of 32 columns: waves that share no barrier drift apart and
// spread over the memory channels); with fewer strips than CUs, 4 waves split each strip's K.
static bool stream_deep(const Args& a) { return ((a.N + 15) / 16) * a.batch < 512; }

// 17..96 rows: every workgroup reads all of A (from L2) beside its strip of B, so the strip widens with the
// rows to keep A's share of the load traffic at one half.  Measured on N = K = 16384 bf16, B read once from
// HBM (537 MB): 32 rows 87 us (2 waves x 32 columns; 100 us with 16 columns, 93 us with 4 waves x 64
// columns), 48 rows 90 us, 64 rows 97 us (4 waves x 64 columns x 256-byte runs; 104 us with 2 waves x 32
// columns); the split-K form of the tiled kernel took 139-142 us on the same products.  96 rows (six groups of
// A, 484 registers): 113 us against about 150 us for the split-K form; eight groups spill and lose to it.
enum StreamForm { STREAM_16 = 0, STREAM_16_DEEP, STREAM_32, STREAM_48, STREAM_64, STREAM_96 };
static const int STREAM_FORM_ROWS[6] = {16, 16, 32, 48, 64, 96};
static StreamForm stream_form(const Args& a)
{
    const uint32_t forced = (a.flags & GEMM_FLAG_STREAM_FORM_MASK) >> GEMM_FLAG_STREAM_FORM_SHIFT;
    if (forced) return (StreamForm)(forced - 1);
    if (a.M <= 16) return stream_deep(a) ? STREAM_16_DEEP : STREAM_16;
    return a.M <= 32 ? STREAM_32 : a.M <= 48 ? STREAM_48 : a.M <= 64 ? STREAM_64 : STREAM_96;
}

bool k4_stream_form_fits(const Args& a)
{
    const uint32_t forced = (a.flags & GEMM_FLAG_STREAM_FORM_MASK) >> GEMM_FLAG_STREAM_FORM_SHIFT;
    return forced >= 1 && forced <= 6 && a.M <= STREAM_FORM_ROWS[forced - 1];
}

// Whether a product of 17..96 rows is given to the streaming kernel: when its strips fill at least half of
// the CUs (below that the tiled kernel, split along K, has more workgroups to offer).
bool k4_streams_rows(const Args& a)
{
    if (a.M <= 16) return true;
    if (a.M > 96) return false;
    const int cols = a.M <= 32 ? 32 : 64;
    return ((a.N + cols - 1) / cols) * a.batch >= 128;
}

// C = A B with few columns is C^T = B^T A^T with few rows: B's columns (K contiguous) become the rows of the
// first operand, A's rows the columns of the second, and the kernel writes its output transposed.
Args k4_transposed(const Args& a)
{
    Args s = a;
    s.A = a.B; s.a_si = a.b_sj; s.a_sk = a.b_sk; s.stride_a = a.stride_b;
    s.B = a.A; s.b_sj = a.a_si; s.b_sk = a.a_sk; s.stride_b = a.stride_a;
    s.M = a.N; s.N = a.M;
    s.flags = a.flags | ARGS_C_TRANSPOSED;
    return s;
}

template <typename IN>
static hipError_t launch_stream(const Args& a)
{
    switch (stream_form(a)) {
    case STREAM_16: return launch_stream_cfg<StreamK4<IN>>(a);
    case STREAM_16_DEEP: return launch_stream_cfg<StreamK4Deep<IN>>(a);
    case STREAM_32: return launch_stream_cfg<StreamK4Rows32<IN>>(a);
    case STREAM_48: return launch_stream_cfg<StreamK4Rows48<IN>>(a);
    case STREAM_64: return launch_stream_cfg<StreamK4Rows64<IN>>(a);
    default: return launch_stream_cfg<StreamK4Rows96<IN>>(a);
    }
}

// Tile choice of the fast kernel ("templatize" + a measured sweep, Table 1's expression-level intents).
// 256-tiles run one workgroup per CU, 128-tiles two, so a "round" of the machine is 256 or 512 tiles; a
// round of 128-tiles covers half the output of a round of 256-tiles at about 0.7 of its time (0.8 for
// e4m3, whose 64 x 64 wave tiles saturate LDS).  The cheaper estimate wins, 256-tiles on a tie.  Measured
// with operands rotated over three sets (bf16 unless noted; 256-tiles / 128-tiles):
//   2048^3 (64 vs 256 tiles: 1 round vs 0.7) 43 / 25 us;  2048 x 4096 x 4096 (1 vs 0.7) 81 / 65 us;
//   4096 x 3072 x 4096 (192 tiles: 1 round vs 2 x 0.7) 88 / 96 us;  4096 x 4352 x 4096 (2 vs 3 x 0.7) 166 / 168 us;
//   8 x 1024^3 (1 vs 0.7) 32 / 24 us;  64 x 1024^3 e4m3 (4 vs 8 x 0.8) 108 / 131 us.
bool k4_small_tiles(const Args& a)
{
    if (a.flags & GEMM_FLAG_TILE_128) return true;
    if (a.flags & (GEMM_FLAG_TILE_256 | GEMM_FLAG_DEOPT_NO_SWIZZLE | GEMM_FLAG_DEOPT_NO_OVERLAP)) return false;   // the instantiations without swizzle / overlap are 256-tile ones
    const int64_t t256 = ((a.M + 255) / 256) * ((a.N + 255) / 256) * a.batch, t128 = ((a.M + 127) / 128) * ((a.N + 127) / 128) * a.batch;
    const int64_t r256 = (t256 + 255) / 256, r128 = (t128 + 511) / 512;
    const int64_t cost128 = a.in_dtype == GEMM_FP8_E4M3 ? 8 : 7;     // tenths of a 256-tile round
    return r128 * cost128 < r256 * 10;
}

// 128-tiles that number at most one per CU take the nine-region ring (FastCfgDeep) when K is at least 32 slabs: its
// steady-state loop is nine slabs long and entered from 13 slabs on, and what comes before and after it waits for
// every load.  Same box, operands rotated, nine regions against five: bf16 2048^3 (256 tiles, 32 slabs) 23.8 against
// 26.2 us, 2048 x 1024 x 2048 (128 tiles) 20.0 / 23.8, 1536^2 x 8192 (144 tiles, 128 slabs) 55.2 / 58.4, 1024^2 x 4096
// 34.7 / 35.6; with 16 slabs it loses (1024^3 16.9 / 15.6, e4m3 2048^3 19.9 / 18.8) and with 8 badly (2048^2 x 512
// 17.0 / 11.6).  The gain is small: the distance of the prefetch is not what bounds these products (2048^3: the
// matrix pipe is busy in 32 % of wave cycles at 2.35 GHz, a slab takes 1340 cycles against 512 of matrix instructions).
static bool k4_small_tiles_deep(const Args& a)
{
    const int64_t nslab = a.K / (ROW_BYTES / elem_size(a.in_dtype));
    return nslab >= 32 && ((a.M + 127) / 128) * ((a.N + 127) / 128) * a.batch <= 256;
}

// The expert instantiation, or one of its validated simplifications when the caller asks for it.
template <typename IN>
static hipError_t launch_fast_any(const Args& a)
{
    if (k4_uses_ring(a)) return launch_k4_ring(a);
    const bool noswz = a.flags & GEMM_FLAG_DEOPT_NO_SWIZZLE, noovl = a.flags & GEMM_FLAG_DEOPT_NO_OVERLAP;
    if (noswz && noovl) return launch_fast<FastCfg<IN, 256, 8, false, false>>(a);
    if (noswz) return launch_fast<FastCfg<IN, 256, 8, false, true>>(a);
    if (noovl) return launch_fast<FastCfg<IN, 256, 8, true, false>>(a);
    if (k4_small_tiles(a)) return k4_small_tiles_deep(a) ? launch_fast<FastK4SmallDeep<IN>>(a) : launch_fast<FastK4Small<IN>>(a);
    // Two-byte types: 8 x 8 accumulator tiles of v_mfma_f32_16x16x32 per wave.  Same box, operands rotated, against
    // the 32x32x16 form: bf16 8192^3 755 -> 725-737 us, 4096^3 104.7 -> 96.3 us (the package draws the same 1.4 kW at
    // 1.92 instead of 1.64 GHz).  With a long K, 8 instructions of a slab's last k-step go ahead of its barrier
    // (8192^3: 733-737 -> 724-726 us; at 64 slabs they cost 2 %; 16, 24 and 32 of them lose on both).
    if constexpr (IN::BYTES == 2) {
        if (!(a.flags & GEMM_FLAG_MFMA_32X32)) {
            const int64_t nslab = a.K / (ROW_BYTES / IN::BYTES);
            return nslab >= 96 ? launch_fast<FastK4Mi16Long<IN>>(a) : launch_fast<FastK4Mi16<IN>>(a);
        }
    }
    return launch_fast<FastK4<IN>>(a);
}

// A thin remainder of rows (1..64 past the last whole 256-row tile) costs a whole extra row of workgroup
// tiles.  When that row makes the product need one more round of the chip (fp16 4099 x 4093 x 4097: 17 x 16
// tiles, a second round for 3 rows) the remainder is split off and handed to the streaming kernel, which
// reads B once more but finishes in the time of that read; when the extra tiles fit into a round that
// runs anyway, they cost nothing and stay.  Applies to products on 256-tiles whose operands the fast kernel
// accepts (they satisfy the streaming kernel's conditions), up to 16384 columns (beyond, reading B again
// costs about what the extra round does).
bool k4_splits_m_tail(const Args& a)
{
    const int64_t rem = a.M % 256;
    if (a.M <= 256 || rem < 1 || rem > 64 || a.N > 16384 || (a.flags & ~K4_NEUTRAL_FLAGS) != 0 || k4_small_tiles(a)) return false;
    const int64_t per_row = ((a.N + 255) / 256) * a.batch, rows = a.M / 256;
    return (rows * per_row + 255) / 256 < ((rows + 1) * per_row + 255) / 256;
}

template <typename IN>
static hipError_t launch_fast_split(const Args& a)
{
    if (k4_splits_m_tail(a)) {
        const int64_t rem = a.M % 256, top_rows = a.M - rem;
        const int eo = a.out_dtype == GEMM_F32 ? 4 : 2;
        Args top = a;
        top.M = top_rows;
        hipError_t e = launch_fast_any<IN>(top);
        if (e != hipSuccess) return e;
        Args bot = a;
        bot.M = rem;
        bot.A = (const char*)a.A + top_rows * a.a_si * IN::BYTES;
        bot.C = (char*)a.C + top_rows * a.ldc * eo;
        return launch_stream<IN>(bot);
    }
    return launch_fast_any<IN>(a);
}

// Split-K ("split-K / stream-K for small M" among Table 1's expression-level intents).  A product whose
// tiles do not fill the 256 CUs once and whose K is long (decode-like shapes with 17..128 rows: bf16
// 32 x 16384 x 16384 took 206 us on 128 workgroups) is cut along K into `splits` equal ranges that run
// as the batch items of one launch of the fast kernel (batch strides = the K range), each writing fp32
// partial products to caller-lent scratch; a second small kernel adds them, scales, adds the bias and
// rounds once.  The factor: the largest divisor of the slab count that keeps at least 16 slabs per
// range and at most about 512 workgroups, at most 8.
int k4_splitk_factor(const Args& a)
{
    if (a.batch != 1 || (a.flags & ~K4_NEUTRAL_FLAGS) != 0 || a.M <= 16 || k4_splits_m_tail(a)) return 1;
    const int64_t ke = ROW_BYTES / elem_size(a.in_dtype);
    if (a.K <= 0 || a.K % ke != 0) return 1;
    const int64_t nslab = a.K / ke, tiles = ((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (tiles >= 256) return 1;
    int best = 1;
    for (int s = 2; s <= 8; ++s)
        if (nslab % s == 0 && nslab / s >= 16 && tiles * s <= 640) best = s;
    return best;
}

size_t k4_splitk_workspace_bytes(const Args& a, int splits) { return (size_t)splits * (size_t)(a.M * a.N) * 4; }

template <typename IN>
static hipError_t launch_splitk(const Args& a)
{
    const int splits = k4_splitk_factor(a);
    Args p = a;
    p.batch = splits;
    p.K = a.K / splits;
    p.stride_a = p.K;                       // K is contiguous in both operands: the next range starts K/splits elements on
    p.stride_b = p.K;
    p.C = a.workspace; p.ldc = a.N; p.stride_c = a.M * a.N;
    p.out_dtype = GEMM_F32;
    p.scale_a = p.scale_b = nullptr; p.bias = nullptr;
    p.flags = (k4_small_tiles(a) ? GEMM_FLAG_TILE_128 : GEMM_FLAG_TILE_256) | (a.flags & K4_NEUTRAL_FLAGS);   // the tile the product itself would get
    hipError_t e = launch_fast_any<IN>(p);
    if (e != hipSuccess) return e;
    const int64_t threads = a.M * ((a.N + 3) / 4);
    hipLaunchKernelGGL(k4_splitk_reduce<IN>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, a.stream, a, (const float*)a.workspace, splits);
    return hipGetLastError();
}

// The arguments the fast kernel is launched with on each of its three paths, as far as the choice between its
// persistent and its one-tile-per-workgroup form depends on them (mirrors launch_packed, launch_splitk and
// launch_fast_split).
static Args fast_kernel_args(int kind, const Args& a)
{
    Args p = a;
    if (kind == MFMA_SPLITK) {
        const int splits = k4_splitk_factor(a);
        p.batch = splits;
        p.K = a.K / splits;
        p.flags = (k4_small_tiles(a) ? GEMM_FLAG_TILE_128 : GEMM_FLAG_TILE_256) | (a.flags & K4_NEUTRAL_FLAGS);
        return p;
    }
    if (kind == MFMA_PACKED) p.K = k4_packed_k(a);
    if (k4_splits_m_tail(p)) p.M = p.M - p.M % 256;
    return p;
}

bool k4_fast_is_persistent(int kind, const Args& a) { return k4_uses_ring(fast_kernel_args(kind, a)); }

int64_t k4_packed_k(const Args& a)
{
    const int64_t ke = ROW_BYTES / elem_size(a.in_dtype);
    return (a.K + ke - 1) / ke * ke;
}

size_t k4_packed_workspace_bytes(const Args& a, int keep_mask)
{
    const int64_t rows = ((keep_mask & 1) ? 0 : a.M) + ((keep_mask & 2) ? 0 : a.N);
    return (size_t)(a.batch * rows * k4_packed_k(a)) * elem_size(a.in_dtype);
}

// Packed path: the operands are rewritten K-contiguous, aligned and zero-padded along K in the workspace
// ([batch][M][Kp] then [batch][N][Kp]), then the fast kernel runs on the copies.  An operand that already
// meets the fast kernel's conditions (and K is whole slabs, so nothing needs padding) is used in place.
template <typename IN>
static hipError_t launch_packed(const Args& a, int keep_mask)
{
    using raw = typename IN::raw;
    constexpr int KE = ROW_BYTES / IN::BYTES;
    const int64_t Kp = k4_packed_k(a);
    const bool keep_a = (keep_mask & 1) != 0, keep_b = (keep_mask & 2) != 0;
    raw* pa = (raw*)a.workspace;
    raw* pb = keep_a ? pa : pa + a.batch * a.M * Kp;
    // one operand: `rows` logical rows (M or N), element strides sr along rows and sk along K
    auto pack = [&](const void* src, int64_t sr, int64_t sk, int64_t rows, int64_t src_batch, raw* dst) {
        if (rows <= 0 || Kp <= 0) return;
        const int64_t dst_batch_bytes = rows * Kp * IN::BYTES, src_batch_bytes = src_batch * IN::BYTES;
        if (sk == 1) {
            const int64_t threads = rows * (Kp / (16 / IN::BYTES));
            dim3 g((unsigned)((threads + 255) / 256), (unsigned)a.batch, 1);
            hipLaunchKernelGGL(k4_pack_rows<IN>, g, dim3(256), 0, a.stream, (const char*)src, sr * IN::BYTES, rows, a.K, Kp,
                               (char*)dst, src_batch_bytes, dst_batch_bytes);
        } else {   // sr == 1: row- or column-major storage leaves no other case
            const int64_t row_tiles = (rows + PackRows<IN> - 1) / PackRows<IN>, k_groups = (Kp / KE + 7) / 8;
            dim3 g((unsigned)(8 * k_groups * row_tiles), (unsigned)a.batch, 1);
            hipLaunchKernelGGL(k4_pack_transpose<IN>, g, dim3(256), 0, a.stream, (const char*)src, sk * IN::BYTES, rows, a.K, Kp,
                               (char*)dst, src_batch_bytes, dst_batch_bytes, (int)row_tiles);
        }
    };
    if (!keep_a) pack(a.A, a.a_si, a.a_sk, a.M, a.stride_a, pa);
    if (!keep_b) pack(a.B, a.b_sj, a.b_sk, a.N, a.stride_b, pb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    Args p = a;
    p.K = Kp;
    if (!keep_a) { p.A = pa; p.a_si = Kp; p.a_sk = 1; p.stride_a = a.M * Kp; }
    if (!keep_b) { p.B = pb; p.b_sj = Kp; p.b_sk = 1; p.stride_b = a.N * Kp; }
    return launch_fast_split<IN>(p);
}

// `path`: low byte = MfmaPath, next byte = bitmask of operands whose 16-byte loads are legal.
hipError_t launch_k4(int path, const Args& a)
{
    const int kind = path & 0xFF, vec_mask = (path >> 8) & 3;   // (packed path: the mask of operands used in place)
    if (kind == MFMA_PACKED) {
        switch (a.in_dtype) {
        case GEMM_BF16: return launch_packed<BF16>(a, vec_mask);
        case GEMM_F16: return launch_packed<F16>(a, vec_mask);
        case GEMM_FP8_E4M3: return launch_packed<E4M3>(a, vec_mask);
        default: return hipErrorInvalidValue;
        }
    }
    if (kind == MFMA_SPLITK) {
        switch (a.in_dtype) {
        case GEMM_BF16: return launch_splitk<BF16>(a);
        case GEMM_F16: return launch_splitk<F16>(a);
        case GEMM_FP8_E4M3: return launch_splitk<E4M3>(a);
        default: return hipErrorInvalidValue;
        }
    }
    if (kind == MFMA_SKINNY || kind == MFMA_SKINNY_N) {
        const Args s = kind == MFMA_SKINNY_N ? k4_transposed(a) : a;
        if (a.in_dtype == GEMM_BF16) return launch_stream<BF16>(s);
        if (a.in_dtype == GEMM_F16) return launch_stream<F16>(s);
        if (a.in_dtype == GEMM_FP8_E4M3) return launch_stream<E4M3>(s);
        return hipErrorInvalidValue;
    }
    if (kind == MFMA_VEC16_BROW) return launch_k4_ring_row_major_b(a);
    if (kind == MFMA_THIN_BROW) return launch_k4_thin_row_major_b(a);
    if (kind == MFMA_VEC16) {
        switch (a.in_dtype) {
        case GEMM_BF16: return launch_fast_split<BF16>(a);
        case GEMM_F16: return launch_fast_split<F16>(a);
        case GEMM_FP8_E4M3: return launch_fast_split<E4M3>(a);
        default: return hipErrorInvalidValue;
        }
    }
    switch (a.in_dtype) {
    case GEMM_F32: return launch_masked<F32>(a, vec_mask);
    case GEMM_BF16: return launch_masked<BF16>(a, vec_mask);
    case GEMM_F16: return launch_masked<F16>(a, vec_mask);
    case GEMM_FP8_E4M3: return launch_masked<E4M3>(a, vec_mask);
    default: return hipErrorInvalidValue;
    }
}

// Convolution layer on the fast kernel: 128 x 128 tiles (the layer sizes this is built for have 64-256
// filters; 64 x 64 per wave leaves the registers the gather's per-lane pixel state needs).
template <typename IN> using ConvK4 = FastCfg<IN, 128, 8, true, true, 0, true>;

hipError_t launch_k4_conv(const Args& a)
{
    switch (a.in_dtype) {
    case GEMM_BF16: return launch_fast<ConvK4<BF16>>(a);
    case GEMM_F16: return launch_fast<ConvK4<F16>>(a);
    case GEMM_FP8_E4M3: return launch_fast<ConvK4<E4M3>>(a);
    default: return hipErrorInvalidValue;
    }
}

Geometry geometry_k4_conv(const Args& a)
{
    using C = ConvK4<BF16>;
    const int es = elem_size(a.in_dtype);
    const int64_t g = ((a.M + C::BM - 1) / C::BM) * ((a.N + C::BN - 1) / C::BN);
    return Geometry{C::BM, C::BN, ROW_BYTES / es, C::T, 2, C::LDS_BYTES, g};
}

Geometry geometry_k4(int path, const Args& a)
{
    const int kind = path & 0xFF;
    const int es = elem_size(a.in_dtype);
    if (kind == MFMA_SKINNY || kind == MFMA_SKINNY_N) {
        const bool tr = kind == MFMA_SKINNY_N;          // transposed product: the strip runs along M
        const Args s = tr ? k4_transposed(a) : a;
        auto of = [&](auto cfg) {
            using C = decltype(cfg);
            return Geometry{tr ? C::COLS : C::ROWS, tr ? C::ROWS : C::COLS, C::TK * 2 / es, C::WAVES * 64, 2, C::LDS_BYTES,
                            ((s.N + C::COLS - 1) / C::COLS) * a.batch};
        };
        switch (stream_form(s)) {
        case STREAM_16: return of(StreamK4<BF16>{});
        case STREAM_16_DEEP: return of(StreamK4Deep<BF16>{});
        case STREAM_32: return of(StreamK4Rows32<BF16>{});
        case STREAM_48: return of(StreamK4Rows48<BF16>{});
        case STREAM_64: return of(StreamK4Rows64<BF16>{});
        default: return of(StreamK4Rows96<BF16>{});
        }
    }
    if (kind == MFMA_THIN_BROW) {
        const int cols = k4_thin_cols(a);
        return Geometry{a.M <= 16 ? 16 : a.M <= 32 ? 32 : 64, cols, 2048 / cols, 512, 2, cols == 64 ? 33280 : 32768, ((a.N + cols - 1) / cols) * a.batch};
    }
    if (kind == MFMA_VEC16_BROW) return Geometry{256, 256, ROW_BYTES / es, 256, 2, FastK4<BF16>::LDS_BYTES, K4_RING_WORKGROUPS};
    if (kind == MFMA_VEC16 || kind == MFMA_PACKED || kind == MFMA_SPLITK) {
        // (with a row remainder split off, the grid of the tiled part: the remainder is a second launch)
        Args top = a;
        if (kind != MFMA_SPLITK && k4_splits_m_tail(a)) top.M = a.M - a.M % 256;
        const bool small = k4_small_tiles(top);
        const int bt = small ? FastK4Small<BF16>::BM : FastK4<BF16>::BM;
        int64_t g = ((top.M + bt - 1) / bt) * ((a.N + bt - 1) / bt) * a.batch * (kind == MFMA_SPLITK ? k4_splitk_factor(a) : 1);
        if (k4_fast_is_persistent(kind, a)) g = K4_RING_WORKGROUPS;      // persistent workgroups, several tiles each
        // stages: slabs in flight beyond the one in use
        const Args p = fast_kernel_args(kind, a);
        if (k4_small_tiles(p) && !k4_uses_ring(p) && !(p.flags & (GEMM_FLAG_DEOPT_NO_SWIZZLE | GEMM_FLAG_DEOPT_NO_OVERLAP)) && k4_small_tiles_deep(p))
            return Geometry{bt, bt, ROW_BYTES / es, 256, FastK4SmallDeep<BF16>::DEPTH, FastK4SmallDeep<BF16>::LDS_BYTES, g};
        return Geometry{bt, bt, ROW_BYTES / es, 256, 2, small ? FastK4Small<BF16>::LDS_BYTES : FastK4<BF16>::LDS_BYTES, g};
    }
    const int bt = masked_tile(a);
    const int64_t g = ((a.M + bt - 1) / bt) * ((a.N + bt - 1) / bt) * a.batch;
    return Geometry{bt, bt, ROW_BYTES / es, MASKED_WM * MASKED_WN * 64, 2, 4 * bt * ROW_BYTES, g};
}

}  // namespace gl
