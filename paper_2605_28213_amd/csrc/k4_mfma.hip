// K4, the expert end of the lineage: K3 + "mma" + "ldmatrix.swizzle" (paper Table 1,
// "Compute & layout"), realised for CDNA4: wave64 MFMA with fp32 accumulators and an LDS
// operand layout in which every 16-byte fragment read is bank-conflict free.
//
// Preconditions recorded for this state (Table 1: "tile fits mma", "mma fragment layout";
// Sec. 1: matrix intrinsics need compatible tile shapes, layouts and hardware support):
//   - the input dtype has a matrix instruction (bf16, fp16, OCP e4m3);
//   - fast loads need K contiguous in both operands, 16-byte aligned bases and leading
//     dimensions; any other operand is gathered element by element under a mask.
//
// Data movement per workgroup and K slab of 128 bytes per row:
//   global --16 B/lane--> registers --ds_write_b128--> LDS[buf^1]     (next slab)
//   LDS[buf] --ds_read_b128--> MFMA operand registers --> v_mfma_f32_32x32x16   (this slab)
// LDS rows are 128 bytes (eight 16-byte chunks); chunk c of row r lives at chunk position
// c ^ swz(r), so the 16 lanes served together read 16 different bank groups.
#include "common.hpp"

namespace gl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

constexpr int ROW_BYTES = 128;            // bytes of K per LDS row and per slab
constexpr int CHUNKS = ROW_BYTES / 16;    // 16-byte chunks per row

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// One 32x32 MFMA step on a 16-byte operand chunk per lane.  For 2-byte types the chunk is one
// K=16 instruction; for e4m3 it is two K=16 instructions on its low and high halves.  Which k a
// lane's bytes stand for is irrelevant as long as A and B agree, and both come through here.
template <typename IN>
__device__ __forceinline__ void mfma_chunk(const u32x4_t& a, const u32x4_t& b, f32x16_t& c)
{
    if constexpr (IN::ID == GEMM_BF16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    } else if constexpr (IN::ID == GEMM_F16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    } else {
        const long alo = (long)(((uint64_t)a.y << 32) | a.x), ahi = (long)(((uint64_t)a.w << 32) | a.z);
        const long blo = (long)(((uint64_t)b.y << 32) | b.x), bhi = (long)(((uint64_t)b.w << 32) | b.z);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(alo, blo, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(ahi, bhi, c, 0, 0, 0);
    }
}

struct TileSrc {
    const char* base;   // operand base for this batch item (bytes)
    int64_t sr, sk;     // element strides along rows and along K
    int64_t rows;       // logical rows (M for A, N for B)
    int64_t r0;         // first row of the workgroup tile
    bool vec;           // 16-byte loads along K are legal
};

// Fetch this thread's share of a BR x 128-byte slab into registers (NCH chunks of 16 bytes).
template <typename IN, int BR, int THREADS, int NCH>
__device__ __forceinline__ void fetch_tile(const TileSrc& x, int64_t k0, int64_t K, int t, u32x4_t (&R)[NCH])
{
    using raw = typename IN::raw;
    constexpr int V = 16 / IN::BYTES;
    static_assert(BR * CHUNKS == NCH * THREADS, "tile must divide evenly over the threads");
    const bool kcontig = x.sk == 1;
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
        const int q = t + n * THREADS;
        // along K first when K is contiguous (8 lanes cover one 128-byte row), along rows otherwise
        const int c = kcontig ? q % CHUNKS : q / BR;
        const int r = kcontig ? q / CHUNKS : q % BR;
        const int64_t gr = x.r0 + r, gk = k0 + (int64_t)c * V;
        u32x4_t w = u32x4_t{0, 0, 0, 0};
        if (gr < x.rows && gk < K) {
            const raw* p = (const raw*)x.base + gr * x.sr + gk * x.sk;
            if (x.vec && gk + V <= K) {
                w = *(const u32x4_t*)p;
            } else {
                raw tmp[V];
#pragma unroll
                for (int e = 0; e < V; ++e) tmp[e] = (gk + e < K) ? p[e * x.sk] : (raw)0;
                __builtin_memcpy(&w, tmp, 16);
            }
        }
        R[n] = w;
    }
}

template <int BR, int THREADS, int NCH>
__device__ __forceinline__ void commit_tile(bool kcontig, int t, const u32x4_t (&R)[NCH], char* lds)
{
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
        const int q = t + n * THREADS;
        const int c = kcontig ? q % CHUNKS : q / BR;
        const int r = kcontig ? q / CHUNKS : q % BR;
        *(u32x4_t*)(lds + r * ROW_BYTES + ((c ^ swz(r)) << 4)) = R[n];
    }
}

// Workgroup id -> (tile_m, tile_n).  Hardware hands consecutive workgroup ids to the 8 XCDs in
// turn; ids are first regrouped so that each XCD (own L2) works on one contiguous run of tiles,
// then tiles are walked in bands of GROUP_M tile-rows so that a run reuses few A rows and B columns.
__device__ __forceinline__ void tile_of(int pid, int total, int tiles_m, int tiles_n, int& tm, int& tn)
{
    constexpr int XCD = 8, GROUP_M = 8;
    const int x = pid % XCD, local = pid / XCD;
    const int base = total / XCD, rem = total % XCD;
    const int id = x * base + (x < rem ? x : rem) + local;
    const int width = GROUP_M * tiles_n;
    const int g = id / width, first = g * GROUP_M;
    const int gsz = (tiles_m - first) < GROUP_M ? (tiles_m - first) : GROUP_M;
    tm = first + (id % width) % gsz;
    tn = (id % width) / gsz;
}

template <typename IN, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void k4_mfma(Args a, int vec_mask, int tiles_m, int tiles_n)
{
    constexpr int T = WM * WN * 64;
    constexpr int KE = ROW_BYTES / IN::BYTES;      // K elements per slab
    constexpr int TMI = BM / WM / 32, TNI = BN / WN / 32;
    constexpr int NCA = BM * CHUNKS / T, NCB = BN * CHUNKS / T;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* As = lds;                               // [2][BM][128]
    char* Bs = lds + 2 * BM * ROW_BYTES;          // [2][BN][128]

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t b = blockIdx.y;
    int tm, tn;
    tile_of(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);

    TileSrc sa{(const char*)a.A + b * a.stride_a * IN::BYTES, a.a_si, a.a_sk, a.M, (int64_t)tm * BM, (vec_mask & 1) != 0};
    TileSrc sb{(const char*)a.B + b * a.stride_b * IN::BYTES, a.b_sj, a.b_sk, a.N, (int64_t)tn * BN, (vec_mask & 2) != 0};
    const bool kca = a.a_sk == 1, kcb = a.b_sk == 1;

    f32x16_t acc[TMI][TNI];
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < TNI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4_t ra[NCA], rb[NCB];
    const int64_t nslab = (a.K + KE - 1) / KE;

    if (nslab > 0) {
        fetch_tile<IN, BM, T>(sa, 0, a.K, t, ra);
        fetch_tile<IN, BN, T>(sb, 0, a.K, t, rb);
        commit_tile<BM, T>(kca, t, ra, As);
        commit_tile<BN, T>(kcb, t, rb, Bs);
    }
    __syncthreads();

    const int lrow = lane & 31, lhalf = lane >> 5;
    int cur = 0;
    for (int64_t s = 0; s < nslab; ++s) {
        const bool more = s + 1 < nslab;
        if (more) {
            fetch_tile<IN, BM, T>(sa, (s + 1) * KE, a.K, t, ra);
            fetch_tile<IN, BN, T>(sb, (s + 1) * KE, a.K, t, rb);
        }
        const char* Ac = As + cur * BM * ROW_BYTES + (wm * (BM / WM)) * ROW_BYTES;
        const char* Bc = Bs + cur * BN * ROW_BYTES + (wn * (BN / WN)) * ROW_BYTES;
#pragma unroll
        for (int ks = 0; ks < CHUNKS / 2; ++ks) {
            const int c = 2 * ks + lhalf;
            u32x4_t fa[TMI], fb[TNI];
#pragma unroll
            for (int i = 0; i < TMI; ++i) {
                const int r = i * 32 + lrow;
                fa[i] = *(const u32x4_t*)(Ac + r * ROW_BYTES + ((c ^ swz(r)) << 4));
            }
#pragma unroll
            for (int j = 0; j < TNI; ++j) {
                const int r = j * 32 + lrow;
                fb[j] = *(const u32x4_t*)(Bc + r * ROW_BYTES + ((c ^ swz(r)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TMI; ++i)
#pragma unroll
                for (int j = 0; j < TNI; ++j) mfma_chunk<IN>(fa[i], fb[j], acc[i][j]);
        }
        if (more) {
            commit_tile<BM, T>(kca, t, ra, As + (cur ^ 1) * BM * ROW_BYTES);
            commit_tile<BN, T>(kcb, t, rb, Bs + (cur ^ 1) * BN * ROW_BYTES);
        }
        __syncthreads();
        cur ^= 1;
    }

    // Epilogue.  A 32x32 accumulator tile keeps, in register r of lane l, the element at
    // row 8*(r/4) + 4*(l/32) + r%4 and column l%32.
    const float sc = batch_scale(a, b);
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < TNI; ++j) {
            const int64_t gj = sb.r0 + wn * (BN / WN) + j * 32 + lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t gi = sa.r0 + wm * (BM / WM) + i * 32 + 8 * (r / 4) + 4 * lhalf + (r % 4);
                if (gi < a.M && gj < a.N)
                    store_out(a.C, b * a.stride_c + gi * a.ldc + gj, acc[i][j][r] * sc, a.out_dtype);
            }
        }
}

// ------------------------------------------------------------------------------------------------
// Streaming path for M <= 16 (decode-like shapes): the product is bound by reading B once from
// HBM, so there is no LDS staging of B at all.  A workgroup owns SK_COLS columns of C; its waves
// split K, each streaming its share of B with 16-byte loads straight into the B operand of
// v_mfma_f32_16x16x32 while A (M x K, cache resident) supplies the other operand; partial sums
// meet in LDS.  Needs: A row-major, B column-major, 16-byte aligned, K a multiple of 8.
// ------------------------------------------------------------------------------------------------
constexpr int SK_WAVES = 4;       // K split inside the workgroup
constexpr int SK_NB = 2;          // 16-column blocks per wave
constexpr int SK_COLS = 16 * SK_NB;
constexpr int SK_UNROLL = 4;      // k steps of 32 in flight per wave

template <typename IN>
__device__ __forceinline__ void mfma16(const u32x4_t& a, const u32x4_t& b, f32x4_t& c)
{
    if constexpr (IN::ID == GEMM_BF16)
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

template <typename IN>
__global__ __launch_bounds__(SK_WAVES * 64) void k4_skinny(Args a)
{
    __shared__ float part[SK_WAVES][16][SK_COLS + 1];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int l16 = lane & 15, lq = lane >> 4;          // operand row/column and 8-element k group
    const int64_t b = blockIdx.y;
    const int64_t j0 = (int64_t)blockIdx.x * SK_COLS;
    const uint16_t* A = (const uint16_t*)a.A + b * a.stride_a;
    const uint16_t* B = (const uint16_t*)a.B + b * a.stride_b;

    // K is cut into SK_WAVES contiguous ranges, each a multiple of 32
    const int64_t ksteps = (a.K + 31) / 32;
    const int64_t per = (ksteps + SK_WAVES - 1) / SK_WAVES;
    const int64_t kbeg = wave * per * 32;
    const int64_t kend = (kbeg + per * 32 < a.K) ? kbeg + per * 32 : a.K;

    const bool arow = l16 < a.M;
    const uint16_t* ap = A + (int64_t)(arow ? l16 : 0) * a.a_si + lq * 8;
    const uint16_t* bp[SK_NB];
    bool bcol[SK_NB];
#pragma unroll
    for (int n = 0; n < SK_NB; ++n) {
        const int64_t j = j0 + n * 16 + l16;
        bcol[n] = j < a.N;
        bp[n] = B + (bcol[n] ? j : 0) * a.b_sj + lq * 8;
    }

    f32x4_t acc[SK_NB];
#pragma unroll
    for (int n = 0; n < SK_NB; ++n) acc[n] = f32x4_t{0, 0, 0, 0};

    const u32x4_t zero = u32x4_t{0, 0, 0, 0};
    for (int64_t k = kbeg; k < kend; k += 32 * SK_UNROLL) {
        u32x4_t fa[SK_UNROLL], fb[SK_UNROLL][SK_NB];
#pragma unroll
        for (int u = 0; u < SK_UNROLL; ++u) {
            const int64_t kk = k + u * 32 + lq * 8;      // this lane's 8 elements; K % 8 == 0
            const bool in = kk < kend;
            fa[u] = (in && arow) ? *(const u32x4_t*)(ap + k + u * 32) : zero;
#pragma unroll
            for (int n = 0; n < SK_NB; ++n)
                fb[u][n] = (in && bcol[n]) ? __builtin_nontemporal_load((const u32x4_t*)(bp[n] + k + u * 32)) : zero;
        }
#pragma unroll
        for (int u = 0; u < SK_UNROLL; ++u)
#pragma unroll
            for (int n = 0; n < SK_NB; ++n) mfma16<IN>(fa[u], fb[u][n], acc[n]);
    }

    // 16x16 accumulator: register r of lane l holds row 4*(l/16) + r, column l%16
#pragma unroll
    for (int n = 0; n < SK_NB; ++n)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][4 * lq + r][n * 16 + l16] = acc[n][r];
    __syncthreads();
    const float sc = batch_scale(a, b);
    for (int o = t; o < 16 * SK_COLS; o += SK_WAVES * 64) {
        const int i = o / SK_COLS, j = o % SK_COLS;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < SK_WAVES; ++w) v += part[w][i][j];
        if (i < a.M && j0 + j < a.N) store_out(a.C, b * a.stride_c + (int64_t)i * a.ldc + j0 + j, v * sc, a.out_dtype);
    }
}

// ------------------------------------------------------------------------------------------------
constexpr int K4_BM = 256, K4_BN = 256, K4_WM = 2, K4_WN = 2;
constexpr int K4_LDS = 2 * (K4_BM + K4_BN) * ROW_BYTES;

template <typename IN>
static hipError_t launch_general(const Args& a, int vec_mask)
{
    auto kern = k4_mfma<IN, K4_BM, K4_BN, K4_WM, K4_WN>;
    static bool configured = false;   // per instantiation; raising the dynamic-LDS limit is idempotent
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, K4_LDS);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int tiles_m = (int)((a.M + K4_BM - 1) / K4_BM), tiles_n = (int)((a.N + K4_BN - 1) / K4_BN);
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)a.batch, 1), block(K4_WM * K4_WN * 64, 1, 1);
    hipLaunchKernelGGL(kern, grid, block, K4_LDS, a.stream, a, vec_mask, tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t launch_k4(int path, const Args& a)
{
    if (path == MFMA_SKINNY) {
        dim3 grid((unsigned)((a.N + SK_COLS - 1) / SK_COLS), (unsigned)a.batch, 1), block(SK_WAVES * 64, 1, 1);
        if (a.in_dtype == GEMM_BF16) hipLaunchKernelGGL(k4_skinny<BF16>, grid, block, 0, a.stream, a);
        else if (a.in_dtype == GEMM_F16) hipLaunchKernelGGL(k4_skinny<F16>, grid, block, 0, a.stream, a);
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    // general path: `path` carries the operand bitmask of legal 16-byte loads in its upper bits
    const int vec_mask = path >> 8;
    switch (a.in_dtype) {
    case GEMM_BF16: return launch_general<BF16>(a, vec_mask);
    case GEMM_F16: return launch_general<F16>(a, vec_mask);
    case GEMM_FP8_E4M3: return launch_general<E4M3>(a, vec_mask);
    default: return hipErrorInvalidValue;
    }
}

Geometry geometry_k4(int path, const Args& a)
{
    if (path == MFMA_SKINNY)
        return Geometry{16, SK_COLS, 32 * SK_UNROLL, SK_WAVES * 64, 1, (int)sizeof(float) * SK_WAVES * 16 * (SK_COLS + 1),
                        ((a.N + SK_COLS - 1) / SK_COLS) * a.batch};
    const int64_t g = ((a.M + K4_BM - 1) / K4_BM) * ((a.N + K4_BN - 1) / K4_BN) * a.batch;
    const int es = a.in_dtype == GEMM_FP8_E4M3 ? 1 : 2;
    return Geometry{K4_BM, K4_BN, ROW_BYTES / es, K4_WM * K4_WN * 64, 2, K4_LDS, g};
}

}  // namespace gl
