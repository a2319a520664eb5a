// K4 kernels: K3 + "mma" + "ldmatrix.swizzle" (paper Table 1, "Compute & layout"), realised for
// CDNA4 as wave64 MFMA with fp32 accumulators and an LDS operand layout in which the 16-byte
// fragment reads of a wave are bank-conflict free.
//
// Preconditions recorded for this state (Table 1: "tile fits mma", "mma fragment layout";
// Sec. 1: matrix intrinsics need compatible tile shapes, layouts and hardware support):
//   - the input dtype has a matrix instruction (bf16, fp16, OCP e4m3);
//   - the fast kernel needs K contiguous in both operands, 16-byte aligned bases and leading
//     dimensions, and K a whole number of 128-byte slabs; otherwise the masked kernel gathers
//     the offending operand element by element.
//
// Data movement per workgroup and K slab of 128 bytes per row:
//   fast kernel:   global --global_load_lds_dwordx4 (no registers)--> LDS[buf^1]   (next slab)
//   masked kernel: global --> registers --ds_write_b128--> LDS[buf^1]               (next slab)
//   LDS[buf] --ds_read_b128--> MFMA operand registers --> v_mfma_f32_32x32x16       (this slab)
// LDS rows are 128 bytes (eight 16-byte chunks); chunk c of row r lives at chunk position
// c ^ swz(r).
#pragma once
#include <type_traits>

#include "common.hpp"

namespace gl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

constexpr int ROW_BYTES = 128;            // bytes of K per LDS row and per slab
constexpr int CHUNKS = ROW_BYTES / 16;    // 16-byte chunks per row

// XOR mask of row r.  Within any aligned group of 8 rows the masks are a permutation of 0..7, and
// within any aligned group of 16 rows the even rows and the odd rows each get 8 different masks, so
// a column of chunks read by consecutive rows is spread over all banks whether the LDS serves 8
// lanes over 32 banks or 16 lanes over 64 banks per cycle.
__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

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

// Workgroup id -> (tile_m, tile_n).  Hardware hands consecutive workgroup ids to the 8 XCDs in
// turn; ids are first regrouped so that each XCD (own L2) works on one contiguous run of tiles,
// then tiles are walked in bands of GROUP_M tile-rows so that a run reuses few A rows and B columns.
template <int GROUP_M>
__device__ __forceinline__ void tile_of(int pid, int total, int tiles_m, int tiles_n, int& tm, int& tn)
{
    constexpr int XCD = 8;
    const int x = pid % XCD, local = pid / XCD;
    const int base = total / XCD, rem = total % XCD;
    const int id = x * base + (x < rem ? x : rem) + local;
    const int width = GROUP_M * tiles_n;
    const int g = id / width, first = g * GROUP_M;
    const int gsz = (tiles_m - first) < GROUP_M ? (tiles_m - first) : GROUP_M;
    tm = first + (id % width) % gsz;
    tn = (id % width) / gsz;
}

// Epilogue shared by both kernels.  A 32x32 accumulator tile keeps, in register r of lane l, the
// element at row 8*(r/4) + 4*(l/32) + r%4 and column l%32.  The output type is resolved once,
// outside the fully unrolled tile loops, so that every accumulator index is a compile-time constant.
template <int OUT, int TMI, int TNI>
__device__ __forceinline__ void store_tiles_as(const Args& a, int64_t b, const f32x16_t (&acc)[TMI][TNI],
                                               int64_t row0, int64_t col0, int lane, float sc)
{
    const int lrow = lane & 31, lhalf = lane >> 5;
    char* C = (char*)a.C + (b * a.stride_c) * (OUT == GEMM_F32 ? 4 : 2);
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < TNI; ++j) {
            const int64_t gj = col0 + j * 32 + lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t gi = row0 + i * 32 + 8 * (r / 4) + 4 * lhalf + (r % 4);
                if (gi < a.M && gj < a.N) {
                    const float v = acc[i][j][r] * sc;
                    const int64_t idx = gi * a.ldc + gj;
                    if constexpr (OUT == GEMM_F32) ((float*)C)[idx] = v;
                    else if constexpr (OUT == GEMM_BF16) ((uint16_t*)C)[idx] = encode_bf16(v);
                    else ((uint16_t*)C)[idx] = encode_f16(v);
                }
            }
        }
}

template <int TMI, int TNI>
__device__ __forceinline__ void store_tiles(const Args& a, int64_t b, const f32x16_t (&acc)[TMI][TNI],
                                            int64_t row0, int64_t col0, int lane)
{
    const float sc = batch_scale(a, b);
    if (a.out_dtype == GEMM_F32) store_tiles_as<GEMM_F32>(a, b, acc, row0, col0, lane, sc);
    else if (a.out_dtype == GEMM_BF16) store_tiles_as<GEMM_BF16>(a, b, acc, row0, col0, lane, sc);
    else store_tiles_as<GEMM_F16>(a, b, acc, row0, col0, lane, sc);
}

// ------------------------------------------------------------------------------------------------
// Epilogue of the fast kernel.  The fast kernel feeds the B fragment as the first MFMA operand and
// the A fragment as the second, so a 32x32 accumulator tile keeps, in register r of lane l, the
// element at row (of C) l%32 and column 8*(r/4) + 4*(l/32) + r%4: four consecutive columns per
// register quad.  Each wave rounds its accumulators to the output type, parks one 32-row block at a
// time in a private LDS area (row pitch padded by 16 bytes) and writes it out again row by row, so
// that global stores are 16 bytes per lane and whole 128-byte lines per row.
// ------------------------------------------------------------------------------------------------
template <int OUT, int TMI, int TNI>
__device__ __forceinline__ void store_tiles_staged(const Args& a, int64_t b, const f32x16_t (&acc)[TMI][TNI],
                                                   int64_t row0, int64_t col0, int lane, char* stage, bool vec_ok)
{
    constexpr int OB = OUT == GEMM_F32 ? 4 : 2;            // bytes per output element
    constexpr int ROWB = TNI * 32 * OB, PITCH = ROWB + 16; // bytes per staged row
    constexpr int CPR = ROWB / 16, PASSES = 32 * CPR / 64; // 16-byte chunks per row; read passes per block
    constexpr int EPC = 16 / OB;                           // elements per chunk
    const float sc = batch_scale(a, b);
    const int lrow = lane & 31, lhalf = lane >> 5;
    char* C = (char*)a.C + (b * a.stride_c) * OB;
#pragma unroll
    for (int i = 0; i < TMI; ++i) {
#pragma unroll
        for (int j = 0; j < TNI; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float v0 = acc[i][j][4 * g] * sc, v1 = acc[i][j][4 * g + 1] * sc;
                const float v2 = acc[i][j][4 * g + 2] * sc, v3 = acc[i][j][4 * g + 3] * sc;
                char* dst = stage + lrow * PITCH + (j * 32 + 8 * g + 4 * lhalf) * OB;
                if constexpr (OUT == GEMM_F32) {
                    *(f32x4_t*)dst = f32x4_t{v0, v1, v2, v3};
                } else if constexpr (OUT == GEMM_BF16) {
                    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
                    *(bf16x4_t*)dst = bf16x4_t{(__bf16)v0, (__bf16)v1, (__bf16)v2, (__bf16)v3};
                } else {
                    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
                    *(f16x4_t*)dst = f16x4_t{(_Float16)v0, (_Float16)v1, (_Float16)v2, (_Float16)v3};
                }
            }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int q = lane + 64 * p, r = q / CPR, c = q % CPR;
            const u32x4_t w = *(const u32x4_t*)(stage + r * PITCH + c * 16);
            const int64_t gi = row0 + i * 32 + r, gj = col0 + c * EPC;
            if (gi < a.M) {
                char* out = C + (gi * a.ldc + gj) * OB;
                if (vec_ok && gj + EPC <= a.N) {
                    *(u32x4_t*)out = w;
                } else {
#pragma unroll
                    for (int e = 0; e < EPC; ++e)
                        if (gj + e < a.N) {
                            if constexpr (OB == 4) ((uint32_t*)out)[e] = w[e];
                            else ((uint16_t*)out)[e] = (uint16_t)(w[e / 2] >> (16 * (e & 1)));
                        }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Fast kernel: both operands K-contiguous and 16-byte aligned, K a whole number of 128-byte slabs.
//
// Software pipeline, per workgroup and slab s (4 k-steps of 32 bytes of K each; `cur` = LDS buffer
// s%2, `nxt` the other one):
//   k-steps 0..2:  MFMAs of the step, interleaved with the fragment reads of the next step
//   k-step 3:      wait until this wave's loads of slab s+1 have landed and its reads of `cur` have
//                  returned; barrier; then, interleaved with the step's MFMAs: fragment reads of
//                  k-step 0 of slab s+1 from `nxt`, and the direct-to-LDS loads of slab s+2 into `cur`
// so there is one barrier per slab, it sits in the shadow of MFMAs already issued, and no fragment
// read is ever issued later than a full k-step before its use.
// ------------------------------------------------------------------------------------------------
enum { FAST_VEC_C = 1 };   // kernel flag: 16-byte stores to C are legal (base and ldc 16-byte aligned)

template <typename IN, int BM_, int BN_, int WM_, int WN_, int WAVES_PER_SIMD_, int GROUP_M_ = 8>
struct FastCfg {
    using In = IN;
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, GROUP_M = GROUP_M_;
    static constexpr int WAVES_PER_SIMD = WAVES_PER_SIMD_;
    static constexpr int T = WM * WN * 64;
    static constexpr int TMI = BM / WM / 32, TNI = BN / WN / 32;
    static constexpr int LDS_BYTES = 2 * (BM + BN) * ROW_BYTES;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tiles are made of 32x32 MFMA tiles");
    // the epilogue parks 32 rows of fp32 per wave, half of the waves in each LDS buffer
    static_assert((WM * WN / 2) * 32 * (TNI * 32 * 4 + 16) <= (BM + BN) * ROW_BYTES, "epilogue staging must fit");
};

#define GL_SCHED_GROUP(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

template <typename CFG>
__global__ __launch_bounds__(CFG::T) __attribute__((amdgpu_waves_per_eu(CFG::WAVES_PER_SIMD, CFG::WAVES_PER_SIMD)))
void k4_mfma_fast(Args a, int tiles_m, int tiles_n, int flags)
{
    using IN = typename CFG::In;
    constexpr int BM = CFG::BM, BN = CFG::BN, WN = CFG::WN, T = CFG::T, NW = T / 64;
    constexpr int TMI = CFG::TMI, TNI = CFG::TNI;
    constexpr int KE = ROW_BYTES / IN::BYTES;        // K elements per slab
    constexpr int V = 16 / IN::BYTES;                // K elements per chunk
    constexpr int NK = CHUNKS / 2;                   // k-steps per slab
    constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW; // direct loads per wave per slab (8 rows each)
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0 && NW % 2 == 0, "row octets must divide over the waves");
    // Two separately declared buffers, each [A rows | B rows][128 bytes]: distinct objects let the
    // compiler see that a direct load into one never aliases a fragment read from the other, so it
    // does not wait for the loads before the reads.
    constexpr int BUF_BYTES = (BM + BN) * ROW_BYTES;
    __shared__ __attribute__((aligned(1024))) char lds0[BUF_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds1[BUF_BYTES];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int64_t b = blockIdx.y;
    int tm, tn;
    tile_of<CFG::GROUP_M>(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    // ---- global -> LDS, without passing through registers -------------------------------------
    // One wave-wide 16-byte load fills 8 consecutive LDS rows (lane L lands at byte 16*L of the
    // 1 KiB block), so lane L must fetch, for row L/8, the chunk whose swizzled position is L%8.
    // Wave w owns row octets w, w + NW, ...; NW is even, so all its octets share one parity and the
    // lane's chunk index is the same for every one of them.
    const int orow = lane >> 3;                                  // row inside the octet
    const int gchunk = (lane & 7) ^ swz(orow + 8 * (wave & 1));  // chunk this lane fetches
    const char* A = (const char*)a.A + (b * a.stride_a) * IN::BYTES;
    const char* B = (const char*)a.B + (b * a.stride_b) * IN::BYTES;
    const char* pa[LA];
    const char* pb[LB];
#pragma unroll
    for (int n = 0; n < LA; ++n) {
        const int64_t r = m0 + (wave + n * NW) * 8 + orow;       // rows past M are clamped: their products
        pa[n] = A + ((r < a.M ? r : a.M - 1) * a.a_si + gchunk * V) * IN::BYTES;   // are never stored
    }
#pragma unroll
    for (int n = 0; n < LB; ++n) {
        const int64_t r = n0 + (wave + n * NW) * 8 + orow;
        pb[n] = B + ((r < a.N ? r : a.N - 1) * a.b_sj + gchunk * V) * IN::BYTES;
    }
    using gptr = const __attribute__((address_space(1))) void*;
    using lptr = __attribute__((address_space(3))) void*;
    auto issue = [&](int64_t s, char* buf) __attribute__((always_inline)) {
        const int64_t koff = s * ROW_BYTES;
        char* base = buf + wave * 1024;
#pragma unroll
        for (int n = 0; n < LA; ++n)
            __builtin_amdgcn_global_load_lds((gptr)(pa[n] + koff), (lptr)(base + n * NW * 1024), 16, 0, 0);
#pragma unroll
        for (int n = 0; n < LB; ++n)
            __builtin_amdgcn_global_load_lds((gptr)(pb[n] + koff), (lptr)(base + BM * ROW_BYTES + n * NW * 1024), 16, 0, 0);
    };

    // ---- LDS read side: lane reads row (lane % 32) of each 32-row block, chunk 2*ks + lane/32 ---
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int rd_mask = lhalf ^ swz(lrow);
    const int rd_a = (wm * (BM / CFG::WM) + lrow) * ROW_BYTES;
    const int rd_b = (BM + wn * (BN / WN) + lrow) * ROW_BYTES;

    f32x16_t acc[TMI][TNI];
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < TNI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4_t fa[2][TMI], fb[2][TNI];                  // two fragment slots: the step in use, the step in flight
    auto read = [&](const char* base, int ks, int slot) __attribute__((always_inline)) {
        const int pos = ((2 * ks) ^ rd_mask) << 4;
#pragma unroll
        for (int i = 0; i < TMI; ++i) fa[slot][i] = *(const u32x4_t*)(base + rd_a + i * 32 * ROW_BYTES + pos);
#pragma unroll
        for (int j = 0; j < TNI; ++j) fb[slot][j] = *(const u32x4_t*)(base + rd_b + j * 32 * ROW_BYTES + pos);
    };
    auto mfmas = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TMI; ++i)
#pragma unroll
            for (int j = 0; j < TNI; ++j) mfma_chunk<IN>(fb[slot][j], fa[slot][i], acc[i][j]);   // B first: see the epilogue
    };
    constexpr int NMF = TMI * TNI * (IN::BYTES == 1 ? 2 : 1);   // MFMA instructions per k-step
    constexpr int NRD = TMI + TNI;                               // fragment reads per k-step
    constexpr int NLD = LA + LB;                                 // direct loads per slab
    static_assert(NMF > NRD, "the schedule hangs one read on each of the first MFMAs of a step");

    const int64_t nslab = a.K / KE;                  // K is a whole number of slabs
    // `full` = every prefetch of this slab is in range, so the body is free of branches and the
    // requested interleaving can be realised by the instruction scheduler.
    auto slab = [&](auto full, int64_t s, char* cur, char* nxt) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full)::value;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            if (ks + 1 < NK) {
                read(cur, ks + 1, (ks + 1) & 1);
                mfmas(ks & 1);
#pragma unroll
                for (int n = 0; n < NRD; ++n) { GL_SCHED_GROUP(0x008, 1); GL_SCHED_GROUP(0x100, 1); }
                GL_SCHED_GROUP(0x008, NMF - NRD);
            } else {
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                __syncthreads();
                if (FULL || s + 1 < nslab) read(nxt, 0, 0);
                if (FULL || s + 2 < nslab) issue(s + 2, cur);
                mfmas(ks & 1);
                if constexpr (FULL) {
                    constexpr int REST = NMF - NRD, PER = (NLD + REST - 1) / REST;
#pragma unroll
                    for (int n = 0; n < NRD; ++n) { GL_SCHED_GROUP(0x008, 1); GL_SCHED_GROUP(0x100, 1); }
#pragma unroll
                    for (int n = 0; n < REST; ++n) { GL_SCHED_GROUP(0x008, 1); GL_SCHED_GROUP(0x020, PER); }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (nslab > 0) issue(0, lds0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (nslab > 1) issue(1, lds1);
    if (nslab > 0) read(lds0, 0, 0);
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int64_t s = 0;
    for (; s + 3 < nslab; s += 2) {                  // steady state: slabs s and s+1, both with s+2 in range
        slab(yes{}, s, lds0, lds1);
        slab(yes{}, s + 1, lds1, lds0);
    }
    for (; s + 1 < nslab; s += 2) {
        slab(no{}, s, lds0, lds1);
        slab(no{}, s + 1, lds1, lds0);
    }
    if (s < nslab) slab(no{}, s, lds0, lds1);

    // After the barrier of the last slab nobody reads LDS any more: the buffers can hold the
    // epilogue's staging areas, one per wave, half of the waves in each buffer.
    constexpr int STAGE = 32 * (TNI * 32 * 4 + 16);
    char* stage = (wave < NW / 2 ? lds0 : lds1) + (wave % (NW / 2)) * STAGE;
    const int64_t row0 = m0 + wm * (BM / CFG::WM), col0 = n0 + wn * (BN / WN);
    const bool vec_ok = (flags & FAST_VEC_C) != 0;
    if (a.out_dtype == GEMM_F32) store_tiles_staged<GEMM_F32, TMI, TNI>(a, b, acc, row0, col0, lane, stage, vec_ok);
    else if (a.out_dtype == GEMM_BF16) store_tiles_staged<GEMM_BF16, TMI, TNI>(a, b, acc, row0, col0, lane, stage, vec_ok);
    else store_tiles_staged<GEMM_F16, TMI, TNI>(a, b, acc, row0, col0, lane, stage, vec_ok);
}

// ------------------------------------------------------------------------------------------------
// Masked kernel: any layout, any alignment, any K.  An operand whose 16-byte loads are legal
// (bit in vec_mask) is still fetched by chunks; any other operand, and every chunk that crosses
// the end of K, is gathered element by element under a mask.
// ------------------------------------------------------------------------------------------------
struct TileSrc {
    const char* base;   // operand base for this batch item (bytes)
    int64_t sr, sk;     // element strides along rows and along K
    int64_t rows;       // logical rows (M for A, N for B)
    int64_t r0;         // first row of the workgroup tile
    bool vec;           // 16-byte loads along K are legal
};

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
        u32x4_t w = {0, 0, 0, 0};
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

template <typename IN, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM* WN * 64) void k4_mfma_masked(Args a, int vec_mask, int tiles_m, int tiles_n)
{
    constexpr int T = WM * WN * 64;
    constexpr int KE = ROW_BYTES / IN::BYTES;
    constexpr int TMI = BM / WM / 32, TNI = BN / WN / 32;
    constexpr int NCA = BM * CHUNKS / T, NCB = BN * CHUNKS / T;
    __shared__ __attribute__((aligned(16))) char As[2][BM * ROW_BYTES];
    __shared__ __attribute__((aligned(16))) char Bs[2][BN * ROW_BYTES];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t b = blockIdx.y;
    int tm, tn;
    tile_of<8>(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);

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
        commit_tile<BM, T>(kca, t, ra, As[0]);
        commit_tile<BN, T>(kcb, t, rb, Bs[0]);
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
        const char* Ac = As[cur] + (wm * (BM / WM)) * ROW_BYTES;
        const char* Bc = Bs[cur] + (wn * (BN / WN)) * ROW_BYTES;
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
            commit_tile<BM, T>(kca, t, ra, As[cur ^ 1]);
            commit_tile<BN, T>(kcb, t, rb, Bs[cur ^ 1]);
        }
        __syncthreads();
        cur ^= 1;
    }
    store_tiles<TMI, TNI>(a, b, acc, sa.r0 + wm * (BM / WM), sb.r0 + wn * (BN / WN), lane);
}

template <typename IN>
__device__ __forceinline__ void mfma16(const u32x4_t& a, const u32x4_t& b, f32x4_t& c)
{
    if constexpr (IN::ID == GEMM_BF16)
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------------
// Streaming kernel for M <= 16 (decode-like shapes): the product is bound by reading B once from
// HBM.  A workgroup owns a strip of 16*NB columns of C; its WAVES waves split K, partial sums meet
// in LDS at the end.  Needs: A row-major, B column-major, 16-byte aligned, K a multiple of 8.
//
// The B operand of v_mfma_f32_16x16x32 wants, per instruction, 16 columns x 64 bytes of K; fetched
// that way every wave instruction opens 16 separate 64-byte streams 2*ldb bytes apart, and HBM
// delivers about half of what it gives to contiguous reads.  Here a wave instead fetches, per load
// instruction, 64/LPC columns' worth of LPC*16 contiguous bytes (LPC = lanes per column = TK/8),
// parks the registers in a wave-private LDS tile of NB*16 rows (one per column) x TK*2 bytes, and
// reads the MFMA operand layout back from there.  Chunk q (16 bytes) of row c is kept at chunk
// position q ^ (c % 16): writes (16 consecutive q of one row) and operand reads (16 rows at one q)
// are both bank-conflict free.  The tile is private to the wave and LDS serves a wave's requests in
// order, so the main loop has no barrier: waves only meet for the final sum over the K split.
//
// Per wave and tile: NB*TK/32 loads of B stay in flight in registers while the previous tile is
// multiplied; A (M <= 16 rows, cache resident) is fetched straight into the other MFMA operand.
// ------------------------------------------------------------------------------------------------
template <typename IN, int WAVES_, int NB_, int TK_>
struct StreamCfg {
    using In = IN;
    static constexpr int WAVES = WAVES_, NB = NB_, TK = TK_, COLS = 16 * NB_;
    static constexpr int LPC = TK / 8;                     // lanes (16-byte chunks) per column per tile
    static constexpr int CPL = 64 / LPC;                   // columns covered by one load instruction
    static constexpr int NLD = COLS / CPL;                 // B loads per tile per lane
    static constexpr int KS = TK / 32;                     // MFMA k-steps per tile
    static constexpr int TILE_BYTES = COLS * TK * 2;
    static constexpr int LDS_BYTES = WAVES * TILE_BYTES;
    static_assert(LPC >= 16 && LPC <= 64 && (LPC & (LPC - 1)) == 0, "a column's run is 16..64 lanes wide");
    static_assert(WAVES * 16 * (COLS + 1) * 4 <= LDS_BYTES, "the K-split partial sums reuse the tiles");
};

template <typename CFG>
__global__ __launch_bounds__(CFG::WAVES * 64) void k4_stream(Args a)
{
    using IN = typename CFG::In;
    constexpr int WAVES = CFG::WAVES, NB = CFG::NB, TK = CFG::TK, COLS = CFG::COLS;
    constexpr int LPC = CFG::LPC, CPL = CFG::CPL, NLD = CFG::NLD, KS = CFG::KS;
    constexpr int ROWB = TK * 2;                            // bytes per LDS row
    __shared__ __attribute__((aligned(16))) char lds[CFG::LDS_BYTES];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int64_t b = blockIdx.y;
    const int64_t j0 = (int64_t)blockIdx.x * COLS;
    const uint16_t* A = (const uint16_t*)a.A + b * a.stride_a;
    const uint16_t* B = (const uint16_t*)a.B + b * a.stride_b;
    char* tile = lds + wave * CFG::TILE_BYTES;

    // K is cut into WAVES contiguous ranges, each a whole number of 32-element MFMA steps
    const int64_t ksteps = (a.K + 31) / 32;
    const int64_t per = (ksteps + WAVES - 1) / WAVES;
    const int64_t kbeg = wave * per * 32;
    const int64_t kend = (kbeg + per * 32 < a.K) ? kbeg + per * 32 : a.K;

    // load side: lane fetches chunk lc of column (n*CPL + lcol) of the strip; columns past N are
    // clamped (their sums are never stored)
    // (the host has checked that a strip's extent, COLS * ldb elements, fits 32-bit byte offsets)
    const int lcol = lane / LPC, lc = lane % LPC;
    const char* Bs = (const char*)(B + j0 * a.b_sj);       // wave-uniform base of the strip
    uint32_t bo[NLD];
    int wr[NLD];
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
        const int c = n * CPL + lcol;
        const int64_t cc = j0 + c < a.N ? c : a.N - 1 - j0;
        bo[n] = (uint32_t)((cc * a.b_sj + lc * 8) * 2);
        wr[n] = c * ROWB + ((lc ^ (c & 15)) << 4);
    }
    // operand side: lane (l16, lq) holds, for k-step s, chunk 4s+lq of row l16 (A) / column l16 (B)
    const uint16_t* ap = A + (int64_t)(l16 < a.M ? l16 : a.M - 1) * a.a_si + lq * 8;
    const int rd = l16 * ROWB;

    f32x4_t acc[NB];
#pragma unroll
    for (int n = 0; n < NB; ++n) acc[n] = f32x4_t{0, 0, 0, 0};
    const u32x4_t zero = {0, 0, 0, 0};
    u32x4_t rb[NLD], ra[KS];

    // `full`: the whole tile lies inside [kbeg, kend), no lane needs a mask
    auto fetch = [&](auto full, int64_t k) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full)::value;
#pragma unroll
        for (int n = 0; n < NLD; ++n) {
            if (FULL || k + lc * 8 < kend) rb[n] = __builtin_nontemporal_load((const u32x4_t*)(Bs + k * 2 + bo[n]));
            else rb[n] = zero;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (FULL || k + s * 32 + lq * 8 < kend) ra[s] = *(const u32x4_t*)(ap + k + s * 32);
            else ra[s] = zero;
        }
    };
    auto park = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < NLD; ++n) *(u32x4_t*)(tile + wr[n]) = rb[n];
    };
    auto multiply = [&](const u32x4_t (&fa)[KS]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                const u32x4_t fb = *(const u32x4_t*)(tile + n * 16 * ROWB + rd + (((4 * s + lq) ^ l16) << 4));
                mfma16<IN>(fa[s], fb, acc[n]);
            }
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;

    // Tile i is parked and multiplied while the loads of tile i+1 are in flight.  The steady-state
    // loop runs over whole tiles only and is free of branches; a ragged last tile is fetched under
    // masks after it.
    const int64_t span = kend > kbeg ? kend - kbeg : 0;
    const int64_t nfull = span / TK;
    const bool ragged = span % TK != 0;
    int64_t k = kbeg;
    if (nfull > 0) {
        fetch(yes{}, k);
        for (int64_t i = 1; i < nfull; ++i) {
            u32x4_t fa[KS];
#pragma unroll
            for (int s = 0; s < KS; ++s) fa[s] = ra[s];
            park();
            k += TK;
            fetch(yes{}, k);
            multiply(fa);
        }
        u32x4_t fa[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) fa[s] = ra[s];
        park();
        k += TK;
        if (ragged) fetch(no{}, k);
        multiply(fa);
    } else if (ragged) {
        fetch(no{}, k);
    }
    if (ragged) {
        park();
        multiply(ra);
    }

    // 16x16 accumulator: register r of lane l holds row 4*(l/16) + r, column l%16
    __syncthreads();
    float* part = (float*)lds;
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[(wave * 16 + 4 * lq + r) * (COLS + 1) + n * 16 + l16] = acc[n][r];
    __syncthreads();
    const float sc = batch_scale(a, b);
    for (int o = t; o < 16 * COLS; o += WAVES * 64) {
        const int i = o / COLS, j = o % COLS;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += part[(w * 16 + i) * (COLS + 1) + j];
        if (i < a.M && j0 + j < a.N) store_out(a.C, b * a.stride_c + (int64_t)i * a.ldc + j0 + j, v * sc, a.out_dtype);
    }
}

}  // namespace gl
