// K4 kernels: K3 + "mma" + "ldmatrix.swizzle" (paper Table 1, "Compute & layout"), realised for
// CDNA4 as wave64 MFMA with fp32 accumulators and an LDS operand layout in which the 16-byte
// fragment reads of a wave are bank-conflict free.
//
// Preconditions recorded for this state (Table 1: "tile fits mma", "mma fragment layout"; Sec. 1):
//   - the input dtype has a matrix instruction (bf16, fp16, OCP e4m3);
//   - the fast kernel needs K contiguous in both operands, 16-byte aligned bases and leading
//     dimensions, and K a whole number of 128-byte slabs; otherwise the masked kernel gathers
//     the offending operand element by element.
//
// Data movement per workgroup and K slab of 128 bytes per row:
//   fast kernel:   global --global_load_lds_dwordx4 (no registers)--> LDS[buf^1]   (next slab)
//   masked kernel: global --> registers --ds_write_b128--> LDS[buf^1]               (next slab)
//   LDS[buf] --ds_read_b128--> MFMA operand registers --> v_mfma_f32_32x32x16       (this slab)
//                              (bf16 / fp16 on 256 x 256 tiles, one tile per workgroup: v_mfma_f32_16x16x32, see FastCfg)
// LDS rows are 128 bytes (eight 16-byte chunks); chunk c of row r lives at chunk position
// c ^ swz(r).
#pragma once
#include <type_traits>
#include <utility>

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
    } else if constexpr (IN::ID == GEMM_F32) {
        // fp32 operands: the chunk holds four k values, one v_mfma_f32_32x32x2_f32 (K = 2: one k per lane half) each
#pragma unroll
        for (int e = 0; e < 4; ++e)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]), c, 0, 0, 0);
    } else {
        const long alo = (long)(((uint64_t)a.y << 32) | a.x), ahi = (long)(((uint64_t)a.w << 32) | a.z);
        const long blo = (long)(((uint64_t)b.y << 32) | b.x), bhi = (long)(((uint64_t)b.w << 32) | b.z);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(alo, blo, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(ahi, bhi, c, 0, 0, 0);
    }
}

// Workgroup id -> (batch item, tile_m, tile_n) on a one-dimensional grid of tiles_m*tiles_n*batch
// workgroups.  Hardware hands consecutive workgroup ids to the 8 XCDs in turn; ids are first
// regrouped so that each XCD (own L2) works on one contiguous run of the (batch, tile) sequence --
// whole problems when there are at least 8 of them, so that every operand tile is fetched into one
// L2 only -- then the tiles of a problem are walked in bands of GROUP_M tile-rows so that a run
// reuses few A rows and B columns.
template <int GROUP_M>
__device__ __forceinline__ void tile_of(int pid, int total, int tiles_m, int tiles_n, int64_t& b, int& tm, int& tn)
{
    constexpr int XCD = 8;
    const int x = pid % XCD, local = pid / XCD;
    const int base = total / XCD, rem = total % XCD;
    const int flat = x * base + (x < rem ? x : rem) + local;
    const int per = tiles_m * tiles_n;
    b = __builtin_amdgcn_readfirstlane(flat / per);     // wave-uniform by construction: keep it scalar
    const int id = flat % per;
    const int width = GROUP_M * tiles_n;
    const int g = id / width, first = g * GROUP_M;
    const int gsz = (tiles_m - first) < GROUP_M ? (tiles_m - first) : GROUP_M;
    tm = __builtin_amdgcn_readfirstlane(first + (id % width) % gsz);
    tn = __builtin_amdgcn_readfirstlane((id % width) / gsz);
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
                    const float v = acc[i][j][r] * sc + (a.bias ? a.bias[gj] : 0.0f);
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
// that global stores are 16 bytes per lane and whole 128-byte lines per row (also when C's rows are
// aligned to an element only: then the stores are declared under-aligned).
// ------------------------------------------------------------------------------------------------
template <int OUT, bool INTERIOR, int TMI, int TNI>
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
    // bias of the four columns a lane holds per (column tile, register quad), the same for every row block
    f32x4_t bv[TNI][4];
#pragma unroll
    for (int j = 0; j < TNI; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bv[j][g] = f32x4_t{0, 0, 0, 0};
            if (a.bias) {
                const int64_t gj = col0 + j * 32 + 8 * g + 4 * lhalf;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (INTERIOR || gj + c < a.N) bv[j][g][c] = a.bias[gj + c];
            }
        }
#pragma unroll
    for (int i = 0; i < TMI; ++i) {
#pragma unroll
        for (int j = 0; j < TNI; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float v0 = acc[i][j][4 * g] * sc + bv[j][g][0], v1 = acc[i][j][4 * g + 1] * sc + bv[j][g][1];
                const float v2 = acc[i][j][4 * g + 2] * sc + bv[j][g][2], v3 = acc[i][j][4 * g + 3] * sc + bv[j][g][3];
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
        if constexpr (INTERIOR) {
            // the wave's whole sub-tile lies inside C and 16-byte stores are legal: no masks, all reads
            // of the block in flight before the first store
            u32x4_t w[PASSES];
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int q = lane + 64 * p;
                w[p] = *(const u32x4_t*)(stage + (q / CPR) * PITCH + (q % CPR) * 16);
            }
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int q = lane + 64 * p;
                *(u32x4_t*)(C + ((row0 + i * 32 + q / CPR) * a.ldc + col0 + (q % CPR) * EPC) * OB) = w[p];
            }
            continue;
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int q = lane + 64 * p, r = q / CPR, c = q % CPR;
            const u32x4_t w = *(const u32x4_t*)(stage + r * PITCH + c * 16);
            const int64_t gi = row0 + i * 32 + r, gj = col0 + c * EPC;
            if (gi < a.M) {
                char* out = C + (gi * a.ldc + gj) * OB;
                if (gj + EPC <= a.N) {
                    // C rows aligned to an element only: the same 16 bytes per lane, declared under-aligned
                    // (global memory takes vector stores at any element boundary; they cost more line splits)
                    typedef u32x4_t __attribute__((aligned(2))) u32x4_a2_t;
                    typedef u32x4_t __attribute__((aligned(4))) u32x4_a4_t;
                    if (vec_ok) *(u32x4_t*)out = w;
                    else if constexpr (OB == 4) *(u32x4_a4_t*)out = w;
                    else *(u32x4_a2_t*)out = w;
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

// The same epilogue for 16 x 16 accumulator tiles (v_mfma_f32_16x16x32 with the B fragment first): register c of lane l
// holds the element at row (of C) l%16 and column 4*(l/16) + c of its tile.  Two rows of tiles make one staged
// block of 32 rows; the way back out of the staging area is the one above.
template <int OUT, bool INTERIOR, int TMI, int TNI>
__device__ __forceinline__ void store_tiles_staged(const Args& a, int64_t b, const f32x4_t (&acc)[TMI][TNI],
                                                   int64_t row0, int64_t col0, int lane, char* stage, bool vec_ok)
{
    constexpr int OB = OUT == GEMM_F32 ? 4 : 2;            // bytes per output element
    constexpr int ROWB = TNI * 16 * OB, PITCH = ROWB + 16; // bytes per staged row
    constexpr int CPR = ROWB / 16, PASSES = 32 * CPR / 64; // 16-byte chunks per row; read passes per block
    constexpr int EPC = 16 / OB;                           // elements per chunk
    static_assert(TMI % 2 == 0, "a staged block is two rows of tiles");
    const float sc = batch_scale(a, b);
    const int lrow = lane & 15, lq = lane >> 4;
    char* C = (char*)a.C + (b * a.stride_c) * OB;
    f32x4_t bv[TNI];                                       // bias of the four columns a lane holds per column tile
#pragma unroll
    for (int j = 0; j < TNI; ++j) {
        bv[j] = f32x4_t{0, 0, 0, 0};
        if (a.bias) {
            const int64_t gj = col0 + j * 16 + 4 * lq;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (INTERIOR || gj + c < a.N) bv[j][c] = a.bias[gj + c];
        }
    }
#pragma unroll
    for (int ib = 0; ib < TMI / 2; ++ib) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int j = 0; j < TNI; ++j) {
                const f32x4_t& t = acc[2 * ib + ii][j];
                const float v0 = t[0] * sc + bv[j][0], v1 = t[1] * sc + bv[j][1], v2 = t[2] * sc + bv[j][2], v3 = t[3] * sc + bv[j][3];
                char* dst = stage + (ii * 16 + lrow) * PITCH + (j * 16 + 4 * lq) * OB;
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
        if constexpr (INTERIOR) {
            u32x4_t w[PASSES];
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int q = lane + 64 * p;
                w[p] = *(const u32x4_t*)(stage + (q / CPR) * PITCH + (q % CPR) * 16);
            }
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int q = lane + 64 * p;
                *(u32x4_t*)(C + ((row0 + ib * 32 + q / CPR) * a.ldc + col0 + (q % CPR) * EPC) * OB) = w[p];
            }
            continue;
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int q = lane + 64 * p, r = q / CPR, c = q % CPR;
            const u32x4_t w = *(const u32x4_t*)(stage + r * PITCH + c * 16);
            const int64_t gi = row0 + ib * 32 + r, gj = col0 + c * EPC;
            if (gi < a.M) {
                char* out = C + (gi * a.ldc + gj) * OB;
                if (gj + EPC <= a.N) {
                    typedef u32x4_t __attribute__((aligned(2))) u32x4_a2_t;
                    typedef u32x4_t __attribute__((aligned(4))) u32x4_a4_t;
                    if (vec_ok) *(u32x4_t*)out = w;
                    else if constexpr (OB == 4) *(u32x4_a4_t*)out = w;
                    else *(u32x4_a2_t*)out = w;
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
// (Sizes below are those of the 256-tile configuration.)
// One workgroup = 4 waves (one per SIMD) on a 256x256 tile of C, each wave on a 128x128 quarter =
// 4x4 accumulator tiles of 32x32.  K advances in slabs of 128 bytes per row.  LDS is a ring of five
// 32 KB regions, each one operand slab (256 rows x 128 bytes); operand slab q (A of slab s: q = 2s,
// B of slab s: q = 2s+1) lives in region q % 5, so that while slab s is multiplied its successor is
// complete or landing and the slab after that is already being fetched:
//
//      region of      A_s    B_s    A_s+1   B_s+1   (fifth: held B_s-1, free since the last barrier)
//      during slab s  read   read   landed  landing  receives A_s+2;   B_s+2 goes to A_s's region
//                                                     once slab s has been read (after the barrier)
//
// Global -> LDS uses buffer loads that write LDS directly (no registers); one wave instruction
// fills 8 consecutive LDS rows, and the lane -> global chunk assignment applies the swizzle.  The
// loads of a slab are issued in four groups spread over the slab's k-steps, so the memory pipe sees
// an even stream instead of a burst per slab.  Rows past the end of the matrix lie outside the
// buffer resource and read as zero.
//
// Per slab there is one barrier; before it a wave waits until all but its youngest 8 loads (the
// A_s+2 group) have landed and its own LDS reads have returned.  The barrier is a bare s_barrier: a
// fence would drain the loads that are meant to stay in flight.  Fragment reads run one k-step ahead
// of the MFMAs that use them, in two register slots.
//
// A k-step is 32 bytes of K per lane half for 2-byte types (one chunk per lane, v_mfma 32x32x16) and
// 64 bytes for e4m3 (two chunks per lane, v_mfma_scale 32x32x64 with unit scales: the form that runs
// at twice the 16-bit rate on gfx950; the 32x32x16 fp8 form runs at the 16-bit rate).
// ------------------------------------------------------------------------------------------------
enum {
    FAST_VEC_C = 1,          // kernel flag: 16-byte stores to C are legal (base and ldc 16-byte aligned)
    FAST_PLAIN_RASTER = 2    // kernel flag: workgroup i takes tile i in row-major order (a validated simplification)
};

typedef __attribute__((ext_vector_type(8))) int i32x8_t;

// One 16x16x32 step (two-byte types): `a` supplies accumulator columns, `b` accumulator rows, as below.
template <typename IN>
__device__ __forceinline__ void mfma_step16(const u32x4_t& a, const u32x4_t& b, f32x4_t& c)
{
    if constexpr (IN::ID == GEMM_BF16) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

template <typename IN> struct Frag { static constexpr int CPS = IN::BYTES == 1 ? 2 : 1; u32x4_t c[CPS]; };

// acc += a . b^T for one k-step; `a` supplies accumulator columns, `b` accumulator rows (see the
// epilogue).  Which k a lane's bytes stand for is irrelevant as long as both operands agree.
template <typename IN>
__device__ __forceinline__ void mfma_step(const Frag<IN>& a, const Frag<IN>& b, f32x16_t& c)
{
    if constexpr (IN::ID == GEMM_BF16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a.c[0]), __builtin_bit_cast(bf16x8_t, b.c[0]), c, 0, 0, 0);
    } else if constexpr (IN::ID == GEMM_F16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a.c[0]), __builtin_bit_cast(f16x8_t, b.c[0]), c, 0, 0, 0);
    } else {
        const i32x8_t av = {(int)a.c[0].x, (int)a.c[0].y, (int)a.c[0].z, (int)a.c[0].w, (int)a.c[1].x, (int)a.c[1].y, (int)a.c[1].z, (int)a.c[1].w};
        const i32x8_t bv = {(int)b.c[0].x, (int)b.c[0].y, (int)b.c[0].z, (int)b.c[0].w, (int)b.c[1].x, (int)b.c[1].y, (int)b.c[1].z, (int)b.c[1].w};
        // cbsz = blgp = 0 select e4m3 for both operands; scale exponents 127 (E8M0) = 2^0
        c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
    }
}

#define GL_SCHED_GROUP(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// Requested issue order of one k-step: NMF MFMAs, the NRD LDS reads (0x100) behind the first of them
// (one each, or more where there are more reads than MFMAs), NLOADS direct loads (VMEM, 0x020) spread
// evenly over all of them.
template <int NMF, int NRD, int NLOADS, int N = 0>
__device__ __forceinline__ void sched_kstep()
{
    if constexpr (N < NMF) {
        constexpr int RPM = (NRD + NMF - 1) / NMF;
        constexpr int R = NRD - N * RPM >= RPM ? RPM : (NRD - N * RPM > 0 ? NRD - N * RPM : 0);
        GL_SCHED_GROUP(0x008, 1);
        if constexpr (R > 0) GL_SCHED_GROUP(0x100, R);
        constexpr int L = ((N + 1) * NLOADS) / NMF - (N * NLOADS) / NMF;
        if constexpr (L > 0) GL_SCHED_GROUP(0x020, L);
        sched_kstep<NMF, NRD, NLOADS, N + 1>();
    }
}

template <int... KS, typename F>
__device__ __forceinline__ void for_each_step(std::integer_sequence<int, KS...>, F&& f)
{
    (f(std::integral_constant<int, KS>{}), ...);
}

// SWIZZLE and OVERLAP are on in the expert state.  Switching one off is one edge of the backward walk
// from it (paper Sec. 3.2); the result goes through the gate like any state, and the latency it costs
// is the evidence for what that optimisation buys on this hardware.
//   SWIZZLE = false: LDS rows keep their chunks in order; a wave's operand read then hits the same
//                    banks from all 32 rows
//   OVERLAP = false: every group of direct loads is waited for right after it is issued, so no load is
//                    in flight while MFMAs issue
//
// TILE is the side of the square workgroup tile: 256 (one workgroup per CU, 128x128 per wave, all of
// LDS: the compute-bound shape) or 128 (64x64 per wave, half the LDS, two workgroups per CU that cover
// each other's prologue, epilogue and memory waits: for short K, or when 256-tiles would leave CUs idle).
//
// CONV: the A operand is gathered from the activations of a convolution layer (ConvGeom): row m is
// output pixel (n, p, q), K slab s is one tap's run of 128 bytes of channels.  Everything after the
// loads (LDS layout, ring, MFMAs, epilogue) is the matrix product's.
//
// MI16: the matrix instruction is v_mfma_f32_16x16x32 (two-byte types) instead of 32x32x16: the wave's 128 x 128
// quarter is 8 x 8 accumulator tiles of 16 x 16, a k-step is 64 bytes of K.  Same flops per cycle, same LDS bytes per
// flop, half the accumulator traffic per flop: under the package power limit the chip holds a higher clock with
// it (register-resident loops on N(0,1)/sqrt(K) operands: 2017 against 1743 TFLOP/s).
template <typename IN, int TILE_ = 256, int GROUP_M_ = 8, bool SWIZZLE_ = true, bool OVERLAP_ = true, int PRE_ = 0, bool CONV_ = false,
          bool MI16_ = false>
struct FastCfg {
    using In = IN;
    static constexpr bool SWIZZLE = SWIZZLE_, OVERLAP = OVERLAP_, CONV = CONV_, MI16 = MI16_;
    static constexpr int PRE_BARRIER_MFMAS = PRE_;
    static constexpr int BM = TILE_, BN = TILE_, WM = 2, WN = 2, GROUP_M = GROUP_M_;
    static constexpr int T = WM * WN * 64;
    static constexpr int TR = MI16_ ? 16 : 32;           // rows (and columns) of an accumulator tile
    static constexpr int TMI = BM / WM / TR, TNI = BN / WN / TR;
    static_assert(!MI16_ || IN::BYTES == 2, "the 16x16x32 instruction used here is the two-byte one");
    // DEPTH = slabs ahead of the one in use that the ring holds or is being sent (the last of them half: A only)
    static constexpr int DEPTH = 2;
    static constexpr int REGION = TILE_ * ROW_BYTES, REGIONS = 2 * DEPTH + 1;
    static constexpr int LDS_BYTES = REGIONS * REGION;
    static constexpr int WAVES_PER_SIMD = TILE_ == 256 ? 1 : 2;
    static_assert(TILE_ == 256 || TILE_ == 128, "square tiles of 256 or 128");
    // the epilogue parks 32 rows of fp32 per wave, one wave per region
    static_assert(32 * (BN / WN * 4 + 16) <= REGION, "epilogue staging must fit a region");
};

// 128-tiles with a ring of nine regions (144 KB: one workgroup per CU), for products that give each CU at most one
// 128-tile anyway: the second workgroup that would hide this one's memory waits is not there, so the LDS it would
// have used holds two more slabs of prefetch (distance 3.5 slabs instead of 1.5).
template <typename IN>
struct FastCfgDeep : FastCfg<IN, 128> {
    static constexpr int DEPTH = 4;
    static constexpr int REGIONS = 2 * DEPTH + 1;
    static constexpr int LDS_BYTES = REGIONS * FastCfg<IN, 128>::REGION;
    static constexpr int WAVES_PER_SIMD = 1;
};

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <typename CFG>
__global__ __launch_bounds__(CFG::T) __attribute__((amdgpu_waves_per_eu(CFG::WAVES_PER_SIMD, CFG::WAVES_PER_SIMD)))
void k4_mfma_fast(Args a, int tiles_m, int tiles_n, int flags)
{
    using IN = typename CFG::In;
    constexpr int BM = CFG::BM, BN = CFG::BN, WN = CFG::WN, NW = CFG::T / 64;
    constexpr int TMI = CFG::TMI, TNI = CFG::TNI, REGION = CFG::REGION;
    constexpr int KE = ROW_BYTES / IN::BYTES;            // K elements per slab
    constexpr int V = 16 / IN::BYTES;                    // K elements per chunk
    constexpr int CPS = Frag<IN>::CPS;                   // chunks per lane per k-step
    constexpr int TR = CFG::TR, LG = 64 / TR;            // rows of an accumulator tile; lane groups along K (2 or 4)
    constexpr int NK = CHUNKS / (LG * CPS);              // k-steps per slab
    constexpr int LD = BM / 8 / NW;                      // direct loads per wave per operand slab
    constexpr int D = CFG::DEPTH, R = CFG::REGIONS;      // slabs of prefetch; regions of the ring
    static_assert(BM == BN && NW == 4 && LD % 2 == 0, "the ring schedule is written for square tiles and four waves");
    static_assert(R == 2 * D + 1 && (R == 5 || R == 9) && (2 * D - 1) * LD < 64, "five or nine regions; waits count loads in six bits");
    // (one object per region: the compiler then knows that a load into one region and a read from another cannot
    // touch the same bytes, and waits for no load on its own account)
    __shared__ __attribute__((aligned(1024))) char r0[REGION];
    __shared__ __attribute__((aligned(1024))) char r1[REGION];
    __shared__ __attribute__((aligned(1024))) char r2[REGION];
    __shared__ __attribute__((aligned(1024))) char r3[REGION];
    __shared__ __attribute__((aligned(1024))) char r4[REGION];
    __shared__ __attribute__((aligned(1024))) char r5[R > 5 ? REGION : 1024];   // (never referenced with five regions)
    __shared__ __attribute__((aligned(1024))) char r6[R > 5 ? REGION : 1024];
    __shared__ __attribute__((aligned(1024))) char r7[R > 5 ? REGION : 1024];
    __shared__ __attribute__((aligned(1024))) char r8[R > 5 ? REGION : 1024];
    auto region = [&](auto idx) __attribute__((always_inline)) -> char* {        // region idx mod R, known at compile time
        constexpr int i = decltype(idx)::value % R;
        if constexpr (i == 0) return r0; else if constexpr (i == 1) return r1; else if constexpr (i == 2) return r2;
        else if constexpr (i == 3) return r3; else if constexpr (i == 4) return r4; else if constexpr (i == 5) return r5;
        else if constexpr (i == 6) return r6; else if constexpr (i == 7) return r7; else return r8;
    };

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;
    int64_t b;
    int tm, tn;
    if (flags & FAST_PLAIN_RASTER) {
        const int per = tiles_m * tiles_n, id = (int)blockIdx.x % per;
        b = (int)blockIdx.x / per;
        tm = id / tiles_n;
        tn = id % tiles_n;
    } else {
        tile_of<CFG::GROUP_M>(blockIdx.x, (int)gridDim.x, tiles_m, tiles_n, b, tm, tn);
    }
    // Integer division runs on the vector unit and the two forms may be merged by a select: say once
    // more, after the merge, that the coordinates are wave-uniform, or every buffer load below is
    // wrapped in a loop over the lanes' "different" resources.
    b = __builtin_amdgcn_readfirstlane((int)b);
    tm = __builtin_amdgcn_readfirstlane(tm);
    tn = __builtin_amdgcn_readfirstlane(tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    // ---- global -> LDS ---------------------------------------------------------------------------
    // One buffer resource per operand, based at the tile's first row and ending with the matrix.
    // A wave-wide 16-byte load lands lane L at byte 16*L of a 1 KiB block = 8 LDS rows, so lane L
    // fetches, for row L/8 of the octet, the chunk whose swizzled position is L%8.  Wave w owns row
    // octets w, w+4, ...: all of one parity, so one per-lane offset serves every load; the octet and
    // the slab enter through the scalar offset.  (The host has checked that a tile's extent fits 32
    // bits of byte offset.)
    const int orow = lane >> 3;
    const int gchunk = (lane & 7) ^ (CFG::SWIZZLE ? swz(orow + 8 * (wave & 1)) : 0);
    const char* A = CFG::CONV ? (const char*)a.A : (const char*)a.A + (b * a.stride_a + m0 * a.a_si) * IN::BYTES;
    const char* B = (const char*)a.B + (b * a.stride_b + n0 * a.b_sj) * IN::BYTES;
    const int64_t bytes_a = CFG::CONV ? (int64_t)a.conv.x_bytes : ((a.M - 1 - m0) * a.a_si + a.K) * IN::BYTES;
    const int64_t bytes_b = ((a.N - 1 - n0) * a.b_sj + a.K) * IN::BYTES;
    constexpr int64_t CAP = 0xFFFFFFFFll;
    constexpr int RSRC_FLAGS = 0x00020000;               // raw buffer, 32-bit data format
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, (int)(uint32_t)(bytes_a < CAP ? bytes_a : CAP), RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc((void*)B, 0, (int)(uint32_t)(bytes_b < CAP ? bytes_b : CAP), RSRC_FLAGS);
    const int voff_a = (int)((orow * a.a_si + gchunk * V) * IN::BYTES);
    const int voff_b = (int)((orow * a.b_sj + gchunk * V) * IN::BYTES);
    const int oct_a = (int)(8 * a.a_si * IN::BYTES), oct_b = (int)(8 * a.b_sj * IN::BYTES);   // bytes per row octet
    using lptr = __attribute__((address_space(3))) void*;
    // Gather (CONV): per load of this wave (row octet wave + n*NW, row orow of it) the lane keeps the
    // byte offset of its output pixel's window origin (channel chunk included; the origin may lie in
    // the padding, a tap's offset is only added when the tap is inside the image) and the origin's
    // input coordinates.  Rows past M get coordinates that fail every tap's range test.
    constexpr int NCONV = CFG::CONV ? LD : 1;
    constexpr int OUT_OF_RANGE = (int)0x80000000;          // as an unsigned offset: past any x below 2 GiB
    int conv_base[NCONV], conv_h[NCONV], conv_w[NCONV];
    if constexpr (CFG::CONV) {
        const ConvGeom& g = a.conv;
#pragma unroll
        for (int n = 0; n < LD; ++n) {
            const int64_t m = m0 + 8 * (wave + n * NW) + orow;
            const bool in = m < a.M;
            const int mm = in ? (int)m : 0;
            const int img = mm / (g.P * g.Q), rem = mm - img * (g.P * g.Q);
            const int p = rem / g.Q, q = rem - p * g.Q;
            const int h0 = p * g.stride_h - g.pad_h;
            conv_h[n] = in ? h0 : -(1 << 24);
            conv_w[n] = q * g.stride_w - g.pad_w;
            conv_base[n] = (((img * g.H + h0) * g.W + conv_w[n]) * g.C + gchunk * V) * IN::BYTES;
        }
    }
    // loads [lo, hi) of this wave's share of operand slab s into region `reg`
    auto issue_a = [&](int64_t s, char* reg, int lo, int hi) __attribute__((always_inline)) {
        if constexpr (CFG::CONV) {
            const ConvGeom& g = a.conv;
            const int tap = (int)s / g.slabs_per_tap, cb = (int)s - tap * g.slabs_per_tap;
            const int r = tap / g.S, sx = tap - r * g.S;
            const int delta = (r * g.W + sx) * g.C * IN::BYTES + cb * ROW_BYTES;
#pragma unroll
            for (int n = lo; n < hi; ++n) {
                const bool inside = (unsigned)(conv_h[n] + r) < (unsigned)g.H && (unsigned)(conv_w[n] + sx) < (unsigned)g.W;
                // (a named value: with the select written as the builtin's argument the host pass drops the kernel's stub)
                const int voff = inside ? conv_base[n] + delta : OUT_OF_RANGE;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lptr)(reg + (wave + n * NW) * 1024), 16, voff, 0, 0, 0);
            }
        } else {
            const int k0 = (int)(s * ROW_BYTES);
#pragma unroll
            for (int n = lo; n < hi; ++n)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lptr)(reg + (wave + n * NW) * 1024), 16, voff_a, k0 + (wave + n * NW) * oct_a, 0, 0);
        }
    };
    auto issue_b = [&](int64_t s, char* reg, int lo, int hi) __attribute__((always_inline)) {
        const int k0 = (int)(s * ROW_BYTES);
#pragma unroll
        for (int n = lo; n < hi; ++n)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lptr)(reg + (wave + n * NW) * 1024), 16, voff_b, k0 + (wave + n * NW) * oct_b, 0, 0);
    };

    // ---- LDS -> registers: lane reads row (lane % 32) of each 32-row block, CPS chunks starting at
    // chunk CPS * (2*ks + lane/32) ---------------------------------------------------------------
    const int lrow = lane & (TR - 1), lhalf = lane / TR;
    const int rd_mask = (lhalf * CPS) ^ (CFG::SWIZZLE ? swz(lrow) : 0);
    const int rd_a = (wm * (BM / CFG::WM) + lrow) * ROW_BYTES;
    const int rd_b = (wn * (BN / WN) + lrow) * ROW_BYTES;

    using AccT = std::conditional_t<CFG::MI16, f32x4_t, f32x16_t>;
    constexpr int ACC_REGS = CFG::MI16 ? 4 : 16;
    AccT acc[TMI][TNI];
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < TNI; ++j)
#pragma unroll
            for (int r = 0; r < ACC_REGS; ++r) acc[i][j][r] = 0.0f;

    Frag<IN> fa[2][TMI], fb[2][TNI];                 // two fragment slots: the step in use, the step in flight
    auto read = [&](const char* ra, const char* rb, int ks, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < CPS; ++q) {
            const int pos = ((LG * CPS * ks + q) ^ rd_mask) << 4;
#pragma unroll
            for (int j = 0; j < TNI; ++j) fb[slot][j].c[q] = *(const u32x4_t*)(rb + rd_b + j * TR * ROW_BYTES + pos);
#pragma unroll
            for (int i = 0; i < TMI; ++i) fa[slot][i].c[q] = *(const u32x4_t*)(ra + rd_a + i * TR * ROW_BYTES + pos);
        }
    };
    // B first: see the epilogue.  Columns are walked back and forth so that consecutive MFMAs share
    // one operand.
    auto mfmas = [&](int slot, int lo, int hi) __attribute__((always_inline)) {    // MFMAs lo..hi-1 of a k-step
#pragma unroll
        for (int i = 0; i < TMI; ++i)
#pragma unroll
            for (int jj = 0; jj < TNI; ++jj) {
                const int j = (i & 1) ? TNI - 1 - jj : jj;
                if (i * TNI + jj >= lo && i * TNI + jj < hi) {
                    if constexpr (CFG::MI16) mfma_step16<IN>(fb[slot][j].c[0], fa[slot][i].c[0], acc[i][j]);
                    else mfma_step<IN>(fb[slot][j], fa[slot][i], acc[i][j]);
                }
            }
    };
    constexpr int NMF = TMI * TNI;                   // MFMA instructions per k-step
    constexpr int NRD = (TMI + TNI) * CPS;           // fragment reads per k-step
    constexpr int HALF = LD / 2;                     // loads per issue group
    // issue groups of a slab, in order (D = 2 in the five-region ring): B_s+D-1 second half, A_s+D first half,
    // A_s+D second half (before the barrier, spread over the first NK-1 k-steps), B_s+D first half (after it, last
    // k-step, into the region A_s leaves).  Operand slab q lives in region q mod R (A_s: q = 2s, B_s: 2s+1).
    constexpr int GROUPS_PER_STEP = NK > 1 ? (3 + NK - 2) / (NK - 1) : 3;
    static_assert(NK >= 2, "the barrier k-step is not the one that prefetches");

    const int64_t nslab = a.K / KE;                  // K is a whole number of slabs
    // `first`: slab 0 in the branch-free form; its pre-barrier loads were issued by the prologue.  In the
    // branching form the same holds for s == 0.
    auto kstep = [&](auto full, auto first, auto step, int64_t s, char* ra, char* rb, char* na, char* nb, char* pb, char* pa) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full)::value, FIRST = decltype(first)::value;
        constexpr int ks = decltype(step)::value;
        constexpr int G0 = FIRST ? 3 : ks * GROUPS_PER_STEP;
        constexpr int G1 = FIRST ? 3 : ((ks + 1) * GROUPS_PER_STEP < 3 ? (ks + 1) * GROUPS_PER_STEP : 3);
        constexpr int NLOADS = ks + 1 < NK ? (G1 > G0 ? (G1 - G0) * HALF : 0) : HALF;
        constexpr int PRE = (ks + 1 == NK && FULL && CFG::OVERLAP) ? CFG::PRE_BARRIER_MFMAS : 0;
        if constexpr (ks + 1 < NK) {
            read(ra, rb, ks + 1, (ks + 1) & 1);
            if constexpr (G0 <= 0 && 0 < G1) { if (FULL || (s > 0 && s + D - 1 < nslab)) issue_b(s + D - 1, pb, HALF, LD); }
            if constexpr (G0 <= 1 && 1 < G1) { if (FULL || (s > 0 && s + D < nslab)) issue_a(s + D, pa, 0, HALF); }
            if constexpr (G0 <= 2 && 2 < G1) { if (FULL || (s > 0 && s + D < nslab)) issue_a(s + D, pa, HALF, LD); }
        } else {
            // The slab's last k-step holds the barrier.  Its first PRE MFMAs (operands already in
            // registers) are issued ahead of it, so the matrix pipe has work while the waves meet.
            if constexpr (PRE > 0) {
                mfmas(ks & 1, 0, PRE);
                __builtin_amdgcn_sched_barrier(0);
            }
            // landed after this wait: A_s+1, B_s+1; possibly still in flight: what was issued after them, the
            // slabs s+2 .. s+D-1 and A_s+D, LD loads each
            if constexpr (FULL) {
                asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((2 * (D - 2) + 1) * LD) : "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (FULL || s + 1 < nslab) read(na, nb, 0, 0);
            if (FULL || s + D < nslab) issue_b(s + D, ra, 0, HALF);
        }
        if constexpr (!CFG::OVERLAP) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        mfmas(ks & 1, PRE, NMF);
        // one fragment read behind each of the first MFMAs, the direct loads spread over all of them
        if constexpr (FULL && CFG::OVERLAP) sched_kstep<NMF - PRE, NRD, NLOADS>();
        __builtin_amdgcn_sched_barrier(0);
    };
    // `full` = every prefetch of this slab is in range, so the body is free of branches and the
    // requested interleaving can be realised by the instruction scheduler.
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    auto slab = [&](auto full, auto first, int64_t s, char* ra, char* rb, char* na, char* nb, char* pb, char* pa) __attribute__((always_inline)) {
        for_each_step(std::make_integer_sequence<int, NK>{}, [&](auto step) __attribute__((always_inline)) {
            kstep(full, first, step, s, ra, rb, na, nb, pb, pa);
        });
    };
    // slab s with its regions known at compile time: U = 2s mod R
    auto slab_at = [&](auto full, auto first, auto u, int64_t s) __attribute__((always_inline)) {
        constexpr int U = decltype(u)::value;
        using std::integral_constant;
        slab(full, first, s, region(integral_constant<int, U>{}), region(integral_constant<int, U + 1>{}), region(integral_constant<int, U + 2>{}),
             region(integral_constant<int, U + 3>{}), region(integral_constant<int, U + 2 * D - 1>{}), region(integral_constant<int, U + 2 * D>{}));
    };

    // Prologue: fill the whole ring at once (A_0, B_0, ..., A_D-1, B_D-1, A_D: all R regions), then wait for
    // slab 0 only; the rest lands while slab 0 is multiplied.  Slab 0 then issues no pre-barrier loads,
    // and its barrier wait finds the same picture as in the steady state (youngest loads: A_D).
    for_each_step(std::make_integer_sequence<int, D>{}, [&](auto i) __attribute__((always_inline)) {
        constexpr int I = decltype(i)::value;
        if (nslab > I) {
            issue_a(I, region(std::integral_constant<int, 2 * I>{}), 0, LD);
            issue_b(I, region(std::integral_constant<int, 2 * I + 1>{}), 0, LD);
        }
    });
    if (nslab > D) issue_a(D, region(std::integral_constant<int, 2 * D>{}), 0, LD);
    // (everything issued but the 2 LD loads of slab 0 may still be in flight)
    if (nslab > D) {
        wait_vmcnt<(2 * D - 1) * LD>();
    } else {
        bool waited = false;
        for_each_step(std::make_integer_sequence<int, D>{}, [&](auto i) __attribute__((always_inline)) {
            constexpr int N = D - decltype(i)::value;        // D, D-1, ..., 1 slabs issued
            if (!waited && nslab >= N) {
                wait_vmcnt<(2 * N - 2) * LD>();
                waited = true;
            }
        });
        if (!waited) wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (nslab > 0) read(r0, r1, 0, 0);
    int64_t s = 0;
    if (nslab > R + D - 1) {
        slab_at(yes{}, yes{}, std::integral_constant<int, 0>{}, 0);
        s = 1;
    }
    // R slabs bring the ring back to where it was (s = 1 mod R at the top of every trip)
    for (; s + R + D - 1 < nslab; s += R) {
        for_each_step(std::make_integer_sequence<int, R>{}, [&](auto t) __attribute__((always_inline)) {
            constexpr int T = decltype(t)::value;
            slab_at(yes{}, no{}, std::integral_constant<int, (2 * (1 + T)) % R>{}, s + T);
        });
    }
    // tail: at most R + D - 1 slabs, region pointers rotate at run time, waits are conservative
    {
        auto reg = [&](int i) __attribute__((always_inline)) -> char* {
            i %= R;
            if constexpr (R == 5) return i == 0 ? r0 : i == 1 ? r1 : i == 2 ? r2 : i == 3 ? r3 : r4;
            else return i == 0 ? r0 : i == 1 ? r1 : i == 2 ? r2 : i == 3 ? r3 : i == 4 ? r4 : i == 5 ? r5 : i == 6 ? r6 : i == 7 ? r7 : r8;
        };
        for (; s < nslab; ++s) {
            const int u = (int)((2 * s) % R);
            slab(no{}, no{}, s, reg(u), reg(u + 1), reg(u + 2), reg(u + 3), reg(u + 2 * D - 1), reg(u + 2 * D));
        }
    }

    // After the barrier of the last slab nobody reads operands from LDS any more and no load is in
    // flight: the regions can hold the epilogue's staging areas, one wave per region.
    char* stage = wave == 0 ? r0 : wave == 1 ? r1 : wave == 2 ? r2 : r3;
    const int64_t row0 = m0 + wm * (BM / CFG::WM), col0 = n0 + wn * (BN / WN);
    const bool vec_ok = (flags & FAST_VEC_C) != 0;
    const bool interior = vec_ok && row0 + BM / CFG::WM <= a.M && col0 + BN / WN <= a.N;   // wave-uniform
    auto store = [&](auto out) __attribute__((always_inline)) {
        constexpr int OUT = decltype(out)::value;
        if (interior) store_tiles_staged<OUT, true, TMI, TNI>(a, b, acc, row0, col0, lane, stage, vec_ok);
        else store_tiles_staged<OUT, false, TMI, TNI>(a, b, acc, row0, col0, lane, stage, vec_ok);   // (overloaded on the accumulator tile)
    };
    if (a.out_dtype == GEMM_F32) store(std::integral_constant<int, GEMM_F32>{});
    else if (a.out_dtype == GEMM_BF16) store(std::integral_constant<int, GEMM_BF16>{});
    else store(std::integral_constant<int, GEMM_F16>{});
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
    int64_t b;
    int tm, tn;
    tile_of<8>(blockIdx.x, (int)gridDim.x, tiles_m, tiles_n, b, tm, tn);

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

// ------------------------------------------------------------------------------------------------
// Pack kernels: rewrite one operand as [rows][Kp] with K contiguous, rows 16-byte aligned and K
// padded with zeros to a whole number of slabs (Kp), in caller-provided workspace.  They are what
// lets the fast kernel run on operands that violate its conditions (odd leading dimensions, K
// strided, ragged K): Table 1's "smem_transpose" applied ahead of the product.
//
// Source rows are aligned to their element size only.  k4_pack_rows (K contiguous) loads a chunk
// with one 16-byte load declared under-aligned, and a row's ragged end through the aligned dwords that
// contain it (a dword that holds at least one valid byte lies inside the allocation), shifted by
// bytes within a register pair.  k4_pack_transpose (source contiguous along the other axis) loads
// aligned dwords and drops their elements into an LDS tile.
// ------------------------------------------------------------------------------------------------

// K contiguous in the source.  One thread makes one 16-byte chunk of the packed row.
template <typename IN>
__global__ __launch_bounds__(256) void k4_pack_rows(const char* __restrict__ src, int64_t row_bytes, int64_t rows, int64_t K,
                                                    int64_t Kp, char* __restrict__ dst, int64_t src_batch_bytes, int64_t dst_batch_bytes)
{
    constexpr int BYTES = IN::BYTES, V = 16 / BYTES;
    const int64_t chunks = Kp / V;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= rows * chunks) return;
    const int64_t r = id / chunks, c = id % chunks;
    src += (int64_t)blockIdx.y * src_batch_bytes + r * row_bytes;
    const uintptr_t row = (uintptr_t)src, end = row + (uintptr_t)(K * BYTES);   // valid bytes of this row: [row, end)
    const uintptr_t p = row + (uintptr_t)(c * 16);
    u32x4_t out;
    if (p + 16 <= end) {
        // a whole chunk inside the row: one 16-byte load, declared aligned to a byte only
        typedef u32x4_t __attribute__((aligned(1))) u32x4_a1_t;
        out = *(const u32x4_a1_t*)p;
    } else {
        // the row's ragged end (or the zero padding past it): the aligned dwords that hold its last bytes
        const uintptr_t base = p & ~(uintptr_t)3;
        const uint32_t sh = (uint32_t)(p & 3);
        uint32_t d[5];
#pragma unroll
        for (int i = 0; i < 5; ++i) d[i] = (base + 4 * i < end && (i < 4 || sh != 0)) ? *(const uint32_t*)(base + 4 * i) : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t w = __builtin_amdgcn_alignbyte(d[i + 1], d[i], sh);      // bytes p+4i .. p+4i+3
            const int64_t left = (int64_t)(end - p) - 4 * i;                  // valid bytes from here on
            if (left <= 0) w = 0;
            else if (left < 4) w &= (1u << (8 * left)) - 1u;
            out[i] = w;
        }
    }
    *(u32x4_t*)(dst + (int64_t)blockIdx.y * dst_batch_bytes + (r * Kp + c * V) * BYTES) = out;
}

// K strided in the source (elements of one k are contiguous along the rows that become the packed
// rows).  A workgroup transposes a tile of PackRows<IN> rows x 128 bytes of K through LDS.  A tile's
// rows span 248 bytes of a source line: with the line's misalignment at most 63 aligned dwords, one per
// lane of a wave (a 64-row tile left half of the lanes idle and fetched twice the bytes it used).
// Neighbouring row tiles share the memory lines their spans end in: workgroup ids are laid out so that
// all row tiles of one K tile run on the same XCD (ids are dealt to the eight XCDs in turn), one after
// the other, and the shared lines are found in that XCD's L2 instead of being fetched once per L2
// (fp16 4093 x 4097: 66.7 -> 33.7 MB fetched for a source of 33.5 MB; the time, 19 us, did not change).
template <typename IN> constexpr int PackRows = 248 / IN::BYTES;

template <typename IN>
__global__ __launch_bounds__(256) void k4_pack_transpose(const char* __restrict__ src, int64_t k_bytes, int64_t rows, int64_t K,
                                                         int64_t Kp, char* __restrict__ dst, int64_t src_batch_bytes,
                                                         int64_t dst_batch_bytes, int row_tiles)
{
    using raw = typename IN::raw;
    constexpr int BYTES = IN::BYTES, KE = ROW_BYTES / BYTES, V = 16 / BYTES, TR = PackRows<IN>, EPD = 4 / BYTES;
    static_assert((TR * BYTES + 3 + 3) / 4 <= 64, "a line's span of a tile fits one dword per lane");
    constexpr int PITCH = KE + V;                       // elements; keeps rows 16-byte aligned, spreads banks
    __shared__ __attribute__((aligned(16))) raw tile[TR * PITCH];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    // id = 8 * j + xcd: K tile xcd + 8 * (j / row_tiles), row tile j % row_tiles (the grid is padded to
    // eight K tiles per group; a workgroup past the last K tile leaves as a whole)
    const int64_t j = blockIdx.x >> 3;
    const int64_t k0 = ((int64_t)(blockIdx.x & 7) + 8 * (j / row_tiles)) * KE, r0 = (j % row_tiles) * TR;
    if (k0 >= Kp) return;
    src += (int64_t)blockIdx.y * src_batch_bytes;
    dst += (int64_t)blockIdx.y * dst_batch_bytes;
    for (int i = t; i < TR * PITCH * BYTES / 16; i += 256) ((u32x4_t*)tile)[i] = u32x4_t{0, 0, 0, 0};
    __syncthreads();
    // source line of k: elements r0 .. r0+TR-1 are contiguous; lane l loads the l-th aligned dword of
    // the span and drops its elements into column kk of the tile
    const int nvalid = (int)((rows - r0) < TR ? (rows - r0) : TR);
    constexpr int LINES = KE / 4;                       // k lines per wave: wave w takes k = w, w+4, ...
    constexpr int BATCH = 8;                            // loads in flight per lane
    static_assert(LINES % BATCH == 0, "the k lines of a wave come in whole batches");
    const uintptr_t line0 = (uintptr_t)(src + r0 * BYTES);
    for (int i0 = 0; i0 < LINES; i0 += BATCH) {
        uint32_t w[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int64_t k = k0 + wave + 4 * (i0 + i);
            const uintptr_t first = line0 + (uintptr_t)(k * k_bytes), end = first + (uintptr_t)(nvalid * BYTES);
            const uintptr_t q = (first & ~(uintptr_t)3) + 4 * (uintptr_t)lane;
            w[i] = (k < K && q < end) ? *(const uint32_t*)q : 0u;
        }
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int kk = wave + 4 * (i0 + i);
            const int64_t k = k0 + kk;
            const uintptr_t first = line0 + (uintptr_t)(k * k_bytes), end = first + (uintptr_t)(nvalid * BYTES);
            const uintptr_t q = (first & ~(uintptr_t)3) + 4 * (uintptr_t)lane;
            if (k < K && q < end) {
#pragma unroll
                for (int e = 0; e < EPD; ++e) {
                    const int64_t n = ((int64_t)(q - first)) / BYTES + e;      // row inside the tile (-1 for a byte before it)
                    const uintptr_t at = q + (uintptr_t)(e * BYTES);
                    if (at >= first && at < end) tile[n * PITCH + kk] = (raw)(w[i] >> (8 * BYTES * e));
                }
            }
        }
    }
    __syncthreads();
    for (int idx = t; idx < TR * CHUNKS; idx += 256) {
        const int r = idx / CHUNKS, c = idx % CHUNKS;
        if (r0 + r < rows) *(u32x4_t*)(dst + ((r0 + r) * Kp + k0 + c * V) * BYTES) = *(const u32x4_t*)(tile + r * PITCH + c * V);
    }
}

// ------------------------------------------------------------------------------------------------
// Second pass of the split-K form: C = round(s * sum over the K ranges of the fp32 partial products
// + bias).  Partials are [splits][M][N] dense; one thread per four consecutive columns.
// ------------------------------------------------------------------------------------------------
template <typename IN>   // (a template only so that the header can be included by several translation units)
__global__ __launch_bounds__(256) void k4_splitk_reduce(Args a, const float* __restrict__ part, int splits)
{
    const int64_t quads = (a.N + 3) / 4;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= a.M * quads) return;
    const int64_t i = id / quads, j0 = (id % quads) * 4;
    const float sc = batch_scale(a, 0);
    const bool whole = j0 + 3 < a.N && (a.N % 4) == 0;         // the row's partials are 16-byte aligned
    float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < splits; ++s) {
        const float* p = part + ((int64_t)s * a.M + i) * a.N + j0;
        if (whole) {
            const float4 w = *(const float4*)p;
            v[0] += w.x; v[1] += w.y; v[2] += w.z; v[3] += w.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j0 + e < a.N) v[e] += p[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (j0 + e < a.N) store_out(a.C, i * a.ldc + j0 + e, v[e] * sc + (a.bias ? a.bias[j0 + e] : 0.0f), a.out_dtype);
}

// ------------------------------------------------------------------------------------------------
// Streaming kernel for M <= 96 (decode-like shapes; bf16, fp16 and e4m3): the product is bound by reading
// B once from HBM.  A workgroup owns a strip of 16*NB columns of C and all MG groups of 16 rows of A; its WAVES
// waves split K, partial sums meet in LDS at the end.  Needs: A row-major, B column-major, 16-byte
// aligned, K a multiple of 16 bytes.  (Sizes below are those of the 2-byte types; for e4m3 a tile row holds
// the same bytes and twice the elements, and a 64-byte k-step is two v_mfma_f32_16x16x32_fp8_fp8.)
//
// The operands of v_mfma_f32_16x16x32 want, per instruction, 16 rows x 64 bytes of K; fetched that
// way every wave instruction opens 16 separate 64-byte streams a leading dimension apart, and HBM
// delivers about half of what it gives to contiguous reads.  Here a wave instead fetches, per load
// instruction, 64/LPC rows' worth of LPC*16 contiguous bytes (LPC = lanes per row = TK/8), parks
// the registers of one group of 16 rows (16 columns of B, or the 16 rows of A) in a wave-private LDS
// tile of 16 rows x TK*2 bytes, and reads the MFMA operand layout back from there.  Chunk q (16
// bytes) of row c is kept at chunk position q ^ c: writes (LPC consecutive q of a row) and operand
// reads (16 rows at one q) are both bank-conflict free.  The tiles are private to the wave and LDS
// serves a wave's requests in order, so the main loop has no barrier: waves only meet for the final
// sum over the K split.
//
// Per wave and K tile: the MG groups of A and the NB column groups are parked and multiplied one after
// the other (LDS holds A and one column group: (MG+1) * 16 * TK * 2 bytes per wave); as soon as a
// group's registers are parked its loads for the next K tile are issued, so (MG+NB)*TK/32 loads stay
// in flight per lane while the MFMAs of the current tile run.  A column group's fragment is read once
// per k-step and multiplied with every group of A.
// ------------------------------------------------------------------------------------------------
template <typename IN>
__device__ __forceinline__ void mfma16(const u32x4_t& a, const u32x4_t& b, f32x4_t& c)
{
    if constexpr (IN::ID == GEMM_BF16) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    } else if constexpr (IN::ID == GEMM_F16) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    } else {
        // e4m3: the chunk's low and high 8 bytes are one K = 32 instruction each (which k a lane's bytes
        // stand for is irrelevant as long as both operands agree)
        const long alo = (long)(((uint64_t)a.y << 32) | a.x), ahi = (long)(((uint64_t)a.w << 32) | a.z);
        const long blo = (long)(((uint64_t)b.y << 32) | b.x), bhi = (long)(((uint64_t)b.w << 32) | b.z);
        c = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(alo, blo, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(ahi, bhi, c, 0, 0, 0);
    }
}

template <typename IN, int WAVES_, int NB_, int TK_, int ROT_ = 0, int MG_ = 1>
struct StreamCfg {
    using In = IN;
    static constexpr int WAVES = WAVES_, NB = NB_, TK = TK_, COLS = 16 * NB_, ROT = ROT_, MG = MG_, ROWS = 16 * MG_;
    // TK counts 2-byte units: a tile row is TK * 2 bytes of K for every input type (TK elements of a 2-byte
    // type, 2 TK of e4m3)
    static constexpr int TKE = TK * 2 / IN::BYTES;         // K elements per tile
    static constexpr int LPC = TK / 8;                     // lanes (16-byte chunks) per row per tile
    static constexpr int CPL = 64 / LPC;                   // rows covered by one load instruction
    static constexpr int GLD = 16 / CPL;                   // loads per group of 16 rows per lane
    static constexpr int KS = TK / 32;                     // 64-byte k-steps per tile (one MFMA of a 2-byte type, two of e4m3)
    static constexpr int GROUP_BYTES = 16 * TK * 2;
    static constexpr int TILE_BYTES = (MG + 1) * GROUP_BYTES;   // the groups of A and one group of B columns
    static constexpr int LDS_BYTES = WAVES * TILE_BYTES;
    static_assert(LPC >= 16 && LPC <= 64 && (LPC & (LPC - 1)) == 0, "a row's run is 16..64 lanes wide");
    static_assert(MG >= 1 && MG <= 6, "up to 96 rows of A (eight groups spill registers)");
    static_assert(WAVES * ROWS * (COLS + 1) * 4 <= LDS_BYTES, "the K-split partial sums reuse the tiles");
};

template <typename CFG>
__global__ __launch_bounds__(CFG::WAVES * 64) void k4_stream(Args a)
{
    using IN = typename CFG::In;
    constexpr int WAVES = CFG::WAVES, NB = CFG::NB, TK = CFG::TK, COLS = CFG::COLS, MG = CFG::MG, ROWS = CFG::ROWS;
    constexpr int LPC = CFG::LPC, CPL = CFG::CPL, GLD = CFG::GLD, KS = CFG::KS;
    constexpr int ROWB = TK * 2;                            // bytes per LDS row
    constexpr int EB = IN::BYTES, V = 16 / EB, TKE = CFG::TKE;   // element size, elements per chunk and per tile
    __shared__ __attribute__((aligned(16))) char lds[CFG::LDS_BYTES];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int64_t b = blockIdx.y;
    const int64_t j0 = (int64_t)blockIdx.x * COLS;
    const char* A = (const char*)a.A + b * a.stride_a * EB;
    const char* B = (const char*)a.B + b * a.stride_b * EB;
    char* tile_a = lds + wave * CFG::TILE_BYTES;
    char* tile_b = tile_a + MG * CFG::GROUP_BYTES;

    // K tiles are dealt to the waves in turn (wave w takes tiles w, w+WAVES, ...): the waves of a
    // workgroup advance side by side, so that together they read WAVES*TK*2 contiguous bytes of every
    // column at a time, which keeps HBM pages open longer than WAVES far-apart runs would.
    const int64_t kend = a.K;
    constexpr int64_t KSTRIDE = (int64_t)WAVES * TKE;

    // load side: lane fetches chunk lc of row (n*CPL + lrow) of a group.  Rows of A past M and columns
    // past N are clamped (their sums are never stored).  Offsets are 32-bit from wave-uniform bases
    // (the host has checked that a strip's extent, COLS * ldb elements, fits).
    const int lrow = lane / LPC, lc = lane % LPC;
    const char* Bs = B + j0 * a.b_sj * EB;
    const char* As = A;
    uint32_t ao[MG][GLD], bo[NB][GLD];
    int wr[GLD];
#pragma unroll
    for (int n = 0; n < GLD; ++n) {
        const int c = n * CPL + lrow;                       // row inside a group, 0..15
        wr[n] = c * ROWB + ((lc ^ c) << 4);
#pragma unroll
        for (int m = 0; m < MG; ++m) {
            const int64_t rr = m * 16 + c < a.M ? m * 16 + c : a.M - 1;
            ao[m][n] = (uint32_t)((rr * a.a_si + lc * V) * EB);
        }
#pragma unroll
        for (int g = 0; g < NB; ++g) {
            const int64_t cc = j0 + g * 16 + c < a.N ? g * 16 + c : a.N - 1 - j0;
            bo[g][n] = (uint32_t)((cc * a.b_sj + lc * V) * EB);
        }
    }
    // operand side: lane (l16, lq) holds, for k-step s, chunk 4s+lq of row l16 of the group
    const int rd = l16 * ROWB;

    f32x4_t acc[MG][NB];
#pragma unroll
    for (int m = 0; m < MG; ++m)
#pragma unroll
        for (int n = 0; n < NB; ++n) acc[m][n] = f32x4_t{0, 0, 0, 0};
    const u32x4_t zero = {0, 0, 0, 0};
    u32x4_t ra[MG][GLD], rb[NB][GLD];

    // `full`: the whole tile lies inside K, no lane needs a mask
    auto fetch_a = [&](auto full, int64_t k) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full)::value;
#pragma unroll
        for (int m = 0; m < MG; ++m)
#pragma unroll
            for (int n = 0; n < GLD; ++n)
                ra[m][n] = (FULL || k + lc * V < kend) ? *(const u32x4_t*)(As + k * EB + ao[m][n]) : zero;
    };
    auto fetch_b = [&](auto full, int g, int64_t k) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full)::value;
#pragma unroll
        for (int n = 0; n < GLD; ++n)
            rb[g][n] = (FULL || k + lc * V < kend) ? __builtin_nontemporal_load((const u32x4_t*)(Bs + k * EB + bo[g][n])) : zero;
    };
    auto park_a = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < MG; ++m)
#pragma unroll
            for (int n = 0; n < GLD; ++n) *(u32x4_t*)(tile_a + m * CFG::GROUP_BYTES + wr[n]) = ra[m][n];
    };
    auto park_b = [&](int g) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < GLD; ++n) *(u32x4_t*)(tile_b + wr[n]) = rb[g][n];
    };
    auto multiply = [&](int g) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int pos = rd + (((4 * s + lq) ^ l16) << 4);
            const u32x4_t fb = *(const u32x4_t*)(tile_b + pos);
#pragma unroll
            for (int m = 0; m < MG; ++m) {
                const u32x4_t fa = *(const u32x4_t*)(tile_a + m * CFG::GROUP_BYTES + pos);
                mfma16<IN>(fa, fb, acc[m][g]);
            }
        }
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;

    // The steady-state loop runs over whole tiles only and is free of branches; a ragged last tile
    // is fetched under masks after it.
    const int64_t tiles = (a.K + TKE - 1) / TKE;               // all K tiles, the last one possibly ragged
    const int64_t whole = a.K / TKE;                           // tiles without a mask
    const int64_t mine = tiles > wave ? (tiles - wave + WAVES - 1) / WAVES : 0;
    const int64_t nfull = whole > wave ? (whole - wave + WAVES - 1) / WAVES : 0;
    const bool ragged = mine > nfull;                          // this wave owns the ragged tile
    // The whole tiles are walked from a start that differs from one workgroup to the next and wraps
    // round (sums commute): at any moment the workgroups then read different offsets inside their
    // columns instead of all the same one, a leading dimension apart.
    const int64_t kwrap = ((int64_t)wave + WAVES * nfull) * TKE; // this wave's first tile past the whole ones
    int64_t k = (int64_t)wave * TKE;
    if (CFG::ROT && nfull > 0) k += ((int64_t)blockIdx.x * CFG::ROT % nfull) * KSTRIDE;
    if (nfull > 0) {
        fetch_a(yes{}, k);
#pragma unroll
        for (int g = 0; g < NB; ++g) fetch_b(yes{}, g, k);
        for (int64_t i = 1; i < nfull; ++i) {
            k += KSTRIDE;
            if (CFG::ROT && k >= kwrap) k -= nfull * KSTRIDE;
            park_a();
            fetch_a(yes{}, k);
#pragma unroll
            for (int g = 0; g < NB; ++g) {
                park_b(g);
                fetch_b(yes{}, g, k);
                multiply(g);
            }
        }
        k = kwrap;
        park_a();
        if (ragged) fetch_a(no{}, k);
#pragma unroll
        for (int g = 0; g < NB; ++g) {
            park_b(g);
            if (ragged) fetch_b(no{}, g, k);
            multiply(g);
        }
    } else if (ragged) {
        fetch_a(no{}, k);
#pragma unroll
        for (int g = 0; g < NB; ++g) fetch_b(no{}, g, k);
    }
    if (ragged) {
        park_a();
#pragma unroll
        for (int g = 0; g < NB; ++g) {
            park_b(g);
            multiply(g);
        }
    }

    // 16x16 accumulator: register r of lane l holds row 4*(l/16) + r, column l%16
    __syncthreads();
    float* part = (float*)lds;
#pragma unroll
    for (int m = 0; m < MG; ++m)
#pragma unroll
        for (int n = 0; n < NB; ++n)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[(wave * ROWS + m * 16 + 4 * lq + r) * (COLS + 1) + n * 16 + l16] = acc[m][n][r];
    __syncthreads();
    const float sc = batch_scale(a, b);
    // (transposed product: the kernel's row i is C's column, so consecutive threads take consecutive i)
    const bool tr = (a.flags & ARGS_C_TRANSPOSED) != 0;
    for (int o = t; o < ROWS * COLS; o += WAVES * 64) {
        const int i = tr ? o % ROWS : o / COLS, j = tr ? o / ROWS : o % COLS;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += part[(w * ROWS + i) * (COLS + 1) + j];
        if (i < a.M && j0 + j < a.N) {
            const int64_t at = tr ? (j0 + j) * a.ldc + i : (int64_t)i * a.ldc + j0 + j;
            store_out(a.C, b * a.stride_c + at, v * sc + (a.bias ? a.bias[tr ? i : j0 + j] : 0.0f), a.out_dtype);
        }
    }
}

}  // namespace gl
