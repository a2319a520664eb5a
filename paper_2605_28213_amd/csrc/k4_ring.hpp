// K4, persistent form of the direct-to-LDS kernel (256 x 256 tiles): one workgroup per CU walks a list of
// output tiles and keeps the five-region LDS ring running ACROSS tile boundaries.
//
// In k4_mfma_fast every tile pays a prologue (the ring is filled from a cold start while no MFMA issues)
// and an epilogue during which nothing is fetched; on products with a short K (e4m3 64 x 1024^3: 8 slabs
// per tile) those two phases were 37 % of a workgroup's cycles and the main loop ran at memory latency.
// Here the operand slabs of a workgroup's tiles form one stream: slab q of the stream (A of slab g: 2g,
// B: 2g+1) lives in region q mod 5 as before, the last two slabs of a tile already fetch the first two
// slabs of the next tile, and the epilogue runs with 1.5 slabs of the next tile landed or in flight.
// What remains per tile is the epilogue itself; the prologue is paid once per workgroup.
//
// Loads the compiler does not see.  The compiler orders LDS reads against pending direct-to-LDS loads by
// the alias scope of the __shared__ variable they touch; with regions that rotate at run time it cannot
// tell a fragment read of one region from the loads in flight into another and would drain them before
// every read.  The direct loads are therefore issued from inline assembly (M0 = LDS destination, then
// buffer_load_dwordx4 ... offen lds) and waited for by the explicit s_waitcnt vmcnt before each slab's
// barrier, exactly the waits k4_mfma_fast already places by hand.  Fragment reads stay ordinary loads
// (their lgkmcnt waits are the compiler's).  No compiler-issued vector memory load is in flight while
// these loads are issued (scales come through the scalar cache, the bias is loaded and consumed inside
// the epilogue); and a compiler-computed vmcnt wait that does not know of them can only wait longer than
// needed, never shorter (the counter is in order and it undercounts the younger operations).
//
// Epilogue staging.  After the barrier of a tile's last slab its B region is free until the A loads of
// the slab after next are issued.  Wave w stages in exactly the 1 KB blocks w, w+4, ... of that region
// that its own next loads will overwrite, so no barrier is needed between the epilogue and those loads.
// A staged unit is 32 rows x 256 bytes (128 two-byte or 64 fp32 columns) = 8 blocks; chunk c of row r is
// kept at c ^ (r & 15) (rows are 256 B apart and would otherwise share all banks).
//
// Conditions on top of k4_mfma_fast's: at least 3 slabs per tile (the kinds first / last-but-one / last are
// distinct slabs), at least as many tiles as workgroups launched.  Paper Table 1: "cp.async + pipeline"
// carried across tile boundaries; the persistent tile loop is the "stream-K" family's scheduling.
//
// A second form of the same kernel (RingCfg<..., BROW = true>) reads a ROW-MAJOR B in place, with transposing LDS
// reads, from rows that need not be aligned and a K that need not be whole slabs: see RingCfg below.
#pragma once
#include "k4_kernels.hpp"

namespace gl {

// Bytes past an operand's end that the row-major-B form may read.  Buffer loads are range-checked dword by dword,
// and a row with an odd number of two-byte elements ends in the middle of a dword (rows are loaded as dwords from
// their first element): that dword is wanted, and its other half is the one element after the operand.
constexpr int RING_BROW_SLACK = 2;
constexpr int RING_WORKGROUPS = 256;      // one per CU of the GPU this library is written for (8 XCDs x 32)

// BROW: B is stored row-major (N contiguous; two-byte types).  Its slab is then kept in LDS as it lies in
// memory, 64 rows of k x 512 bytes of n, and the MFMA fragment (8 consecutive k per lane for one n) is read with the
// transposing LDS read ds_read_b64_tr_b16.  That instruction works on blocks of 16 lanes: lane 4 kk + q of a block
// points at 4 consecutive 16-bit elements (here: k row kk, columns 4q..4q+3 of a 4 x 16 patch), and lane 4 q + e
// receives element e of the lanes q, q+4, q+8, q+12 (here: the four k of column 4q+e).  Two such reads give a
// lane its 8 k.  Chunk c (16 bytes = 8 columns) of k row r is kept at c ^ 4 (r % 4): the four rows a block reads
// then lie in four different quarters of the banks.  (Table 1 "smem_transpose" / "ldmatrix.swizzle" with the
// transpose done by the read instead of by a pass over the operand.)
template <typename IN, int GROUP_M_ = 8, bool BROW_ = false>
struct RingCfg {
    using In = IN;
    static constexpr bool BROW = BROW_;
    static_assert(!BROW_ || IN::BYTES == 2, "the transposing read used here is the 16-bit one");
    static constexpr int BM = 256, BN = 256, WM = 2, WN = 2, GROUP_M = GROUP_M_;
    static constexpr int T = WM * WN * 64;
    static constexpr int TMI = BM / WM / 32, TNI = BN / WN / 32;
    static constexpr int REGION = BM * ROW_BYTES, REGIONS = 5;
    static constexpr int LDS_BYTES = REGIONS * REGION;
};

enum RingSlabKind { RING_FIRST = 0, RING_MID = 1, RING_PEN = 2, RING_LAST = 3 };

// One staged unit of the epilogue: 32 rows x 256 bytes in the wave's own blocks of the staging region.
__device__ __forceinline__ char* ring_stage_row(char* stage, int wave, int r)
{
    return stage + ((wave + 4 * (r >> 2)) << 10) + ((r & 3) << 8);
}

// One fp32 through the scalar cache (read-only inputs: the per-problem scales).  The compiler loads them with a
// vector load, and the wait for that load would drain the next tile's direct loads (one counter for both).
__device__ __forceinline__ float scalar_load_f32(const float* p)
{
    float v;
    // (s_nop first: the address may have been reloaded from a spill by a vector instruction just before)
    asm volatile("s_nop 4\n\ts_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
    return v;
}

// BIAS is a template parameter: with the test at run time the compiler waits, where the two paths join, for the
// bias loads of the path not taken, and that wait (the counter is shared) drains the next tile's direct loads.
template <int OUT, bool INTERIOR, bool BIAS, int TMI, int TNI>
__device__ __forceinline__ void store_tiles_ring(const Args& a, int64_t b, const f32x16_t (&acc)[TMI][TNI], int64_t row0,
                                                 int64_t col0, int wave, char* stage, bool vec_ok)
{
    constexpr int OB = OUT == GEMM_F32 ? 4 : 2;            // bytes per output element
    constexpr int UCOLS = 256 / OB;                        // columns per staged unit
    constexpr int JP = UCOLS / 32, UNITS = TNI / JP;       // column tiles per unit; units per 32-row block
    constexpr int EPC = 16 / OB;                           // elements per 16-byte chunk
    static_assert(TNI % JP == 0, "a wave's columns are whole staged units");
    float sc = 1.0f;
    if (a.scale_a) sc *= scalar_load_f32(a.scale_a + b);
    if (a.scale_b) sc *= scalar_load_f32(a.scale_b + b);
    // Everything the epilogue derives from the lane id is derived here, per tile, from a lane id that is itself
    // recomputed behind an opaque statement: the compiler can then neither hoist those two dozen address
    // constants out of the tile loop nor keep the lane id for them, where they would sit in registers (or
    // scratch, whose reload waits on the same counter as the direct loads) across the whole main loop.
    unsigned all = ~0u;
    asm volatile("" : "+s"(all));
    const int lane = (int)__builtin_amdgcn_mbcnt_hi(all, __builtin_amdgcn_mbcnt_lo(all, 0u));
    const int lrow = lane & 31, lhalf = lane >> 5;
    char* C = (char*)a.C + (b * a.stride_c) * OB;
    char* wrow = ring_stage_row(stage, wave, lrow);
    const int wx = lrow & 15;
    // bias of the four columns a lane holds per (column tile, register quad), the same for every row block
    f32x4_t bv[TNI][4];
#pragma unroll
    for (int j = 0; j < TNI; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bv[j][g] = f32x4_t{0, 0, 0, 0};
            if constexpr (BIAS) {
                const int64_t gj = col0 + j * 32 + 8 * g + 4 * lhalf;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (INTERIOR || gj + c < a.N) bv[j][g][c] = a.bias[gj + c];
            }
        }
#pragma unroll
    for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
#pragma unroll
            for (int jj = 0; jj < JP; ++jj) {
                const int j = u * JP + jj;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[c] = BIAS ? acc[i][j][4 * g + c] * sc + bv[j][g][c] : acc[i][j][4 * g + c] * sc;
                    if constexpr (OUT == GEMM_F32) {
                        const int chunk = jj * 8 + 2 * g + lhalf;
                        *(f32x4_t*)(wrow + ((chunk ^ wx) << 4)) = f32x4_t{v[0], v[1], v[2], v[3]};
                    } else if constexpr (OUT == GEMM_BF16) {
                        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
                        const int chunk = jj * 4 + g;
                        *(bf16x4_t*)(wrow + ((chunk ^ wx) << 4) + 8 * lhalf) = bf16x4_t{(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
                    } else {
                        typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
                        const int chunk = jj * 4 + g;
                        *(f16x4_t*)(wrow + ((chunk ^ wx) << 4) + 8 * lhalf) = f16x4_t{(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
                    }
                }
            }
            // 32 rows x 16 chunks = 8 passes of 64 lanes: 4 whole rows per pass
            u32x4_t w[8];
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int r = 4 * p + (lane >> 4), cc = lane & 15;
                w[p] = *(const u32x4_t*)(ring_stage_row(stage, wave, r) + ((cc ^ (r & 15)) << 4));
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int r = 4 * p + (lane >> 4), cc = lane & 15;
                const int64_t gi = row0 + i * 32 + r, gj = col0 + u * UCOLS + cc * EPC;
                char* out = C + (gi * a.ldc + gj) * OB;
                if constexpr (INTERIOR) {
                    *(u32x4_t*)out = w[p];
                } else if (gi < a.M) {
                    if (gj + EPC <= a.N) {
                        typedef u32x4_t __attribute__((aligned(2))) u32x4_a2_t;
                        typedef u32x4_t __attribute__((aligned(4))) u32x4_a4_t;
                        if (vec_ok) *(u32x4_t*)out = w[p];
                        else if constexpr (OB == 4) *(u32x4_a4_t*)out = w[p];
                        else *(u32x4_a2_t*)out = w[p];
                    } else {
#pragma unroll
                        for (int e = 0; e < EPC; ++e)
                            if (gj + e < a.N) {
                                if constexpr (OB == 4) ((uint32_t*)out)[e] = w[p][e];
                                else ((uint16_t*)out)[e] = (uint16_t)(w[p][e / 2] >> (16 * (e & 1)));
                            }
                    }
                }
            }
        }
}

template <typename CFG>
__global__ __launch_bounds__(CFG::T) __attribute__((amdgpu_waves_per_eu(1, 1)))
void k4_mfma_ring(Args a, int tiles_m, int tiles_n, int total, int flags)
{
    using IN = typename CFG::In;
    constexpr int BM = CFG::BM, BN = CFG::BN, WN = CFG::WN, NW = CFG::T / 64;
    constexpr int TMI = CFG::TMI, TNI = CFG::TNI, REGION = CFG::REGION;
    constexpr int KE = ROW_BYTES / IN::BYTES;            // K elements per slab
    constexpr int V = 16 / IN::BYTES;                    // K elements per chunk
    constexpr int CPS = Frag<IN>::CPS;                   // chunks per lane per k-step
    constexpr int NK = CHUNKS / (2 * CPS);               // k-steps per slab
    constexpr int LD = BM / 8 / NW;                      // direct loads per wave per operand slab
    constexpr int HALF = LD / 2;
    static_assert(BM == 256 && BN == 256 && NW == 4 && LD == 8 && NK >= 2, "written for 256 x 256 tiles and four waves");
    __shared__ __attribute__((aligned(1024))) char lds[CFG::LDS_BYTES];

    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- this workgroup's tiles ------------------------------------------------------------------
    // Workgroup ids are dealt to the 8 XCDs in turn; XCD x owns a contiguous run of the (batch, tile)
    // sequence (the same runs k4_mfma_fast's tile walk gives it) and its workgroups take the run's
    // positions l, l + per_x, l + 2 per_x, ...
    const int G = (int)gridDim.x, per_x = G / 8;
    const int x = (int)blockIdx.x % 8, l = (int)blockIdx.x / 8;
    const int base = total / 8, rem = total % 8;
    const int start_x = x * base + (x < rem ? x : rem), count_x = base + (x < rem ? 1 : 0);
    const int n_mine = l < count_x ? (count_x - l + per_x - 1) / per_x : 0;
    if (n_mine <= 0) return;
    const int per = tiles_m * tiles_n;

    typedef __attribute__((ext_vector_type(4))) int rsrc_t;   // raw buffer descriptor: base, base high | stride 0, bytes, format
    struct Tile {
        rsrc_t ra, rb;
        int64_t b, m0, n0;
    };
    constexpr int64_t CAP = 0xFFFFFFFFll;
    constexpr int RSRC_FLAGS = 0x00020000;               // raw buffer, 32-bit data format
    // tile number i of this workgroup; past the end: empty resources (their loads fetch nothing and bring zeros)
    auto tile_at = [&](int i) __attribute__((always_inline)) -> Tile {
        const bool valid = i < n_mine;
        const int flat = start_x + l + per_x * (valid ? i : 0);
        const int bb = flat / per, id = flat % per;
        const int width = CFG::GROUP_M * tiles_n;
        const int g = id / width, first = g * CFG::GROUP_M;
        const int gsz = (tiles_m - first) < CFG::GROUP_M ? (tiles_m - first) : CFG::GROUP_M;
        const int tm = __builtin_amdgcn_readfirstlane(first + (id % width) % gsz);
        const int tn = __builtin_amdgcn_readfirstlane((id % width) / gsz);
        Tile T;
        T.b = __builtin_amdgcn_readfirstlane(bb);
        T.m0 = (int64_t)tm * BM;
        T.n0 = (int64_t)tn * BN;
        const char* A = (const char*)a.A + (T.b * a.stride_a + T.m0 * a.a_si) * IN::BYTES;
        const char* B = (const char*)a.B + (T.b * a.stride_b + T.n0 * a.b_sj) * IN::BYTES;
        const int64_t bytes_a = valid ? ((a.M - 1 - T.m0) * a.a_si + a.K) * IN::BYTES : 0;
        // (row-major B: the tile's columns start at n0 of every k row; the resource ends with the last row's last column)
        const int64_t bytes_b = !valid ? 0 : CFG::BROW ? ((a.K - 1) * a.b_sk + (a.N - T.n0)) * IN::BYTES
                                                        : ((a.N - 1 - T.n0) * a.b_sj + a.K) * IN::BYTES;
        auto desc = [&](const char* p, int64_t bytes) __attribute__((always_inline)) -> rsrc_t {
            const uint64_t u = (uint64_t)(uintptr_t)p;
            return rsrc_t{__builtin_amdgcn_readfirstlane((int)(uint32_t)u), __builtin_amdgcn_readfirstlane((int)(uint32_t)((u >> 32) & 0xFFFFu)),
                          __builtin_amdgcn_readfirstlane((int)(uint32_t)(bytes < CAP ? bytes : CAP)), RSRC_FLAGS};
        };
        // (row-major B form: the dword that holds the last element of an odd-length last row reaches one element past
        // the operand; the resources end SLACK bytes later, which the host has checked to lie in the page of the
        // operand's last byte; that element lands beyond K in A, where clear_tail removes it, and in a column past N
        // in B, which only feeds outputs that are never stored)
        constexpr int64_t SLACK = CFG::BROW ? RING_BROW_SLACK : 0;
        T.ra = desc(A, valid ? bytes_a + SLACK : 0);
        T.rb = desc(B, valid ? bytes_b + SLACK : 0);
        return T;
    };

    // ---- global -> LDS (as in k4_mfma_fast: lane L of a wave-wide 16-byte load lands at byte 16 L of a 1 KB
    // block = 8 LDS rows; the lane -> chunk assignment applies the swizzle; octet and slab are scalar) ----
    // Everything derived from the lane id is (re)computed by lane_setup() at the top of every tile, from a lane id
    // taken behind an opaque statement: kept across the epilogue (which needs most of the registers) such values get
    // spilled, and a scratch reload waits on the same counter as the direct loads in flight.
    int lane, orow, gchunk, voff_a, voff_b, lrow, lhalf, rd_mask, rd_a, rd_b, tr_jx, tr_base;
    auto lane_setup = [&]() __attribute__((always_inline)) {
        unsigned all = ~0u;
        asm volatile("" : "+s"(all));
        lane = (int)__builtin_amdgcn_mbcnt_hi(all, __builtin_amdgcn_mbcnt_lo(all, 0u));
        orow = lane >> 3;
        gchunk = (lane & 7) ^ swz(orow + 8 * (wave & 1));
        voff_a = (int)((orow * a.a_si + gchunk * V) * IN::BYTES);
        // row-major B: a wave-wide load covers two k rows x 512 bytes; lane L fetches, for k row L/32 of the pair, the
        // chunk whose swizzled position is L%32 (instruction number idx = wave + 4n holds rows 2 idx, 2 idx + 1 of the
        // slab, so a row's number modulo 4 is 2 (wave % 2) + L/32 for every n)
        const int brow_g = 4 * ((2 * (wave & 1) + (lane >> 5)) & 3);
        voff_b = CFG::BROW ? (int)(((lane >> 5) * a.b_sk + ((lane & 31) ^ brow_g) * V) * IN::BYTES)
                           : (int)((orow * a.b_sj + gchunk * V) * IN::BYTES);
        // LDS -> registers
        lrow = lane & 31;
        lhalf = lane >> 5;
        rd_mask = (lhalf * CPS) ^ swz(lrow);
        rd_a = (wm * (BM / CFG::WM) + lrow) * ROW_BYTES;
        rd_b = (wn * (BN / WN) + lrow) * ROW_BYTES;
        // row-major B: the lane's place in its block of 16 (see RingCfg): k row 8 (lane/32) + (lane%16)/4 of a k-step,
        // columns 16 ((lane/16)%2) + 4 (lane%4) .. +3 of a 32-column tile; per column tile j the swizzled chunk
        // differs in the tile number only (j ^ (lane%16)/4)
        tr_jx = (lane & 15) >> 2;
        const int tr_n = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        tr_base = (8 * lhalf + tr_jx) * 512 + ((wn * 16 + (tr_n >> 3)) << 4) + ((tr_n >> 2) & 1) * 8;
    };
    lane_setup();
    const int oct_a = (int)(8 * a.a_si * IN::BYTES), oct_b = CFG::BROW ? (int)(2 * a.b_sk * IN::BYTES) : (int)(8 * a.b_sj * IN::BYTES);
    // bytes from one K slab of an operand to the next
    const int slab_a = ROW_BYTES, slab_b = CFG::BROW ? (int)(KE * a.b_sk * IN::BYTES) : ROW_BYTES;
    using lptr = __attribute__((address_space(3))) char*;
    const int lds0 = (int)(uint32_t)(uintptr_t)(lptr)lds;      // LDS address of region 0
    // loads [lo, hi) of this wave's share of slab `sidx` of an operand into the region at byte offset `reg`
    //
    // Wait states the hardware does not interlock and the compiler's hazard pass cannot place inside inline assembly:
    // one between a scalar write of M0 and a load to LDS that reads it, and five between a vector instruction that
    // writes a scalar register -- the reload of a spilled scalar is one -- and a memory instruction that reads that
    // register as descriptor or offset.  `guarded` loads carry s_nop 4 (six wait states with the s_mov); they are
    // the ones issued outside the steady-state loop, where such reloads occur.  The loads of the middle slabs carry
    // the one wait state for M0 only (the five cost 4 % there): the steady-state loop has no vector instruction that
    // writes a scalar register at all, which tests/test_codegen.py checks on the compiled code for every
    // instantiation, as it checks the distance to such a write for every other load.  M0 is reserved: the compiler
    // keeps nothing in it and this kernel has no other user.
    auto issue = [&](auto guarded, rsrc_t rsrc, int voff, int oct, int slab_bytes, int sidx, int reg, int lo, int hi) __attribute__((always_inline)) {
        const int k0 = sidx * slab_bytes;
#pragma unroll
        for (int n = lo; n < hi; ++n) {
            const int dst = lds0 + reg + (wave + n * NW) * 1024, soff = k0 + (wave + n * NW) * oct;
            if constexpr (decltype(guarded)::value)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(dst), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
            else
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(dst), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
        }
    };

    constexpr int NMF = TMI * TNI;                   // MFMA instructions per k-step
    constexpr int NRD = CFG::BROW ? TMI + 2 * TNI : (TMI + TNI) * CPS;   // fragment reads per k-step
    typedef short v4s_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4s_t* tr_ptr;
    f32x16_t acc[TMI][TNI];
    Frag<IN> fa[2][TMI], fb[2][TNI];
    // fragment reads of k-step ks into `slot`, part `part` of PARTS (B fragments first, as the MFMA walk needs them)
    auto read_part = [&](int ra, int rb, int ks, int slot, auto part_, auto parts_) __attribute__((always_inline)) {
        constexpr int part = decltype(part_)::value, PARTS = decltype(parts_)::value;
        constexpr int TOTAL = NRD, PER = TOTAL / PARTS;
        static_assert(TOTAL % PARTS == 0, "fragment reads split evenly");
#pragma unroll
        for (int n = part * PER; n < (part + 1) * PER; ++n) {
            if constexpr (CFG::BROW) {
                if (n < 2 * TNI) {
                    // B tile j = n/2, k 4 (n%2) .. +3 of the lane's eight: the low or the high half of the fragment
                    const int j = n >> 1, half = n & 1;
                    const int off = rb + tr_base + (((j ^ tr_jx) << 2) << 4) + (16 * ks + 4 * half) * 512;
                    const v4s_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(lds + off));
                    const uint32_t lo = (uint32_t)(uint16_t)v[0] | ((uint32_t)(uint16_t)v[1] << 16);
                    const uint32_t hi = (uint32_t)(uint16_t)v[2] | ((uint32_t)(uint16_t)v[3] << 16);
                    if (half == 0) { fb[slot][j].c[0].x = lo; fb[slot][j].c[0].y = hi; }
                    else { fb[slot][j].c[0].z = lo; fb[slot][j].c[0].w = hi; }
                } else {
                    const int i = n - 2 * TNI;
                    const int pos = ((2 * ks) ^ rd_mask) << 4;
                    fa[slot][i].c[0] = *(const u32x4_t*)(lds + ra + rd_a + i * 32 * ROW_BYTES + pos);
                }
            } else {
                const int q = n / (TMI + TNI), m = n % (TMI + TNI);
                const int pos = ((2 * CPS * ks + q) ^ rd_mask) << 4;
                if (m < TNI) fb[slot][m].c[q] = *(const u32x4_t*)(lds + rb + rd_b + m * 32 * ROW_BYTES + pos);
                else fa[slot][m - TNI].c[q] = *(const u32x4_t*)(lds + ra + rd_a + (m - TNI) * 32 * ROW_BYTES + pos);
            }
        }
    };
    auto read = [&](int ra, int rb, int ks, int slot) __attribute__((always_inline)) {
        read_part(ra, rb, ks, slot, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});
    };
    // MFMAs [lo, hi) of a k-step's walk (row tiles outermost, columns back and forth so that consecutive
    // instructions share an operand).  `fresh`: the first k-step of a tile starts the sums (the matrix
    // instruction adds to zero), so the accumulators need no clearing pass between tiles.
    auto mfmas = [&](auto fresh, int slot, int lo, int hi) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TMI; ++i)
#pragma unroll
            for (int jj = 0; jj < TNI; ++jj) {
                const int j = (i & 1) ? TNI - 1 - jj : jj;
                if (i * TNI + jj < lo || i * TNI + jj >= hi) continue;
                if constexpr (decltype(fresh)::value) {
                    f32x16_t z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
                    mfma_step<IN>(fb[slot][j], fa[slot][i], z);
                    acc[i][j] = z;
                } else {
                    mfma_step<IN>(fb[slot][j], fa[slot][i], acc[i][j]);
                }
            }
    };
    constexpr int GROUPS_PER_STEP = (3 + NK - 2) / (NK - 1);

    Tile cur = tile_at(0), nxt = tile_at(1);
    int stores_behind = 0;                           // 16-byte stores this wave issued in the epilogue before the current tile (unmasked path only)
    // Slabs per tile, at least 3 (checked by the launcher).  Only the row-major-B form takes a K that is not whole
    // slabs: `ktail` is the number of valid k in its last slab (0: the slab is whole).
    const int nslab = CFG::BROW ? (int)((a.K + KE - 1) / KE) : (int)(a.K / KE);
    const int ktail = CFG::BROW ? (int)(a.K % KE) : 0;
    // Ragged K: the last slab of A holds, beyond k = K, the next row's first elements (or the element after the
    // operand), and B's rows beyond K are zeros from the range check; anything but zeros on either side could turn
    // into NaN (0 x NaN), so both are cleared.  Once the slab has landed (the wait of the slab before it) and before the barrier that releases it
    // to the readers, every lane clears what lies beyond K in the chunks its own loads wrote.
    auto clear_tail = [&](int reg_a, int reg_b) __attribute__((always_inline)) {
        unsigned zero = 0;                        // (opaque: a zero vector kept in registers across the main loop would be spilled)
        asm volatile("" : "+v"(zero));
#pragma unroll
        for (int n = 0; n < LD; ++n) {
            const int blk = (wave + n * NW) * 1024 + lane * 16;
            {   // A: row 8 (wave + 4n) + orow, logical chunk gchunk = elements gchunk*V .. +V-1 of the slab
                const int valid = ktail - gchunk * V;
                if (valid < V) {
                    u32x4_t w = *(const u32x4_t*)(lds + reg_a + blk);
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const int left = valid - 2 * d;           // valid 16-bit elements of this dword
                        w[d] = left <= 0 ? 0u : left == 1 ? (w[d] & 0xFFFFu) : w[d];
                    }
                    *(u32x4_t*)(lds + reg_a + blk) = w;
                }
            }
            // B: k row 2 (wave + 4n) + lane/32 of the slab
            if (2 * (wave + n * NW) + (lane >> 5) >= ktail) *(u32x4_t*)(lds + reg_b + blk) = u32x4_t{zero, zero, zero, zero};
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };

    // One slab of the stream; ra, rb: byte offsets of the regions holding its A and B, na, nb: those of the
    // next slab, fifth: the free one.  Prefetches, in issue order: second half of B of the next slab, both
    // halves of A of the slab after next (before the barrier), first half of B of the slab after next (after
    // it).  Which tile those slabs belong to depends on the kind.
    //
    // A k-step is issued in four quarters of NMF/4 MFMAs; the fragment reads of the next k-step ride behind
    // the MFMAs of the first two quarters and the k-step's direct loads close the quarters in equal shares:
    // the inline-assembly loads keep their place in program order, so the source order is the issue order
    // (bunched, the four waves' loads queue up in the CU's one address unit and stall the MFMAs behind them).
    //
    // BWHOLE (slabs of two k-steps: e4m3): the whole of B of the slab after next is issued behind the barrier
    // and nothing of it in the next slab's first k-step.  With one k-step ahead of the barrier a load issued
    // there has half a slab (about 1000 cycles) to land before the wave waits for it; issued behind the
    // barrier it has a whole slab, and the slab's 16 loads still split 8 : 8 over its two k-steps.
    constexpr bool BWHOLE = NK == 2;
    constexpr int QUARTERS = 4, QM = NMF / QUARTERS;
    static_assert(NMF % QUARTERS == 0 && NRD % 2 == 0, "quarters of a k-step");
    auto slab = [&](auto kind_, int s, int ra, int rb, int na, int nb, int fifth) __attribute__((always_inline)) {
        constexpr int KIND = decltype(kind_)::value;
        constexpr std::integral_constant<bool, KIND != RING_MID> guard{};     // (see `issue`)
        // sources of the prefetches
        const rsrc_t b1 = KIND == RING_LAST ? nxt.rb : cur.rb;                       // B of slab s+1
        const rsrc_t a2 = (KIND == RING_PEN || KIND == RING_LAST) ? nxt.ra : cur.ra; // A, B of slab s+2
        const rsrc_t b2 = (KIND == RING_PEN || KIND == RING_LAST) ? nxt.rb : cur.rb;
        const int i1 = KIND == RING_LAST ? 0 : s + 1;
        const int i2 = KIND == RING_LAST ? 1 : KIND == RING_PEN ? 0 : s + 2;
        if constexpr (KIND == RING_FIRST) read(ra, rb, 0, 0);     // (the other kinds got theirs from the slab before)
        for_each_step(std::make_integer_sequence<int, NK>{}, [&](auto step) __attribute__((always_inline)) {
            constexpr int ks = decltype(step)::value;
            constexpr bool LASTSTEP = ks + 1 == NK;
            constexpr int G0 = ks * GROUPS_PER_STEP;
            constexpr int G1 = (ks + 1) * GROUPS_PER_STEP < 3 ? (ks + 1) * GROUPS_PER_STEP : 3;
            constexpr bool has0 = !LASTSTEP && G0 <= 0 && 0 < G1 && KIND != RING_FIRST && !BWHOLE;   // (a tile's first slab: issued by the last slab of the tile before)
            constexpr bool has1 = !LASTSTEP && G0 <= 1 && 1 < G1, has2 = !LASTSTEP && G0 <= 2 && 2 < G1;
            // this k-step's loads as one list: [B second half] [A first half] [A second half], or after the barrier [B first half | all of B]
            constexpr int N0 = has0 ? HALF : 0, N1 = has1 ? HALF : 0, N2 = has2 ? HALF : 0;
            constexpr int NL = LASTSTEP ? ((KIND == RING_LAST || BWHOLE) ? LD : HALF) : N0 + N1 + N2;
            auto load_n = [&](int n) __attribute__((always_inline)) {
                if constexpr (LASTSTEP) {
                    issue(guard, b2, voff_b, oct_b, slab_b, i2, ra, n, n + 1);
                } else {
                    if (n < N0) issue(guard, b1, voff_b, oct_b, slab_b, i1, nb, HALF + n, HALF + n + 1);
                    else if (n < N0 + N1) issue(guard, a2, voff_a, oct_a, slab_a, i2, fifth, n - N0, n - N0 + 1);
                    else issue(guard, a2, voff_a, oct_a, slab_a, i2, fifth, HALF + n - N0 - N1, HALF + n - N0 - N1 + 1);
                }
            };
            if constexpr (LASTSTEP) {
                // landed after this wait: A and B of slab s+1; possibly still in flight: the LD loads of A of slab s+2.
                // A tile's first slab follows the epilogue of the tile before: the loads it waits for were issued
                // before that epilogue's stores, so the stores (a known number on the unmasked path) may stay in
                // flight too; the counter is in order, and fewer stores than assumed would make the wait too weak,
                // which is why any other epilogue path reports none.
                if (KIND == RING_FIRST && stores_behind == 32) asm volatile("s_waitcnt vmcnt(40) lgkmcnt(0)" ::: "memory");
                else if (KIND == RING_FIRST && stores_behind == 64) asm volatile("s_waitcnt vmcnt(63) lgkmcnt(0)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
                if constexpr (CFG::BROW && KIND == RING_PEN) {
                    if (ktail != 0) clear_tail(na, nb);       // the tile's last slab has just landed in the next regions
                }
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            constexpr bool READS = !(LASTSTEP && KIND == RING_LAST);      // (a tile's last slab reads nothing ahead: the next tile's first slab does)
            for_each_step(std::make_integer_sequence<int, QUARTERS>{}, [&](auto quarter) __attribute__((always_inline)) {
                constexpr int q = decltype(quarter)::value;
                if constexpr (READS && q < 2) {
                    if constexpr (LASTSTEP) read_part(na, nb, 0, 0, quarter, std::integral_constant<int, 2>{});
                    else read_part(ra, rb, ks + 1, (ks + 1) & 1, quarter, std::integral_constant<int, 2>{});
                }
                if constexpr (KIND == RING_FIRST && ks == 0) mfmas(std::true_type{}, ks & 1, q * QM, (q + 1) * QM);
                else mfmas(std::false_type{}, ks & 1, q * QM, (q + 1) * QM);
                // one fragment read (or more) behind each MFMA of the quarters that carry reads
                sched_kstep<QM, (READS && q < 2) ? NRD / 2 : 0, 0>();
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int n = (q * NL) / QUARTERS; n < ((q + 1) * NL) / QUARTERS; ++n) load_n(n);
            });
        });
    };

    // ---- prologue, once per workgroup: slabs 0 and 1 of the first tile into regions 0..3, wait for slab 0 ----
    int o0 = 0, o1 = REGION, o2 = 2 * REGION, o3 = 3 * REGION, o4 = 4 * REGION;   // ra, rb, na, nb, fifth of the next slab
    issue(std::true_type{}, cur.ra, voff_a, oct_a, slab_a, 0, o0, 0, LD);
    issue(std::true_type{}, cur.rb, voff_b, oct_b, slab_b, 0, o1, 0, LD);
    issue(std::true_type{}, cur.ra, voff_a, oct_a, slab_a, 1, o2, 0, LD);
    issue(std::true_type{}, cur.rb, voff_b, oct_b, slab_b, 1, o3, 0, LD);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // every slab moves the ring on by two regions
    auto rotate = [&]() __attribute__((always_inline)) {
        const int t0 = o0, t1 = o1;
        o0 = o2; o1 = o3; o2 = o4; o3 = t0; o4 = t1;
    };
    const bool vec_ok = (flags & FAST_VEC_C) != 0;
    for (int i = 0; i < n_mine; ++i) {
        lane_setup();
        slab(std::integral_constant<int, RING_FIRST>{}, 0, o0, o1, o2, o3, o4);
        rotate();
        for (int s = 1; s + 2 < nslab; ++s) {
            slab(std::integral_constant<int, RING_MID>{}, s, o0, o1, o2, o3, o4);
            rotate();
        }
        slab(std::integral_constant<int, RING_PEN>{}, nslab - 2, o0, o1, o2, o3, o4);
        rotate();
        slab(std::integral_constant<int, RING_LAST>{}, nslab - 1, o0, o1, o2, o3, o4);
        // the last slab's B region is free until the next slab's A loads (it is that slab's fifth region): staging
        char* stage = lds + o1;
        rotate();
        const int64_t row0 = cur.m0 + wm * (BM / CFG::WM), col0 = cur.n0 + wn * (BN / WN);
        const bool interior = vec_ok && row0 + BM / CFG::WM <= a.M && col0 + BN / WN <= a.N;   // wave-uniform
        auto store = [&](auto out) __attribute__((always_inline)) {
            constexpr int OUT = decltype(out)::value;
            if (a.bias) {
                if (interior) store_tiles_ring<OUT, true, true, TMI, TNI>(a, cur.b, acc, row0, col0, wave, stage, vec_ok);
                else store_tiles_ring<OUT, false, true, TMI, TNI>(a, cur.b, acc, row0, col0, wave, stage, vec_ok);
            } else {
                if (interior) store_tiles_ring<OUT, true, false, TMI, TNI>(a, cur.b, acc, row0, col0, wave, stage, vec_ok);
                else store_tiles_ring<OUT, false, false, TMI, TNI>(a, cur.b, acc, row0, col0, wave, stage, vec_ok);
            }
        };
        if (a.out_dtype == GEMM_F32) store(std::integral_constant<int, GEMM_F32>{});
        else if (a.out_dtype == GEMM_BF16) store(std::integral_constant<int, GEMM_BF16>{});
        else store(std::integral_constant<int, GEMM_F16>{});
        // (unit = 32 rows x 256 bytes = 8 stores per wave; a 128 x 128 sub-tile is 4 row blocks of 1 or 2 units)
        stores_behind = (interior && !a.bias) ? (a.out_dtype == GEMM_F32 ? 64 : 32) : 0;
        cur = nxt;
        // (the tile after next is worked out here, behind the stores, where no fragment is live: passed through an
        // opaque statement its integer divisions cannot be moved up into the slabs, where they cost spills)
        int after_next = i + 2;
        asm volatile("" : "+s"(after_next));
        nxt = tile_at(after_next);
    }
    // the empty prefetches of the tile after the last one write zeros into LDS: let them land before the wave ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace gl
