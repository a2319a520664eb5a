// K3, the pipelined state, in its asynchronous form (paper Table 1, "cp.async + pipeline"; pre: sm-staged).
//
// The next slabs travel global -> LDS without passing through registers (buffer loads that write LDS directly),
// three stages deep: while stage s is multiplied, slab s+1 has landed or is landing and slab s+2 is being
// fetched.  One barrier per slab.  Because such a load cannot decode on its way, LDS holds the operands in
// their STORAGE format (K contiguous, 64 bytes of K per row and slab) and an element is decoded when it is read
// for the FMAs: a two-byte operand then costs half, a one-byte operand a quarter of the LDS read traffic of the
// fp32 slabs K1 and K2 keep (whose 8 x 8 register tile reads 64 bytes per k step and thread, which is exactly
// the LDS bandwidth a CU has per 64 FMAs).
//
// A workgroup of 256 threads owns a 128 x 128 tile (64 x 64 on small problems); thread (ty, tx) owns rows ty + 16 i
// and columns tx + 16 j (i, j = 0..7, or 0..3): within a wave the 16 tx lanes read 16 different rows of B's slab and the same row of A's.  Chunk c
// (16 bytes) of row r is kept at position c ^ ((r / 4) % 4), which spreads rows r, r+4, r+8, r+12 over the banks;
// the swizzle is applied by the lane -> global chunk assignment of the loads (one wave instruction fills 16 rows).
// Rows past M or N lie outside the buffer resource and read as zeros.
//
// Needs what a 16-byte direct load needs of BOTH operands -- K contiguous, base and leading dimension multiples of
// 16 bytes -- and K a whole number of slabs (nothing is masked along K); otherwise K3 runs its register-staged
// form (k123_valu_tiled.hip), and gemm_query says which.
#include "common.hpp"

namespace gl {

template <typename IN, int TM_ = 8>
struct AsyncCfg {
    static constexpr int TM = TM_;                    // outputs per thread along each axis: 8 (128 x 128 tile) or 4 (64 x 64)
    static constexpr int BM = 16 * TM_, BN = 16 * TM_, ROWB = 64, KE = ROWB / IN::BYTES, STAGES = 3, THREADS = 256;
    static constexpr int LOADS = TM_ / 4;             // direct loads per wave, operand and slab (a load fills 16 rows)
    static_assert(TM_ == 4 || TM_ == 8, "64 x 64 or 128 x 128 tiles");
    static constexpr int OPERAND_BYTES = BM * ROWB, STAGE_BYTES = 2 * OPERAND_BYTES, LDS_BYTES = STAGES * STAGE_BYTES;
    static constexpr int KU = 8 / IN::BYTES;          // K elements per 8-byte read unit
};

// element kk of an 8-byte unit in storage format -> fp32
template <typename IN>
__device__ __forceinline__ float unit_elem(const uint2& w, int kk)
{
    if constexpr (IN::ID == GEMM_F32) {
        return __uint_as_float(kk ? w.y : w.x);
    } else if constexpr (IN::ID == GEMM_BF16) {
        const uint32_t d = (kk >> 1) ? w.y : w.x;
        return __uint_as_float((kk & 1) ? (d & 0xFFFF0000u) : (d << 16));
    } else if constexpr (IN::ID == GEMM_F16) {
        const uint32_t d = (kk >> 1) ? w.y : w.x;
        return (float)__builtin_bit_cast(_Float16, (uint16_t)((kk & 1) ? (d >> 16) : (d & 0xFFFFu)));
    } else {
        const uint32_t d = (kk >> 2) ? w.y : w.x;
        switch (kk & 3) {                              // (the byte select is an immediate of the instruction)
        case 0: return __builtin_amdgcn_cvt_f32_fp8((int)d, 0);
        case 1: return __builtin_amdgcn_cvt_f32_fp8((int)d, 1);
        case 2: return __builtin_amdgcn_cvt_f32_fp8((int)d, 2);
        default: return __builtin_amdgcn_cvt_f32_fp8((int)d, 3);
        }
    }
}

// (three workgroups per CU fit LDS; the register budget is set to match: 168 per lane with 128 x 128 tiles)
template <typename IN, int TM_>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void valu_async(Args a)
{
    using CFG = AsyncCfg<IN, TM_>;
    constexpr int BM = CFG::BM, BN = CFG::BN, ROWB = CFG::ROWB, OPB = CFG::OPERAND_BYTES, KU = CFG::KU, TM = CFG::TM;
    static_assert(CFG::STAGES == 3, "the loop below is written for three stages");
    // one array per stage: the compiler orders LDS reads against pending direct loads by the array they name
    __shared__ __attribute__((aligned(1024))) char st0[CFG::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char st1[CFG::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char st2[CFG::STAGE_BYTES];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int tx = t & 15, ty = t >> 4;
    const int64_t b = blockIdx.z;
    const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;

    // ---- global -> LDS: lane L of a wave-wide 16-byte load lands at byte 16 L of a 1 KB block = 16 rows; it
    // fetches, for row L/4 of the block, the chunk whose swizzled position is L%4 ----
    const char* A = (const char*)a.A + (b * a.stride_a + m0 * a.a_si) * IN::BYTES;
    const char* B = (const char*)a.B + (b * a.stride_b + n0 * a.b_sj) * IN::BYTES;
    const int64_t bytes_a = ((a.M - 1 - m0) * a.a_si + a.K) * IN::BYTES;
    const int64_t bytes_b = ((a.N - 1 - n0) * a.b_sj + a.K) * IN::BYTES;
    constexpr int64_t CAP = 0xFFFFFFFFll;
    constexpr int RSRC_FLAGS = 0x00020000;               // raw buffer, 32-bit data format
    typedef __attribute__((ext_vector_type(4))) int rsrc_t;   // raw buffer descriptor: base, base high | stride 0, bytes, format
    auto desc = [&](const char* p, int64_t bytes) __attribute__((always_inline)) -> rsrc_t {
        const uint64_t u = (uint64_t)(uintptr_t)p;
        return rsrc_t{__builtin_amdgcn_readfirstlane((int)(uint32_t)u), __builtin_amdgcn_readfirstlane((int)(uint32_t)((u >> 32) & 0xFFFFu)),
                      __builtin_amdgcn_readfirstlane((int)(uint32_t)(bytes < CAP ? bytes : CAP)), RSRC_FLAGS};
    };
    const rsrc_t rsrc_a = desc(A, bytes_a), rsrc_b = desc(B, bytes_b);
    const int lrow = lane >> 2, gchunk = (lane & 3) ^ ((lane >> 4) & 3);      // (row 16 n + L/4: its (r/4)%4 is (L/16)%4)
    const int voff_a = (int)(lrow * a.a_si * IN::BYTES) + gchunk * 16;
    const int voff_b = (int)(lrow * a.b_sj * IN::BYTES) + gchunk * 16;
    const int blk_a = __builtin_amdgcn_readfirstlane((int)(16 * a.a_si * IN::BYTES)), blk_b = __builtin_amdgcn_readfirstlane((int)(16 * a.b_sj * IN::BYTES));   // bytes per block of 16 rows
    using lptr = __attribute__((address_space(3))) char*;
    // The loads are issued from inline assembly: the compiler orders LDS reads against the direct loads it knows to
    // be pending, and in a loop over stages it drains them (its own s_waitcnt vmcnt(0) ahead of the reads of every
    // third slab); the waits are placed by hand below instead.  One wait state separates the scalar write of M0 from
    // the load that reads it, five a vector instruction's write of a scalar register from a memory instruction
    // that reads it as descriptor or offset; the hardware interlocks neither and the compiler's hazard pass does
    // not look inside inline assembly, hence s_nop 4.  M0 is reserved (the compiler keeps nothing in it) and has no other user here.
    auto load_to_lds = [&](const rsrc_t& rsrc, int dst, int voff, int soff) __attribute__((always_inline)) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(dst), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
    };
    // slab s into stage `st`: TM blocks of 16 rows per operand, wave w takes blocks w (and w + 4) of each
    auto issue = [&](int64_t s, char* st) __attribute__((always_inline)) {
        const int k0 = (int)(s * ROWB);
        const int base = __builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)(lptr)st);
#pragma unroll
        for (int n = 0; n < CFG::LOADS; ++n) {
            const int blk = wave + 4 * n;
            load_to_lds(rsrc_a, base + blk * 1024, voff_a, k0 + blk * blk_a);
            load_to_lds(rsrc_b, base + OPB + blk * 1024, voff_b, k0 + blk * blk_b);
        }
    };

    // ---- LDS -> registers -> FMAs ----
    const int rd_a = ty * ROWB, rd_b = OPB + tx * ROWB;
    const int sw_a = (ty >> 2) & 3, sw_b = (tx >> 2) & 3;     // rows ty + 16 i and tx + 16 j: (r/4)%4 does not depend on i, j
    // An 8-byte read is served 16 lanes at a time from 32 banks: the 16 tx lanes read rows 64 bytes apart, and with
    // the chunk swizzle alone two rows would share each 8-byte slot.  Lanes with (tx/2)%2 = 1 therefore take the two
    // halves of a chunk in the other order (for A as well: a lane multiplies the same k of both operands).
    const int flip = (tx >> 1) & 1;
    float acc[TM][TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) acc[i][j] = 0.0f;

    // The slab's 64 bytes of K per row are consumed in eight 8-byte units; the reads of unit u + 1 are issued before
    // the FMAs of unit u (two register sets taken in turn).
    auto compute = [&](const char* st) __attribute__((always_inline)) {
        uint2 wa[2][TM], wb[2][TM];
        auto read_unit = [&](int u, int set) __attribute__((always_inline)) {
            const int half = (u & 1) ^ flip;               // which 8 bytes of the chunk this lane takes first
            const int pa = (((u >> 1) ^ sw_a) << 4) + half * 8, pb = (((u >> 1) ^ sw_b) << 4) + half * 8;
#pragma unroll
            for (int i = 0; i < TM; ++i) wa[set][i] = *(const uint2*)(st + rd_a + i * 16 * ROWB + pa);
#pragma unroll
            for (int j = 0; j < TM; ++j) wb[set][j] = *(const uint2*)(st + rd_b + j * 16 * ROWB + pb);
        };
        auto fma_unit = [&](int set) __attribute__((always_inline)) {
#pragma unroll
            for (int kk = 0; kk < KU; ++kk) {
                float bv[TM];
#pragma unroll
                for (int j = 0; j < TM; ++j) bv[j] = unit_elem<IN>(wb[set][j], kk);
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const float av = unit_elem<IN>(wa[set][i], kk);
#pragma unroll
                    for (int j = 0; j < TM; ++j) acc[i][j] = __builtin_fmaf(av, bv[j], acc[i][j]);
                }
            }
        };
        read_unit(0, 0);
#pragma unroll 1
        for (int u = 0; u < ROWB / 8; u += 2) {            // (a loop of four trips: unrolled, the reads gather at its top)
            read_unit(u + 1, 1);
            fma_unit(0);
            asm volatile("" ::: "memory");
            read_unit((u + 2) & (ROWB / 8 - 1), 0);        // (the last trip reads unit 0 once more: a valid address, unused)
            fma_unit(1);
            asm volatile("" ::: "memory");
        }
    };

    // One slab: wait until it has landed (this wave's share: everything but the 4 loads of the slab after it, when
    // that one was issued), meet the other waves (their shares have landed, and everyone has finished reading the
    // stage two slabs back), send the loads of the slab after next into that stage, multiply.
    const int64_t nslab = a.K / CFG::KE;                   // K is a whole number of slabs
    auto slab = [&](int64_t s, char* cur, char* free_stage) __attribute__((always_inline)) {
        if (s + 1 < nslab) {
            if constexpr (CFG::LOADS == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (s + 2 < nslab) issue(s + 2, free_stage);
        compute(cur);
    };
    if (nslab > 0) issue(0, st0);
    if (nslab > 1) issue(1, st1);
    int64_t s = 0;
    for (; s + 3 <= nslab; s += 3) {
        slab(s, st0, st2);
        slab(s + 1, st1, st0);
        slab(s + 2, st2, st1);
    }
    if (s < nslab) slab(s, st0, st2);
    if (s + 1 < nslab) slab(s + 1, st1, st0);

    const float sc = batch_scale(a, b);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t gi = m0 + ty + 16 * i;
        if (gi >= a.M) continue;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int64_t gj = n0 + tx + 16 * j;
            if (gj < a.N) store_out(a.C, b * a.stride_c + gi * a.ldc + gj, acc[i][j] * sc + (a.bias ? a.bias[gj] : 0.0f), a.out_dtype);
        }
    }
}

// K contiguous in both operands, K whole slabs, rows within the 32-bit byte offsets of a tile; the caller has
// checked that both operands take 16-byte loads.
bool k3_async_applies(const Args& a)
{
    if (a.flags != 0 || a.a_sk != 1 || a.b_sk != 1 || a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
    const int es = elem_size(a.in_dtype);
    if (a.K % (64 / es) != 0) return false;
    return a.a_si * es <= ((int64_t)1 << 22) && a.b_sj * es <= ((int64_t)1 << 22);
}

// 64 x 64 tiles when 128 x 128 tiles would leave most CUs without a workgroup (as the register-staged states do)
static bool async_small_tiles(const Args& a) { return ((a.M + 127) / 128) * ((a.N + 127) / 128) * a.batch < 256; }

template <int TM>
static hipError_t launch_async_tile(const Args& a)
{
    constexpr int BT = 16 * TM;
    dim3 block(256, 1, 1), grid((unsigned)((a.N + BT - 1) / BT), (unsigned)((a.M + BT - 1) / BT), (unsigned)a.batch);
    switch (a.in_dtype) {
    case GEMM_F32: hipLaunchKernelGGL((valu_async<F32, TM>), grid, block, 0, a.stream, a); break;
    case GEMM_BF16: hipLaunchKernelGGL((valu_async<BF16, TM>), grid, block, 0, a.stream, a); break;
    case GEMM_F16: hipLaunchKernelGGL((valu_async<F16, TM>), grid, block, 0, a.stream, a); break;
    default: hipLaunchKernelGGL((valu_async<E4M3, TM>), grid, block, 0, a.stream, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_k3_async(const Args& a) { return async_small_tiles(a) ? launch_async_tile<4>(a) : launch_async_tile<8>(a); }

Geometry geometry_k3_async(const Args& a)
{
    const bool small = async_small_tiles(a);
    const int bt = small ? 64 : 128;
    const int64_t g = ((a.N + bt - 1) / bt) * ((a.M + bt - 1) / bt) * a.batch;
    return Geometry{bt, bt, 64 / elem_size(a.in_dtype), 256, 3, small ? AsyncCfg<BF16, 4>::LDS_BYTES : AsyncCfg<BF16, 8>::LDS_BYTES, g};
}

}  // namespace gl
