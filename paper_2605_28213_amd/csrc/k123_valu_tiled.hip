// K1, K2, K3: the vector-ALU part of the lineage (paper Table 1, "Staging & movement").
//
//   K1 = K0 + "tile / sm_stage"      each workgroup owns a BM x BN output tile and walks K in
//                                    BK slabs staged through LDS; each thread owns TM x TN outputs.
//   K2 = K1 + "vectorize_global"     slabs are fetched with 16-byte global loads along the
//                                    contiguous dimension.  Precondition (Table 1: 128-bit aligned
//                                    access; Sec. 1): base pointer
//                                    and leading dimension multiples of 16 bytes.  A vector that
//                                    crosses the M/N/K edge, or an operand that breaks the
//                                    precondition, is fetched element by element under a mask.
//   K3 = K2 + "pipeline"             two LDS buffers; slab s+1 travels global->registers while slab
//                                    s is consumed from LDS.  Precondition: staged data movement.
//                                    (This is K3's register-staged form, for operands its asynchronous
//                                    form in k3_async.hip does not take: K strided, K not whole
//                                    64-byte slabs, rows not 16-byte aligned.)
//
// "templatize" (Table 1): the tile shape and the two switches are template parameters, so each
// state is one instantiation of a single kernel and a transition is one changed constant.
#include "common.hpp"

namespace gl {

template <int BM_, int BN_, int BK_, int TM_, int TN_, bool VEC_, bool DBUF_>
struct ValuCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, TM = TM_, TN = TN_;
    static constexpr bool VEC = VEC_, DBUF = DBUF_;
    static constexpr int THREADS = (BM / TM) * (BN / TN);
    static constexpr int PAD = 4;
    static constexpr int NBUF = DBUF ? 2 : 1;
    static constexpr int LDS_BYTES = NBUF * BK * (BM + PAD + BN + PAD) * 4;
};
using CfgK1 = ValuCfg<64, 64, 16, 4, 4, false, false>;
using CfgK2 = ValuCfg<128, 128, 16, 8, 8, true, false>;
using CfgK3 = ValuCfg<128, 128, 16, 8, 8, true, true>;
// The same two states with 64 x 64 tiles, for problems whose 128 x 128 tiles would leave most CUs idle
// (fp32 256^3: 4 workgroups; 66 us with them against 24 us for K1's 16 workgroups).
using CfgK2Small = ValuCfg<64, 64, 16, 4, 4, true, false>;
using CfgK3Small = ValuCfg<64, 64, 16, 4, 4, true, true>;

// K2 / K3 with the vectorised loads taken out again (a validated simplification: GEMM_FLAG_DEOPT_NO_VECTOR)
using CfgK2NoVec = ValuCfg<128, 128, 16, 8, 8, false, false>;
using CfgK3NoVec = ValuCfg<128, 128, 16, 8, 8, false, true>;
using CfgK2SmallNoVec = ValuCfg<64, 64, 16, 4, 4, false, false>;
using CfgK3SmallNoVec = ValuCfg<64, 64, 16, 4, 4, false, true>;

static bool valu_small_tiles(const Args& a)
{
    return ((a.M + CfgK2::BM - 1) / CfgK2::BM) * ((a.N + CfgK2::BN - 1) / CfgK2::BN) * a.batch < 256;
}

// One operand's view of the current tile: `rows` is its M (for A) or N (for B) extent.
struct Operand {
    const void* base;
    int64_t sr, sk;   // element strides along the row dimension and along K
    int64_t rows;     // logical extent along the row dimension
    int64_t r0;       // first row of this workgroup's tile
    bool kcontig;     // K is the contiguous dimension
    bool vec_ok;      // 16-byte loads are legal for this operand
};

// Fetch one BR x BK slab into registers as fp32.  R[] holds EL = BR*BK/THREADS values (scalar)
// or ceil(BR*BK/V / THREADS) * V values (vector).
template <typename IN, int BR, int BK, int THREADS, bool VEC, int NREG>
__device__ __forceinline__ void fetch_slab(const Operand& x, int64_t k0, int64_t K, int t, float (&R)[NREG])
{
    using raw = typename IN::raw;
    const raw* p = (const raw*)x.base;
    if constexpr (!VEC) {
        constexpr int EL = BR * BK / THREADS;
        static_assert(EL == NREG, "register count");
#pragma unroll
        for (int n = 0; n < EL; ++n) {
            const int e = t + n * THREADS;
            const int k = x.kcontig ? e % BK : e / BR;
            const int r = x.kcontig ? e / BK : e % BR;
            const int64_t gr = x.r0 + r, gk = k0 + k;
            R[n] = (gr < x.rows && gk < K) ? decode<IN>(p[gr * x.sr + gk * x.sk]) : 0.0f;
        }
    } else {
        constexpr int V = 16 / IN::BYTES;
        constexpr int NV = BR * BK / V;
        constexpr int NVT = (NV + THREADS - 1) / THREADS;
        static_assert(NVT * V == NREG, "register count");
#pragma unroll
        for (int n = 0; n < NVT; ++n) {
            const int v = t + n * THREADS;
#pragma unroll
            for (int e = 0; e < V; ++e) R[n * V + e] = 0.0f;
            if (NV % THREADS != 0 && v >= NV) continue;
            int r, k;
            if (x.kcontig) { k = (v % (BK / V)) * V; r = v / (BK / V); }
            else           { r = (v % (BR / V)) * V; k = v / (BR / V); }
            const int64_t gr = x.r0 + r, gk = k0 + k;
            if (gr >= x.rows || gk >= K) continue;
            const int64_t along = x.kcontig ? K - gk : x.rows - gr;   // elements left before the edge
            const raw* q = p + gr * x.sr + gk * x.sk;
            if (x.vec_ok && along >= V) {
                const uint4 w = *(const uint4*)q;
                raw tmp[V];
                __builtin_memcpy(tmp, &w, 16);
#pragma unroll
                for (int e = 0; e < V; ++e) R[n * V + e] = decode<IN>(tmp[e]);
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e)
                    if (e < along) R[n * V + e] = decode<IN>(q[e]);   // stride along the contiguous dim is 1
            }
        }
    }
}

// Write the registers fetched above into the LDS slab S[k][r].
template <typename IN, int BR, int BK, int THREADS, bool VEC, int NREG, int LD>
__device__ __forceinline__ void commit_slab(bool kcontig, int t, const float (&R)[NREG], float (*S)[LD])
{
    if constexpr (!VEC) {
        constexpr int EL = BR * BK / THREADS;
#pragma unroll
        for (int n = 0; n < EL; ++n) {
            const int e = t + n * THREADS;
            const int k = kcontig ? e % BK : e / BR;
            const int r = kcontig ? e / BK : e % BR;
            S[k][r] = R[n];
        }
    } else {
        constexpr int V = 16 / IN::BYTES;
        constexpr int NV = BR * BK / V;
        constexpr int NVT = (NV + THREADS - 1) / THREADS;
#pragma unroll
        for (int n = 0; n < NVT; ++n) {
            const int v = t + n * THREADS;
            if (NV % THREADS != 0 && v >= NV) continue;
            if (kcontig) {
                const int k = (v % (BK / V)) * V, r = v / (BK / V);
#pragma unroll
                for (int e = 0; e < V; ++e) S[k + e][r] = R[n * V + e];
            } else {
                const int r = (v % (BR / V)) * V, k = v / (BR / V);
#pragma unroll
                for (int e = 0; e < V; e += 4)
                    *(float4*)&S[k][r + e] = make_float4(R[n * V + e], R[n * V + e + 1], R[n * V + e + 2], R[n * V + e + 3]);
            }
        }
    }
}

template <typename IN, typename CFG>
__global__ __launch_bounds__(CFG::THREADS) void valu_tiled(Args a, int vec_mask)
{
    constexpr int BM = CFG::BM, BN = CFG::BN, BK = CFG::BK, TM = CFG::TM, TN = CFG::TN;
    constexpr int T = CFG::THREADS, PAD = CFG::PAD, NBUF = CFG::NBUF;
    constexpr bool VEC = CFG::VEC;
    constexpr int V = 16 / IN::BYTES;
    constexpr int NRA = VEC ? ((BM * BK / V + T - 1) / T) * V : BM * BK / T;
    constexpr int NRB = VEC ? ((BN * BK / V + T - 1) / T) * V : BN * BK / T;
    constexpr int CM = TM / 4, CN = TN / 4;        // 4-wide chunks per thread, BM/CM (BN/CN) rows apart

    __shared__ __attribute__((aligned(16))) float As[NBUF][BK][BM + PAD];
    __shared__ __attribute__((aligned(16))) float Bs[NBUF][BK][BN + PAD];

    const int t = threadIdx.x;
    const int tx = t % (BN / TN), ty = t / (BN / TN);
    const int64_t b = blockIdx.z;
    const int es = IN::BYTES;

    Operand oa{(const char*)a.A + b * a.stride_a * es, a.a_si, a.a_sk, a.M, (int64_t)blockIdx.y * BM,
               a.a_sk == 1, (vec_mask & 1) != 0};
    Operand ob{(const char*)a.B + b * a.stride_b * es, a.b_sj, a.b_sk, a.N, (int64_t)blockIdx.x * BN,
               a.b_sk == 1, (vec_mask & 2) != 0};

    float acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0.0f;

    float ra[NRA], rb[NRB];

    // Pipelined state: the k loop is unrolled by 2 only.  Fully unrolled, with the next slab's global
    // loads in flight, the scheduler gathers all BK steps' LDS reads at the top of the block (~400
    // registers, one wave per SIMD); two steps keep the reads next to their FMAs.
    constexpr int KUNROLL = CFG::DBUF ? 2 : BK;
    auto compute = [&](int buf) {
#pragma unroll KUNROLL
        for (int kk = 0; kk < BK; ++kk) {
            float av[TM], bv[TN];
#pragma unroll
            for (int c = 0; c < CM; ++c) {
                const float4 w = *(const float4*)&As[buf][kk][c * (BM / CM) + ty * 4];
                av[c * 4 + 0] = w.x; av[c * 4 + 1] = w.y; av[c * 4 + 2] = w.z; av[c * 4 + 3] = w.w;
            }
#pragma unroll
            for (int c = 0; c < CN; ++c) {
                const float4 w = *(const float4*)&Bs[buf][kk][c * (BN / CN) + tx * 4];
                bv[c * 4 + 0] = w.x; bv[c * 4 + 1] = w.y; bv[c * 4 + 2] = w.z; bv[c * 4 + 3] = w.w;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_fmaf(av[i], bv[j], acc[i][j]);
        }
    };

    const int64_t nslab = (a.K + BK - 1) / BK;
    if constexpr (!CFG::DBUF) {
        for (int64_t s = 0; s < nslab; ++s) {
            fetch_slab<IN, BM, BK, T, VEC>(oa, s * BK, a.K, t, ra);
            fetch_slab<IN, BN, BK, T, VEC>(ob, s * BK, a.K, t, rb);
            commit_slab<IN, BM, BK, T, VEC>(oa.kcontig, t, ra, As[0]);
            commit_slab<IN, BN, BK, T, VEC>(ob.kcontig, t, rb, Bs[0]);
            __syncthreads();
            compute(0);
            __syncthreads();
        }
    } else {
        int cur = 0;
        if (nslab > 0) {
            fetch_slab<IN, BM, BK, T, VEC>(oa, 0, a.K, t, ra);
            fetch_slab<IN, BN, BK, T, VEC>(ob, 0, a.K, t, rb);
            commit_slab<IN, BM, BK, T, VEC>(oa.kcontig, t, ra, As[0]);
            commit_slab<IN, BN, BK, T, VEC>(ob.kcontig, t, rb, Bs[0]);
        }
        __syncthreads();
        for (int64_t s = 0; s < nslab; ++s) {
            const bool more = s + 1 < nslab;
            if (more) {   // next slab: global -> registers, in flight during the FMAs below
                fetch_slab<IN, BM, BK, T, VEC>(oa, (s + 1) * BK, a.K, t, ra);
                fetch_slab<IN, BN, BK, T, VEC>(ob, (s + 1) * BK, a.K, t, rb);
            }
            compute(cur);
            if (more) {   // the other buffer was last read before the previous barrier
                commit_slab<IN, BM, BK, T, VEC>(oa.kcontig, t, ra, As[cur ^ 1]);
                commit_slab<IN, BN, BK, T, VEC>(ob.kcontig, t, rb, Bs[cur ^ 1]);
            }
            __syncthreads();
            cur ^= 1;
        }
    }

    const float s = batch_scale(a, b);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t gi = oa.r0 + (i / 4) * (BM / CM) + ty * 4 + (i % 4);
        if (gi >= a.M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t gj = ob.r0 + (j / 4) * (BN / CN) + tx * 4 + (j % 4);
            if (gj < a.N) store_out(a.C, b * a.stride_c + gi * a.ldc + gj, acc[i][j] * s + (a.bias ? a.bias[gj] : 0.0f), a.out_dtype);
        }
    }
}

template <typename CFG>
static hipError_t launch_cfg(const Args& a, int vec_mask)
{
    dim3 block(CFG::THREADS, 1, 1);
    dim3 grid((unsigned)((a.N + CFG::BN - 1) / CFG::BN), (unsigned)((a.M + CFG::BM - 1) / CFG::BM), (unsigned)a.batch);
    switch (a.in_dtype) {
    case GEMM_F32: hipLaunchKernelGGL((valu_tiled<F32, CFG>), grid, block, 0, a.stream, a, vec_mask); break;
    case GEMM_BF16: hipLaunchKernelGGL((valu_tiled<BF16, CFG>), grid, block, 0, a.stream, a, vec_mask); break;
    case GEMM_F16: hipLaunchKernelGGL((valu_tiled<F16, CFG>), grid, block, 0, a.stream, a, vec_mask); break;
    default: hipLaunchKernelGGL((valu_tiled<E4M3, CFG>), grid, block, 0, a.stream, a, vec_mask); break;
    }
    return hipGetLastError();
}

template <typename CFG>
static Geometry geometry_cfg(const Args& a)
{
    const int64_t g = ((a.N + CFG::BN - 1) / CFG::BN) * ((a.M + CFG::BM - 1) / CFG::BM) * a.batch;
    return Geometry{CFG::BM, CFG::BN, CFG::BK, CFG::THREADS, CFG::NBUF, CFG::LDS_BYTES, g};
}

// `path` is the bitmask of operands whose 16-byte loads are legal (bit 0: A, bit 1: B); K1 ignores it.
hipError_t launch_valu_tiled(int variant, int path, const Args& a)
{
    switch (variant) {
    case GEMM_K1_LDS_TILED: return launch_cfg<CfgK1>(a, 0);
    case GEMM_K2_VECTORIZED:
        if (a.flags & GEMM_FLAG_DEOPT_NO_VECTOR) return valu_small_tiles(a) ? launch_cfg<CfgK2SmallNoVec>(a, 0) : launch_cfg<CfgK2NoVec>(a, 0);
        return valu_small_tiles(a) ? launch_cfg<CfgK2Small>(a, path) : launch_cfg<CfgK2>(a, path);
    case GEMM_K3_PIPELINED:
        if (a.flags & GEMM_FLAG_DEOPT_NO_VECTOR) return valu_small_tiles(a) ? launch_cfg<CfgK3SmallNoVec>(a, 0) : launch_cfg<CfgK3NoVec>(a, 0);
        return valu_small_tiles(a) ? launch_cfg<CfgK3Small>(a, path) : launch_cfg<CfgK3>(a, path);
    default: return hipErrorInvalidValue;
    }
}

Geometry geometry_valu_tiled(int variant, int, const Args& a)
{
    switch (variant) {
    case GEMM_K1_LDS_TILED: return geometry_cfg<CfgK1>(a);
    case GEMM_K2_VECTORIZED: return valu_small_tiles(a) ? geometry_cfg<CfgK2Small>(a) : geometry_cfg<CfgK2>(a);
    default: return valu_small_tiles(a) ? geometry_cfg<CfgK3Small>(a) : geometry_cfg<CfgK3>(a);
    }
}

}  // namespace gl
