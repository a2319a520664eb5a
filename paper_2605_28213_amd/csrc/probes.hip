// Measurement probes: three plain kernels whose results say what the machine at hand sustains, so
// that a roofline fraction can be read against a measured ceiling next to the published peak.
//   copy         16-byte grid-stride copy of a known number of bytes: the unit against which HBM
//                byte counters (FETCH_SIZE / WRITE_SIZE) are calibrated
//   stream read  the same loads without the stores: achievable HBM read bandwidth
//   mfma         a register-resident loop of the expert kernel's matrix instruction with the expert
//                kernel's accumulator shape (4x4 tiles of 32x32 per wave, one wave per SIMD), operands
//                taken from a caller buffer: the rate, and through it the clock, the matrix pipe holds
//                on this data when nothing else competes for power
// None of them is part of the lineage; none is used by gemm_run*.
#include "k4_kernels.hpp"

namespace gl {

__global__ __launch_bounds__(256) void probe_copy(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src, size_t n16)
{
    constexpr int U = 4;
    const size_t stride = (size_t)gridDim.x * 256 * U;
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n16; i += stride) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i + 256 * u < n16) v[u] = __builtin_nontemporal_load(src + i + 256 * u);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i + 256 * u < n16) __builtin_nontemporal_store(v[u], dst + i + 256 * u);
    }
}

__global__ __launch_bounds__(256) void probe_stream_read(const u32x4_t* __restrict__ src, size_t n16, uint32_t* sink)
{
    constexpr int U = 8;
    const size_t stride = (size_t)gridDim.x * 256 * U;
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n16; i += stride) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = (i + 256 * u < n16) ? __builtin_nontemporal_load(src + i + 256 * u) : u32x4_t{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;     // practically never true: keeps the loads alive
}

// Two operand sets of 4 + 4 fragments per lane, 2 x 16 MFMAs per iteration, accumulators never leave
// their registers.  Lane l of workgroup w reads fragments from operands + (w*256 + l) * FRAG_BYTES.
template <typename IN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void probe_mfma(const char* __restrict__ operands, int iters, float* sink)
{
    constexpr int NS = 2;
    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    Frag<IN> fa[NS][4], fb[NS][4];
    constexpr int PER_LANE = NS * 8 * Frag<IN>::CPS;           // 16-byte chunks per lane
    const u32x4_t* p = (const u32x4_t*)operands + ((size_t)blockIdx.x * 256 + threadIdx.x) * PER_LANE;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int q = 0; q < Frag<IN>::CPS; ++q) {
                fa[s][i].c[q] = p[((s * 8 + i) * Frag<IN>::CPS) + q];
                fb[s][i].c[q] = p[((s * 8 + 4 + i) * Frag<IN>::CPS) + q];
            }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int j = (i & 1) ? 3 - jj : jj;
                    mfma_step<IN>(fb[s][j], fa[s][i], acc[i][j]);
                }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// The same loop with v_mfma_f32_16x16x32 (two-byte types): 8 x 8 accumulator tiles of 16 x 16 per wave, two k-steps of
// 64 instructions per iteration -- the flops of two iterations of the loop above, on twice the operand bytes per lane.
template <typename IN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void probe_mfma16(const char* __restrict__ operands, int iters, float* sink)
{
    f32x4_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_t{0, 0, 0, 0};
    u32x4_t fa[2][8], fb[2][8];
    const u32x4_t* p = (const u32x4_t*)operands + ((size_t)blockIdx.x * 256 + threadIdx.x) * 32;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) { fa[s][i] = p[s * 16 + i]; fb[s][i] = p[s * 16 + 8 + i]; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const int j = (i & 1) ? 7 - jj : jj;
                    // From inline assembly, with the accumulator tile tied to its registers: through the builtin the
                    // compiler shuffled 80 of the 256 accumulator registers between the register files per 128
                    // instructions at the loop's back edge, and the loop then measured those moves (2100 instead of
                    // 2400 TFLOP/s on zeros).  The loop holds nothing but matrix instructions, which interlock.
                    if constexpr (IN::ID == GEMM_BF16)
                        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[s][j]), "v"(fa[s][i]));
                    else
                        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[s][j]), "v"(fa[s][i]));
                }
    }
    // (the compiler does not know that the statements above are matrix instructions: the wait states their results
    // need before a vector instruction may read them, placed by hand)
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[i][j][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace gl

using namespace gl;

extern "C" {

int gemm_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || bytes == 0 || bytes % 16 || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return GEMM_ERR_BAD_ARG;
    (void)hipGetLastError();
    hipLaunchKernelGGL(probe_copy, dim3(4096), dim3(256), 0, (hipStream_t)stream, (u32x4_t*)dst, (const u32x4_t*)src, bytes / 16);
    return hipGetLastError() == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

int gemm_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 || ((uintptr_t)src & 15u)) return GEMM_ERR_BAD_ARG;
    (void)hipGetLastError();
    hipLaunchKernelGGL(probe_stream_read, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const u32x4_t*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

size_t gemm_probe_mfma_operand_bytes(int dtype, int workgroups)
{
    if (workgroups < 1 || (dtype != GEMM_BF16 && dtype != GEMM_F16 && dtype != GEMM_FP8_E4M3)) return 0;
    return (size_t)workgroups * 256 * 2 * 8 * (dtype == GEMM_FP8_E4M3 ? 2 : 1) * 16;
}

int gemm_probe_mfma(int dtype, const void* operands, size_t operand_bytes, int workgroups, int iters, void* sink,
                    size_t sink_bytes, double* flops, void* stream)
{
    const size_t need = gemm_probe_mfma_operand_bytes(dtype, workgroups);
    if (need == 0) return GEMM_ERR_UNSUPPORTED_DTYPE;
    if (!operands || !sink || iters < 1 || ((uintptr_t)operands & 15u)) return GEMM_ERR_BAD_ARG;
    if (operand_bytes < need || sink_bytes < (size_t)workgroups * 256 * sizeof(float)) return GEMM_ERR_BAD_ARG;
    const double per_mfma = dtype == GEMM_FP8_E4M3 ? 2.0 * 32 * 32 * 64 : 2.0 * 32 * 32 * 16;
    if (flops) *flops = (double)workgroups * 4 * iters * 2 * 16 * per_mfma;
    dim3 grid((unsigned)workgroups), block(256);
    (void)hipGetLastError();
    hipStream_t st = (hipStream_t)stream;
    if (dtype == GEMM_BF16) hipLaunchKernelGGL(probe_mfma<BF16>, grid, block, 0, st, (const char*)operands, iters, (float*)sink);
    else if (dtype == GEMM_F16) hipLaunchKernelGGL(probe_mfma<F16>, grid, block, 0, st, (const char*)operands, iters, (float*)sink);
    else hipLaunchKernelGGL(probe_mfma<E4M3>, grid, block, 0, st, (const char*)operands, iters, (float*)sink);
    return hipGetLastError() == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

int gemm_probe_mfma16(int dtype, const void* operands, size_t operand_bytes, int workgroups, int iters, void* sink,
                      size_t sink_bytes, double* flops, void* stream)
{
    if (dtype != GEMM_BF16 && dtype != GEMM_F16) return GEMM_ERR_UNSUPPORTED_DTYPE;
    const size_t need = 2 * gemm_probe_mfma_operand_bytes(dtype, workgroups);  // 32 chunks of 16 bytes per lane: twice the other loop's
    if (need == 0 || !operands || !sink || iters < 1 || ((uintptr_t)operands & 15u)) return GEMM_ERR_BAD_ARG;
    if (operand_bytes < need || sink_bytes < (size_t)workgroups * 256 * sizeof(float)) return GEMM_ERR_BAD_ARG;
    if (flops) *flops = (double)workgroups * 4 * iters * 2 * 64 * (2.0 * 16 * 16 * 32);
    dim3 grid((unsigned)workgroups), block(256);
    (void)hipGetLastError();
    hipStream_t st = (hipStream_t)stream;
    if (dtype == GEMM_BF16) hipLaunchKernelGGL(probe_mfma16<BF16>, grid, block, 0, st, (const char*)operands, iters, (float*)sink);
    else hipLaunchKernelGGL(probe_mfma16<F16>, grid, block, 0, st, (const char*)operands, iters, (float*)sink);
    return hipGetLastError() == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

}  // extern "C"
