// K0, the naive end of the lineage (paper Sec. 3.1: K_0): one thread per output element,
// both operands read straight from global memory through their strides, fp32 running sum.
#include "common.hpp"

namespace gl {

constexpr int K0_TX = 16, K0_TY = 16;

template <typename IN>
__global__ __launch_bounds__(K0_TX* K0_TY) void k0_naive(Args a)
{
    const int64_t j = (int64_t)blockIdx.x * K0_TX + threadIdx.x;
    const int64_t i = (int64_t)blockIdx.y * K0_TY + threadIdx.y;
    const int64_t b = blockIdx.z;
    if (i >= a.M || j >= a.N) return;
    const typename IN::raw* A = (const typename IN::raw*)a.A + b * a.stride_a + i * a.a_si;
    const typename IN::raw* B = (const typename IN::raw*)a.B + b * a.stride_b + j * a.b_sj;
    float acc = 0.0f;
    for (int64_t k = 0; k < a.K; ++k)
        acc = __builtin_fmaf(decode<IN>(A[k * a.a_sk]), decode<IN>(B[k * a.b_sk]), acc);
    store_out(a.C, b * a.stride_c + i * a.ldc + j, acc * batch_scale(a, b) + (a.bias ? a.bias[j] : 0.0f), a.out_dtype);
}

Geometry geometry_k0(const Args& a)
{
    const int64_t gx = (a.N + K0_TX - 1) / K0_TX, gy = (a.M + K0_TY - 1) / K0_TY;
    return Geometry{K0_TY, K0_TX, 1, K0_TX * K0_TY, 0, 0, gx * gy * a.batch};
}

hipError_t launch_k0(const Args& a)
{
    dim3 block(K0_TX, K0_TY, 1);
    dim3 grid((unsigned)((a.N + K0_TX - 1) / K0_TX), (unsigned)((a.M + K0_TY - 1) / K0_TY), (unsigned)a.batch);
    switch (a.in_dtype) {
    case GEMM_F32: hipLaunchKernelGGL(k0_naive<F32>, grid, block, 0, a.stream, a); break;
    case GEMM_BF16: hipLaunchKernelGGL(k0_naive<BF16>, grid, block, 0, a.stream, a); break;
    case GEMM_F16: hipLaunchKernelGGL(k0_naive<F16>, grid, block, 0, a.stream, a); break;
    default: hipLaunchKernelGGL(k0_naive<E4M3>, grid, block, 0, a.stream, a); break;
    }
    return hipGetLastError();
}

}  // namespace gl
