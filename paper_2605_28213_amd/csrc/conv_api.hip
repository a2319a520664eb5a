// Convolution layer (paper Sec. 4.1 workload table: Conv2d; Sec. 4.2: "im2col + tensor core"): the two
// kernels of its own that the layer's lineage needs (direct, im2col), and the C ABI that dispatches a
// state either to them or to the GEMM lineage's K4 kernel (plain for C1, gathering for C2).
#include <stdio.h>
#include <string.h>

#include "../../include/conv_lineage.h"
#include "common.hpp"

using namespace gl;

namespace {

struct ConvArgs {
    const void* x;
    const void* w;
    void* y;
    const float* bias;
    int64_t N, H, W, C, F, R, S, P, Q;
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t in_dtype, out_dtype;
};

// C0: one thread per output element (filters fastest), the definition's loops in its order.
template <typename IN>
__global__ __launch_bounds__(256) void conv_direct(ConvArgs a)
{
    using raw = typename IN::raw;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.N * a.P * a.Q * a.F) return;
    const int64_t f = idx % a.F, pix = idx / a.F;
    const int64_t q = pix % a.Q, p = (pix / a.Q) % a.P, n = pix / (a.P * a.Q);
    const raw* x = (const raw*)a.x;
    const raw* w = (const raw*)a.w;
    float acc = 0.0f;
    for (int64_t r = 0; r < a.R; ++r) {
        const int64_t h = p * a.stride_h - a.pad_h + r;
        if (h < 0 || h >= a.H) continue;
        for (int64_t s = 0; s < a.S; ++s) {
            const int64_t ww = q * a.stride_w - a.pad_w + s;
            if (ww < 0 || ww >= a.W) continue;
            const raw* xp = x + ((n * a.H + h) * a.W + ww) * a.C;
            const raw* wp = w + ((f * a.R + r) * a.S + s) * a.C;
            for (int64_t c = 0; c < a.C; ++c) acc = __builtin_fmaf(decode<IN>(xp[c]), decode<IN>(wp[c]), acc);
        }
    }
    store_out(a.y, idx, acc + (a.bias ? a.bias[f] : 0.0f), a.out_dtype);
}

// C1, first pass: the patch matrix [N*P*Q][Kp], K = (r, s, c) with c fastest, zero-filled where a tap
// lies in the padding and from K up to Kp (K rounded up to whole 128-byte slabs).  One thread per
// 16-byte chunk of the destination; with `vec` (C a multiple of the chunk, x 16-byte aligned) a chunk
// never straddles two taps and is one 16-byte load.
template <typename IN>
__global__ __launch_bounds__(256) void conv_im2col(ConvArgs a, char* dst, int64_t K, int64_t Kp, int vec)
{
    using raw = typename IN::raw;
    constexpr int V = 16 / IN::BYTES;
    const int64_t cpr = Kp / V;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.N * a.P * a.Q * cpr) return;
    const int64_t m = idx / cpr, k0 = (idx % cpr) * V;
    const int64_t q = m % a.Q, p = (m / a.Q) % a.P, n = m / (a.P * a.Q);
    const raw* x = (const raw*)a.x;
    uint4 out = make_uint4(0, 0, 0, 0);
    auto element = [&](int64_t k) -> const raw* {       // address of K index k of this row, or null in the padding
        const int64_t tap = k / a.C, c = k % a.C, r = tap / a.S, s = tap % a.S;
        const int64_t h = p * a.stride_h - a.pad_h + r, ww = q * a.stride_w - a.pad_w + s;
        if (h < 0 || h >= a.H || ww < 0 || ww >= a.W) return nullptr;
        return x + ((n * a.H + h) * a.W + ww) * a.C + c;
    };
    if (vec) {
        if (k0 < K) {
            const raw* src = element(k0);
            if (src) out = *(const uint4*)src;
        }
    } else {
        raw tmp[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const raw* src = k0 + e < K ? element(k0 + e) : nullptr;
            tmp[e] = src ? *src : (raw)0;
        }
        __builtin_memcpy(&out, tmp, 16);
    }
    *(uint4*)(dst + (m * Kp + k0) * IN::BYTES) = out;
}

// C1: filters copied to rows of Kp elements (zero tail) when K is not a whole number of slabs or w is
// not 16-byte aligned.  One thread per 16-byte chunk of the destination.
template <typename IN>
__global__ __launch_bounds__(256) void conv_pad_rows(const void* src, char* dst, int64_t rows, int64_t K, int64_t Kp)
{
    using raw = typename IN::raw;
    constexpr int V = 16 / IN::BYTES;
    const int64_t cpr = Kp / V;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * cpr) return;
    const int64_t f = idx / cpr, k0 = (idx % cpr) * V;
    raw tmp[V];
#pragma unroll
    for (int e = 0; e < V; ++e) tmp[e] = k0 + e < K ? ((const raw*)src)[f * K + k0 + e] : (raw)0;
    uint4 out;
    __builtin_memcpy(&out, tmp, 16);
    *(uint4*)(dst + (f * Kp + k0) * IN::BYTES) = out;
}

struct Plan {
    int status = GEMM_OK;
    bool empty = false;
    ConvArgs c{};
    Args g{};               // the matrix product of C1 / C2
    int64_t K = 0, Kp = 0;
    bool pad_w = false;     // C1: filters need their padded copy
    hipStream_t stream = nullptr;
    void* workspace = nullptr;
    conv2d_query_t q{};
};

Plan make_plan(int variant, const conv2d_desc_t* d, const void* x, const void* w, const void* y, bool need_ptrs)
{
    Plan p;
    auto fail = [&](int s) { p.status = s; return p; };
    if (variant < 0 || variant >= CONV_VARIANT_COUNT) return fail(GEMM_ERR_BAD_VARIANT);
    if (!d) return fail(GEMM_ERR_BAD_ARG);
    if (d->N < 0 || d->F < 0 || d->H < 1 || d->W < 1 || d->C < 1 || d->R < 1 || d->S < 1) return fail(GEMM_ERR_BAD_ARG);
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0 || d->flags != 0 || d->reserved != 0) return fail(GEMM_ERR_BAD_ARG);
    const int64_t lim = (int64_t)1 << 30;
    if (d->N > lim || d->H > 65535 || d->W > 65535 || d->C > lim || d->F > lim || d->R > 255 || d->S > 255 ||
        d->stride_h > 255 || d->stride_w > 255 || d->pad_h > 255 || d->pad_w > 255)
        return fail(GEMM_ERR_BAD_ARG);
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return fail(GEMM_ERR_BAD_ARG);
    if (d->in_dtype < 0 || d->in_dtype > GEMM_FP8_E4M3 || d->out_dtype < 0 || d->out_dtype > GEMM_FP8_E4M3) return fail(GEMM_ERR_UNSUPPORTED_DTYPE);
    if (!dtype_pair_supported(d->in_dtype, d->out_dtype)) return fail(GEMM_ERR_UNSUPPORTED_DTYPE);
    const int64_t P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1, Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    const int64_t M = d->N * P * Q, K = d->R * d->S * d->C;
    if (M > lim || K > lim || M * d->F >= ((int64_t)1 << 40)) return fail(GEMM_ERR_BAD_ARG);
    p.empty = M == 0 || d->F == 0;
    if (need_ptrs && !p.empty && (!x || !w || !y)) return fail(GEMM_ERR_BAD_ARG);

    const int es = elem_size(d->in_dtype);
    const int64_t KE = 128 / es, Kp = (K + KE - 1) / KE * KE;
    // rows of both operands of the product are addressed with 32-bit byte offsets inside a tile
    if (variant != CONV_C0_DIRECT && d->in_dtype != GEMM_F32 && Kp * es > ((int64_t)1 << 22)) return fail(GEMM_ERR_BAD_ARG);
    p.K = K; p.Kp = Kp;
    p.stream = (hipStream_t)d->stream;
    p.workspace = d->workspace;

    ConvArgs& c = p.c;
    c.x = x; c.w = w; c.y = (void*)y; c.bias = d->bias;
    c.N = d->N; c.H = d->H; c.W = d->W; c.C = d->C; c.F = d->F; c.R = d->R; c.S = d->S; c.P = P; c.Q = Q;
    c.stride_h = d->stride_h; c.stride_w = d->stride_w; c.pad_h = d->pad_h; c.pad_w = d->pad_w;
    c.in_dtype = d->in_dtype; c.out_dtype = d->out_dtype;

    const int64_t x_bytes = d->N * d->H * d->W * d->C * es;
    uint32_t holds = 0;
    if (!x || ((uintptr_t)x & 15u) == 0) holds |= CONV_COND_ALIGN16_X;
    if (!w || ((uintptr_t)w & 15u) == 0) holds |= CONV_COND_ALIGN16_W;
    if (!y || ((uintptr_t)y & 15u) == 0) holds |= CONV_COND_ALIGN16_Y;
    if ((d->C * es) % 128 == 0) holds |= CONV_COND_C_WHOLE_SLABS;
    if (d->in_dtype != GEMM_F32) holds |= CONV_COND_DTYPE_ON_FAST_KERNEL;
    if (x_bytes < ((int64_t)1 << 31)) holds |= CONV_COND_X_BELOW_2GIB;

    // the matrix product both MFMA states run: rows = output pixels, columns = filters
    Args& g = p.g;
    g.C = (void*)y; g.bias = d->bias;
    g.M = M; g.N = d->F; g.batch = 1;
    g.a_sk = 1; g.b_sk = 1; g.ldc = d->F;
    g.in_dtype = d->in_dtype; g.out_dtype = d->out_dtype;
    g.stream = p.stream;

    uint32_t required = 0;
    size_t need = 0;
    Geometry geo{};
    const char* path = "";
    switch (variant) {
    case CONV_C0_DIRECT:
        path = "direct";
        geo = Geometry{0, 0, 0, 256, 0, 0, (M * d->F + 255) / 256};
        if (geo.grid >= ((int64_t)1 << 31)) return fail(GEMM_ERR_BAD_ARG);
        break;
    case CONV_C1_IM2COL_MFMA: {
        required = CONV_COND_DTYPE_ON_FAST_KERNEL | CONV_COND_SCRATCH_LENT;
        p.pad_w = Kp != K || !(holds & CONV_COND_ALIGN16_W);
        need = (size_t)(M * Kp * es) + (p.pad_w ? (size_t)(d->F * Kp * es) : 0);
        if (d->workspace && d->workspace_bytes >= need && ((uintptr_t)d->workspace & 15u) == 0) holds |= CONV_COND_SCRATCH_LENT;
        g.A = d->workspace;
        g.B = p.pad_w ? (const void*)((const char*)d->workspace + M * Kp * es) : w;
        g.K = Kp; g.a_si = Kp; g.b_sj = Kp;
        path = p.pad_w ? "im2col+pad(w)+mfma32-direct-to-lds" : "im2col+mfma32-direct-to-lds";
        if (holds & CONV_COND_DTYPE_ON_FAST_KERNEL) geo = geometry_k4(MFMA_VEC16, g);
        if ((M * (Kp / (16 / es)) + 255) / 256 >= ((int64_t)1 << 31)) return fail(GEMM_ERR_BAD_ARG);
        break;
    }
    default: {  // CONV_C2_IMPLICIT_MFMA
        required = CONV_COND_DTYPE_ON_FAST_KERNEL | CONV_COND_C_WHOLE_SLABS | CONV_COND_ALIGN16_X | CONV_COND_ALIGN16_W | CONV_COND_X_BELOW_2GIB;
        g.A = x; g.B = w;
        g.K = K; g.a_si = 0; g.b_sj = K;
        g.conv = ConvGeom{(int32_t)d->H, (int32_t)d->W, (int32_t)d->C, (int32_t)P, (int32_t)Q, (int32_t)d->S,
                          d->stride_h, d->stride_w, d->pad_h, d->pad_w, (int32_t)(d->C * es / 128), (uint32_t)x_bytes};
        path = "implicit-gather+mfma32-direct-to-lds";
        if (holds & CONV_COND_DTYPE_ON_FAST_KERNEL) geo = geometry_k4_conv(g);
        break;
    }
    }

    conv2d_query_t& q = p.q;
    q.required = required; q.holds = holds; q.violated = required & ~holds;
    q.P = P; q.Q = Q; q.gemm_m = M; q.gemm_n = d->F; q.gemm_k = K;
    q.bm = geo.bm; q.bn = geo.bn; q.bk = geo.bk; q.threads = geo.threads; q.lds_bytes = geo.lds_bytes;
    q.grid = p.empty ? 0 : geo.grid;
    q.workspace_bytes = need;
    strncpy(q.path, path, sizeof(q.path) - 1);

    if (q.violated & ~(uint32_t)CONV_COND_SCRATCH_LENT) p.status = GEMM_ERR_PRECONDITION;
    else if (q.violated & CONV_COND_SCRATCH_LENT) p.status = GEMM_ERR_WORKSPACE;
    return p;
}

template <typename IN>
hipError_t launch_direct(const Plan& p)
{
    const int64_t total = p.c.N * p.c.P * p.c.Q * p.c.F;
    hipLaunchKernelGGL(conv_direct<IN>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, p.stream, p.c);
    return hipGetLastError();
}

template <typename IN>
hipError_t launch_im2col(const Plan& p)
{
    constexpr int V = 16 / IN::BYTES;
    const int64_t M = p.g.M, chunks = M * (p.Kp / V);
    const int vec = p.c.C % V == 0 && ((uintptr_t)p.c.x & 15u) == 0;
    hipLaunchKernelGGL(conv_im2col<IN>, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, p.stream, p.c, (char*)p.workspace, p.K, p.Kp, vec);
    if (p.pad_w) {
        const int64_t wchunks = p.c.F * (p.Kp / V);
        hipLaunchKernelGGL(conv_pad_rows<IN>, dim3((unsigned)((wchunks + 255) / 256)), dim3(256), 0, p.stream, p.c.w,
                           (char*)p.workspace + M * p.Kp * IN::BYTES, p.c.F, p.K, p.Kp);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_k4(MFMA_VEC16 | (3 << 8), p.g);
}

thread_local hipError_t last_conv_launch_error = hipSuccess;

}  // namespace

extern "C" {

int conv2d_default_desc(conv2d_desc_t* d, int64_t N, int64_t H, int64_t W, int64_t C, int64_t F, int64_t R, int64_t S, int dtype)
{
    if (!d) return GEMM_ERR_BAD_ARG;
    if (dtype < 0 || dtype > GEMM_FP8_E4M3) return GEMM_ERR_UNSUPPORTED_DTYPE;
    if (N < 0 || H < 1 || W < 1 || C < 1 || F < 0 || R < 1 || S < 1 || R > 255 || S > 255) return GEMM_ERR_BAD_ARG;
    memset(d, 0, sizeof(*d));
    d->N = N; d->H = H; d->W = W; d->C = C; d->F = F; d->R = R; d->S = S;
    d->stride_h = d->stride_w = 1;
    d->pad_h = (int32_t)(R / 2); d->pad_w = (int32_t)(S / 2);
    d->in_dtype = dtype;
    d->out_dtype = dtype == GEMM_FP8_E4M3 ? GEMM_BF16 : dtype;
    return GEMM_OK;
}

int conv2d_query(int variant, const conv2d_desc_t* d, const void* x, const void* w, const void* y, conv2d_query_t* out)
{
    if (!out) return GEMM_ERR_BAD_ARG;
    Plan p = make_plan(variant, d, x, w, y, /*need_ptrs=*/false);
    memset(out, 0, sizeof(*out));
    if (p.status == GEMM_OK || p.status == GEMM_ERR_PRECONDITION || p.status == GEMM_ERR_WORKSPACE) *out = p.q;
    return p.status;
}

int conv2d_run(int variant, const conv2d_desc_t* d, const void* x, const void* w, void* y)
{
    Plan p = make_plan(variant, d, x, w, y, /*need_ptrs=*/true);
    if (p.status != GEMM_OK) return p.status;
    if (p.empty) return GEMM_OK;
    (void)hipGetLastError();
    hipError_t e = hipErrorInvalidValue;
    if (variant == CONV_C0_DIRECT) {
        switch (p.c.in_dtype) {
        case GEMM_F32: e = launch_direct<F32>(p); break;
        case GEMM_BF16: e = launch_direct<BF16>(p); break;
        case GEMM_F16: e = launch_direct<F16>(p); break;
        default: e = launch_direct<E4M3>(p); break;
        }
    } else if (variant == CONV_C1_IM2COL_MFMA) {
        switch (p.c.in_dtype) {
        case GEMM_BF16: e = launch_im2col<BF16>(p); break;
        case GEMM_F16: e = launch_im2col<F16>(p); break;
        default: e = launch_im2col<E4M3>(p); break;
        }
    } else {
        e = launch_k4_conv(p.g);
    }
    if (e != hipSuccess) last_conv_launch_error = e;
    return e == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

const char* conv2d_last_launch_error(void) { return hipGetErrorString(last_conv_launch_error); }

const char* conv2d_variant_name(int v)
{
    static const char* names[] = {"C0_direct", "C1_im2col_mfma", "C2_implicit_mfma"};
    return (v >= 0 && v < CONV_VARIANT_COUNT) ? names[v] : "?";
}

const char* conv2d_variant_intent(int v)
{
    static const char* intents[] = {"(start of lineage)", "im2col + the matrix product's expert state", "gather fused into the direct-to-LDS loads"};
    return (v >= 0 && v < CONV_VARIANT_COUNT) ? intents[v] : "?";
}

const char* conv2d_cond_name(uint32_t bit)
{
    switch (bit) {
    case CONV_COND_ALIGN16_X: return "ALIGN16_X";
    case CONV_COND_ALIGN16_W: return "ALIGN16_W";
    case CONV_COND_ALIGN16_Y: return "ALIGN16_Y";
    case CONV_COND_C_WHOLE_SLABS: return "C_WHOLE_SLABS";
    case CONV_COND_DTYPE_ON_FAST_KERNEL: return "DTYPE_ON_FAST_KERNEL";
    case CONV_COND_X_BELOW_2GIB: return "X_BELOW_2GIB";
    case CONV_COND_SCRATCH_LENT: return "SCRATCH_LENT";
    default: return "?";
    }
}

int conv2d_variant_count(void) { return CONV_VARIANT_COUNT; }

}  // extern "C"
