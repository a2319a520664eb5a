// Shared device/host declarations for the GEMM lineage kernels (gfx950 only).
//
// Every lineage state computes the same thing (paper Sec. 3.1: a lineage is a sequence of
// validated states of ONE kernel): C[b,i,j] = round_out(s_b * sum_k dec(A[b,i,k]) dec(B[b,k,j]))
// with fp32 accumulation, s_b = scale_a[b]*scale_b[b].  This header holds the pieces all states
// share: the launch argument block, exact decoders of the four storage formats, and the
// round-to-nearest-even output conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm_lineage.h"

namespace gl {

// Geometry of a convolution layer lowered to a matrix product (rows = output pixels n,p,q; columns =
// filters; K = taps x channels in the order r, s, c).  Only K4's gathering instantiation reads it.
struct ConvGeom {
    int32_t H, W, C;              // input height, width, channels
    int32_t P, Q;                 // output height, width
    int32_t S;                    // filter width (taps per filter row)
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t slabs_per_tap;        // C * element size / 128
    uint32_t x_bytes;             // extent of the activations: the gather's buffer resource ends here
};

// Launch arguments, passed to kernels by value.  Strides are in elements.
struct Args {
    const void* A;
    const void* B;
    void* C;
    const float* scale_a;
    const float* scale_b;
    const float* bias;
    void* workspace;
    int64_t M, N, K, batch;
    int64_t a_si, a_sk;  // A(i,k) at i*a_si + k*a_sk
    int64_t b_sk, b_sj;  // B(k,j) at k*b_sk + j*b_sj
    int64_t ldc;
    int64_t stride_a, stride_b, stride_c;
    int32_t in_dtype, out_dtype;
    uint32_t flags;      // GEMM_FLAG_DEOPT_* bits (host side only: they select an instantiation); ARGS_C_TRANSPOSED
    hipStream_t stream;
    ConvGeom conv;       // all zero for a plain matrix product
};

// Set by the launcher of the streaming kernel when it multiplies the transposed product (few columns instead
// of few rows): the kernel's (row, column) is C's (column, row), and the bias belongs to the kernel's rows.
constexpr uint32_t ARGS_C_TRANSPOSED = 1u << 31;

// ---- storage formats ------------------------------------------------------------------------
struct F32 { using raw = float;    static constexpr int BYTES = 4; static constexpr int ID = GEMM_F32; };
struct BF16 { using raw = uint16_t; static constexpr int BYTES = 2; static constexpr int ID = GEMM_BF16; };
struct F16 { using raw = uint16_t; static constexpr int BYTES = 2; static constexpr int ID = GEMM_F16; };
struct E4M3 { using raw = uint8_t;  static constexpr int BYTES = 1; static constexpr int ID = GEMM_FP8_E4M3; };

template <typename T> __device__ __forceinline__ float decode(typename T::raw v);

template <> __device__ __forceinline__ float decode<F32>(float v) { return v; }
template <> __device__ __forceinline__ float decode<BF16>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
template <> __device__ __forceinline__ float decode<F16>(uint16_t v) { return (float)__builtin_bit_cast(_Float16, v); }
// OCP E4M3: bias 7; e==0 is subnormal (m * 2^-9); S.1111.111 is NaN; no infinities.
template <> __device__ __forceinline__ float decode<E4M3>(uint8_t v)
{
    const uint32_t s = (uint32_t)(v & 0x80u) << 24, e = (v >> 3) & 0xFu, m = v & 0x7u;
    if ((v & 0x7Fu) == 0x7Fu) return __uint_as_float(s | 0x7FC00000u);
    if (e == 0) return __uint_as_float(s | __float_as_uint((float)m * 0x1p-9f));
    return __uint_as_float(s | ((e + 120u) << 23) | (m << 20));
}

// fp32 -> bf16 bits, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint16_t encode_bf16(float x)
{
    uint32_t b = __float_as_uint(x);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}
__device__ __forceinline__ uint16_t encode_f16(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }

// Epilogue store of one element; out_dtype is uniform across the launch.
__device__ __forceinline__ void store_out(void* C, int64_t idx, float v, int out_dtype)
{
    if (out_dtype == GEMM_F32) ((float*)C)[idx] = v;
    else if (out_dtype == GEMM_BF16) ((uint16_t*)C)[idx] = encode_bf16(v);
    else ((uint16_t*)C)[idx] = encode_f16(v);
}

__device__ __forceinline__ float batch_scale(const Args& a, int64_t b)
{
    float s = 1.0f;
    if (a.scale_a) s *= a.scale_a[b];
    if (a.scale_b) s *= a.scale_b[b];
    return s;
}

// ---- host-side helpers shared by the entry points -------------------------------------------------
inline int elem_size(int dt) { return dt == GEMM_F32 ? 4 : dt == GEMM_FP8_E4M3 ? 1 : 2; }

// input / output type pairs the library implements (accumulation is always fp32)
inline bool dtype_pair_supported(int in, int out)
{
    switch (in) {
    case GEMM_F32: return out == GEMM_F32;
    case GEMM_BF16: return out == GEMM_BF16 || out == GEMM_F32;
    case GEMM_F16: return out == GEMM_F16 || out == GEMM_F32;
    case GEMM_FP8_E4M3: return out == GEMM_BF16 || out == GEMM_F32;
    default: return false;
    }
}

// ---- host-side launchers, one per translation unit ---------------------------------------------
// Each returns hipSuccess or the launch error.  `path` selects a code path that the caller
// (gemm_api.hip) has already proven legal for these arguments.
enum ValuPath { VALU_SCALAR = 0, VALU_VEC16 = 1, VALU_ASYNC = 4 };    // (K2/K3 paths 0..3: bitmask of operands loaded 16 bytes at a time)
enum MfmaPath { MFMA_ELEMENTWISE = 0, MFMA_VEC16 = 1, MFMA_SKINNY = 2, MFMA_PACKED = 3, MFMA_SPLITK = 4, MFMA_SKINNY_N = 5, MFMA_VEC16_BROW = 6, MFMA_THIN_BROW = 7 };

// Workspace of the packed K4 path: both operands rewritten as [rows][Kp], Kp = K rounded up to a slab.
int64_t k4_packed_k(const Args& a);
size_t k4_packed_workspace_bytes(const Args& a, int keep_mask);   // keep_mask: bit 0 / 1 = A / B is used in place
// Split-K form of the fast kernel: how many K ranges a product with too few tiles to fill the chip
// is cut into (1: not applicable), and the fp32 scratch the partial products need.
int k4_splitk_factor(const Args& a);
size_t k4_splitk_workspace_bytes(const Args& a, int splits);
// True when the fast kernel's launcher hands a thin remainder of rows (M % 256 in 1..64, where that saves a
// round of the chip) to the streaming kernel.
bool k4_splits_m_tail(const Args& a);
bool k4_streams_rows(const Args& a);      // a product of at most 64 rows goes to the streaming kernel
// With a streaming-form override in the flags: whether that form holds the product's rows.
bool k4_stream_form_fits(const Args& a);
Args k4_transposed(const Args& a);        // the same product as C^T = B^T A^T (operands swapped, ARGS_C_TRANSPOSED set)
// True when the fast kernel runs with 128 x 128 workgroup tiles instead of 256 x 256.
bool k4_small_tiles(const Args& a);
// True when the fast path runs as the persistent kernel (256 workgroups walking several 256 x 256 tiles each).
bool k4_uses_ring(const Args& a);
// Whether the tiled part of a product on path `kind` (MFMA_VEC16, MFMA_PACKED, MFMA_SPLITK) runs as the persistent kernel.
bool k4_fast_is_persistent(int kind, const Args& a);
// Switches that change which kernel form multiplies the tiles but not how the product is cut up (row remainder, K ranges).
constexpr uint32_t K4_NEUTRAL_FLAGS = GEMM_FLAG_DEOPT_NO_PERSISTENT | GEMM_FLAG_MFMA_32X32;
constexpr int K4_RING_WORKGROUPS = 256;   // one per CU of the GPU this library is written for (8 XCDs x 32)
hipError_t launch_k4_ring(const Args& a);  // bf16, fp16, e4m3; k4_uses_ring(a) must hold
// The persistent kernel on a row-major B read in place (bf16, fp16), and whether a product qualifies for it.
bool k4_ring_takes_row_major_b(const Args& a);
hipError_t launch_k4_ring_row_major_b(const Args& a);
// Thin products (at most 64 rows) with A and B row-major, two-byte types: B is read once, in place.  The row-major-B
// form above hands this kernel a remainder of rows that would cost it a round of tiles (the rule says when).
bool k4_brow_splits_m_tail(const Args& a);
bool k4_thin_takes_row_major_b(const Args& a);      // a whole product for the thin kernel
bool k4_brow_splits_last_col(const Args& a);        // ... and C's last column to the masked kernel (element after B not known to be mapped)
bool k4_brow_splits_last_row(const Args& a);
int k4_brow_splits(const Args& a);                  // bit 0: last column split off, bit 1: last row, bit 2: thin remainder of rows        // the persistent row-major-B form leaves A's last row to the thin kernel (element after A not known to be mapped)
int k4_thin_cols(const Args& a);                    // columns per strip (= per workgroup) it is launched with: 64 or 32
// Both row-major-B kernels load rows as dwords from their first element, so the dword that holds the last element
// of an odd-length last row reaches one element past the operand.  With the pointer known, such a product is only
// taken when that element lies in the same 4 KiB page as the operand's last byte (mapped whatever follows).
inline bool tail_element_in_last_page(const void* base, int64_t elems, int64_t last_row_len, int es)
{
    if (!base || last_row_len % 2 == 0) return true;          // (a query without pointers; no dword straddles the end)
    const uintptr_t end = (uintptr_t)base + (uintptr_t)(elems * es);     // first byte past the operand
    return (end & 4095u) != 0;
}
hipError_t launch_k4_thin_row_major_b(const Args& a);

hipError_t launch_k0(const Args& a);
hipError_t launch_valu_tiled(int variant, int path, const Args& a);
// K3's asynchronous form (direct-to-LDS loads, three stages, operands kept in storage format in LDS): whether a
// product whose operands both take 16-byte loads qualifies, its launcher and geometry.
bool k3_async_applies(const Args& a);
hipError_t launch_k3_async(const Args& a);
hipError_t launch_k4(int path, const Args& a);
// K4's fast kernel with A gathered from the activations of a convolution layer (a.conv); a.A = x,
// a.B = filters (F rows of K contiguous elements), 2-byte or 1-byte types, whole slabs per tap.
hipError_t launch_k4_conv(const Args& a);

// Geometry reported by gemm_query (kept next to the kernels that define it).
struct Geometry { int bm, bn, bk, threads, stages, lds_bytes; int64_t grid; };
Geometry geometry_k0(const Args& a);
Geometry geometry_valu_tiled(int variant, int path, const Args& a);
Geometry geometry_k3_async(const Args& a);
Geometry geometry_k4(int path, const Args& a);
Geometry geometry_k4_conv(const Args& a);

}  // namespace gl
