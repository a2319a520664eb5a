"""Thin ctypes binding of ``include/gemm_lineage.h`` (argument marshalling only).

Every function has the name and meaning of the C entry point it calls; all arithmetic runs in
the HIP kernels of ``libgemm_lineage.so``.  There is no CPU fallback: if the shared library is
missing or fails to load, every call raises.  Device buffers may be passed as ``torch`` tensors
(their ``data_ptr()`` is used), as objects exposing ``data_ptr()``, or as integer addresses.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Any, List, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgemm_lineage.so")

# enums of gemm_lineage.h
GEMM_OK, GEMM_ERR_BAD_ARG, GEMM_ERR_BAD_VARIANT, GEMM_ERR_UNSUPPORTED_DTYPE = 0, 1, 2, 3
GEMM_ERR_PRECONDITION, GEMM_ERR_WORKSPACE, GEMM_ERR_LAUNCH = 4, 5, 6
GEMM_F32, GEMM_BF16, GEMM_F16, GEMM_FP8_E4M3 = 0, 1, 2, 3
GEMM_ROW_MAJOR, GEMM_COL_MAJOR = 0, 1
GEMM_K0_NAIVE, GEMM_K1_LDS_TILED, GEMM_K2_VECTORIZED, GEMM_K3_PIPELINED, GEMM_K4_MFMA = 0, 1, 2, 3, 4
GEMM_VARIANT_COUNT = 5
GEMM_FLAG_STRICT = 1
GEMM_FLAG_DEOPT_NO_SWIZZLE, GEMM_FLAG_DEOPT_NO_OVERLAP = 2, 4
GEMM_FLAG_TILE_256, GEMM_FLAG_TILE_128 = 8, 16
GEMM_FLAG_DEOPT_NO_RASTER, GEMM_FLAG_DEOPT_NO_VECTOR = 32, 64
GEMM_FLAG_DEOPT_NO_PERSISTENT = 128
GEMM_FLAG_MFMA_32X32 = 1 << 11
GEMM_FLAG_STREAM_FORM_SHIFT, GEMM_FLAG_STREAM_FORM_MASK = 8, 7 << 8


def GEMM_FLAG_STREAM_FORM(form: int) -> int:
    return (form + 1) << GEMM_FLAG_STREAM_FORM_SHIFT
COND_BITS = {name: 1 << i for i, name in enumerate(
    ["ALIGN16_A", "ALIGN16_B", "ALIGN16_C", "LD16_A", "LD16_B", "LD16_C", "TILE_DIV_M", "TILE_DIV_N",
     "TILE_DIV_K", "K_CONTIG_A", "K_CONTIG_B", "DTYPE_HAS_MFMA", "LDS_STAGED", "SMALL_M"])}


class gemm_desc_t(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("batch", ctypes.c_int64),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("layout_a", ctypes.c_int32), ("layout_b", ctypes.c_int32),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("ldc", ctypes.c_int64),
                ("stride_a", ctypes.c_int64), ("stride_b", ctypes.c_int64), ("stride_c", ctypes.c_int64),
                ("scale_a", ctypes.c_void_p), ("scale_b", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p), ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class gemm_query_t(ctypes.Structure):
    _fields_ = [("required", ctypes.c_uint32), ("violated", ctypes.c_uint32), ("holds", ctypes.c_uint32),
                ("bm", ctypes.c_int32), ("bn", ctypes.c_int32), ("bk", ctypes.c_int32),
                ("threads", ctypes.c_int32), ("stages", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
                ("grid", ctypes.c_int64), ("workspace_bytes", ctypes.c_size_t), ("path", ctypes.c_char * 64)]


class GemmLibraryMissing(RuntimeError):
    pass


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises GemmLibraryMissing when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise GemmLibraryMissing(
                f"{LIB_PATH} not found: build it with `python -m paper_2605_28213_amd.build` "
                "(there is no CPU fallback for the GEMM lineage)")
        # PyTorch ships its own copy of the HIP runtime.  If this library were loaded first it would
        # pull in the system's copy, PyTorch would then load its own, and the second runtime in a
        # process cannot open the GPU ("no ROCm-capable device is detected" on the first launch).
        # Importing torch first makes its runtime the one both sides use.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.gemm_run.restype = ci
        L.gemm_run.argtypes = [ci, i64, i64, i64, ci, vp, vp, vp]
        L.gemm_run_ex.restype = ci
        L.gemm_run_ex.argtypes = [ci, ctypes.POINTER(gemm_desc_t), vp, vp, vp]
        L.gemm_run_static.restype = ci
        L.gemm_run_static.argtypes = [ci, ctypes.POINTER(gemm_desc_t), vp, vp, vp]
        L.gemm_static_scratch_bytes.restype = ctypes.c_size_t
        L.gemm_static_scratch_bytes.argtypes = []
        L.gemm_query.restype = ci
        L.gemm_query.argtypes = [ci, ctypes.POINTER(gemm_desc_t), vp, vp, vp, ctypes.POINTER(gemm_query_t)]
        L.gemm_default_desc.restype = ci
        L.gemm_default_desc.argtypes = [ctypes.POINTER(gemm_desc_t), i64, i64, i64, ci]
        for name in ("gemm_status_string", "gemm_variant_name", "gemm_variant_intent"):
            getattr(L, name).restype = ctypes.c_char_p
            getattr(L, name).argtypes = [ci]
        L.gemm_last_launch_error.restype = ctypes.c_char_p
        L.gemm_last_launch_error.argtypes = []
        L.gemm_cond_name.restype = ctypes.c_char_p
        L.gemm_cond_name.argtypes = [ctypes.c_uint32]
        L.gemm_variant_count.restype = ci
        L.gemm_abi_version.restype = ci
        st = ctypes.c_size_t
        L.gemm_probe_copy.restype = ci
        L.gemm_probe_copy.argtypes = [vp, vp, st, vp]
        L.gemm_probe_stream_read.restype = ci
        L.gemm_probe_stream_read.argtypes = [vp, st, vp, vp]
        L.gemm_probe_mfma_operand_bytes.restype = st
        L.gemm_probe_mfma_operand_bytes.argtypes = [ci, ci]
        L.gemm_probe_mfma.restype = ci
        L.gemm_probe_mfma.argtypes = [ci, vp, st, ci, ci, vp, st, ctypes.POINTER(ctypes.c_double), vp]
        L.gemm_probe_mfma16.restype = ci
        L.gemm_probe_mfma16.argtypes = [ci, vp, st, ci, ci, vp, st, ctypes.POINTER(ctypes.c_double), vp]
        _lib = L
    return _lib


def _addr(x: Any) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    raise TypeError(f"cannot take a device address from {type(x).__name__}")


def gemm_default_desc(M: int, N: int, K: int, dtype: int) -> gemm_desc_t:
    d = gemm_desc_t()
    rc = lib().gemm_default_desc(ctypes.byref(d), M, N, K, dtype)
    if rc != GEMM_OK:
        raise ValueError(gemm_status_string(rc))
    return d


def make_desc(M: int, N: int, K: int, in_dtype: int, out_dtype: int, layout_a: int, layout_b: int, *,
              lda: int = 0, ldb: int = 0, ldc: int = 0, batch: int = 1, stride_a: int = -1, stride_b: int = -1,
              stride_c: int = -1, scale_a: Any = None, scale_b: Any = None, bias: Any = None, stream: Any = None,
              workspace: Any = None, workspace_bytes: int = 0, flags: int = 0) -> gemm_desc_t:
    """Fill a descriptor; tight leading dimensions and batch strides unless given."""
    d = gemm_desc_t()
    d.M, d.N, d.K, d.batch = M, N, K, batch
    d.in_dtype, d.out_dtype, d.layout_a, d.layout_b = in_dtype, out_dtype, layout_a, layout_b
    d.lda = lda or max(1, K if layout_a == GEMM_ROW_MAJOR else M)
    d.ldb = ldb or max(1, N if layout_b == GEMM_ROW_MAJOR else K)
    d.ldc = ldc or max(1, N)
    d.stride_a = stride_a if stride_a >= 0 else (M if layout_a == GEMM_ROW_MAJOR else K) * d.lda
    d.stride_b = stride_b if stride_b >= 0 else (K if layout_b == GEMM_ROW_MAJOR else N) * d.ldb
    d.stride_c = stride_c if stride_c >= 0 else M * d.ldc
    d.scale_a, d.scale_b, d.bias = _addr(scale_a), _addr(scale_b), _addr(bias)
    d.workspace, d.workspace_bytes = _addr(workspace), workspace_bytes
    d.stream = _addr(stream) if not hasattr(stream, "cuda_stream") else int(stream.cuda_stream)
    d.flags, d.reserved = flags, 0
    return d


def gemm_run(variant: int, M: int, N: int, K: int, dtype: int, A: Any, B: Any, C: Any) -> int:
    return int(lib().gemm_run(variant, M, N, K, dtype, _addr(A), _addr(B), _addr(C)))


def gemm_run_ex(variant: int, d: gemm_desc_t, A: Any, B: Any, C: Any) -> int:
    return int(lib().gemm_run_ex(variant, ctypes.byref(d), _addr(A), _addr(B), _addr(C)))


def gemm_run_static(variant: int, d: gemm_desc_t, A: Any, B: Any, C: Any) -> int:
    return int(lib().gemm_run_static(variant, ctypes.byref(d), _addr(A), _addr(B), _addr(C)))


def gemm_static_scratch_bytes() -> int:
    return int(lib().gemm_static_scratch_bytes())


@dataclass
class Query:
    status: int
    required: int
    violated: int
    holds: int
    bm: int
    bn: int
    bk: int
    threads: int
    stages: int
    lds_bytes: int
    grid: int
    workspace_bytes: int
    path: str

    @staticmethod
    def names(mask: int) -> List[str]:
        return [n for n, b in COND_BITS.items() if mask & b]


def gemm_query(variant: int, d: gemm_desc_t, A: Any = None, B: Any = None, C: Any = None) -> Query:
    q = gemm_query_t()
    rc = int(lib().gemm_query(variant, ctypes.byref(d), _addr(A), _addr(B), _addr(C), ctypes.byref(q)))
    return Query(rc, q.required, q.violated, q.holds, q.bm, q.bn, q.bk, q.threads, q.stages, q.lds_bytes,
                 q.grid, q.workspace_bytes, q.path.decode())


def gemm_status_string(status: int) -> str:
    return lib().gemm_status_string(status).decode()


def gemm_variant_name(variant: int) -> str:
    return lib().gemm_variant_name(variant).decode()


def gemm_variant_intent(variant: int) -> str:
    return lib().gemm_variant_intent(variant).decode()


def gemm_cond_name(bit: int) -> str:
    return lib().gemm_cond_name(bit).decode()


def gemm_variant_count() -> int:
    return int(lib().gemm_variant_count())


def gemm_abi_version() -> int:
    return int(lib().gemm_abi_version())


def _stream_addr(stream: Any) -> Optional[int]:
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else _addr(stream)


def gemm_probe_copy(dst: Any, src: Any, nbytes: int, stream: Any = None) -> int:
    return int(lib().gemm_probe_copy(_addr(dst), _addr(src), nbytes, _stream_addr(stream)))


def gemm_probe_stream_read(src: Any, nbytes: int, sink: Any, stream: Any = None) -> int:
    return int(lib().gemm_probe_stream_read(_addr(src), nbytes, _addr(sink), _stream_addr(stream)))


def gemm_probe_mfma_operand_bytes(dtype: int, workgroups: int) -> int:
    return int(lib().gemm_probe_mfma_operand_bytes(dtype, workgroups))


def gemm_probe_mfma(dtype: int, operands: Any, operand_bytes: int, workgroups: int, iters: int, sink: Any,
                    sink_bytes: int, stream: Any = None):
    """Returns (status, flops of the launch)."""
    fl = ctypes.c_double(0.0)
    rc = int(lib().gemm_probe_mfma(dtype, _addr(operands), operand_bytes, workgroups, iters, _addr(sink), sink_bytes,
                                   ctypes.byref(fl), _stream_addr(stream)))
    return rc, fl.value


def gemm_probe_mfma16(dtype: int, operands: Any, operand_bytes: int, workgroups: int, iters: int, sink: Any,
                      sink_bytes: int, stream: Any = None):
    """Returns (status, flops of the launch)."""
    fl = ctypes.c_double(0.0)
    rc = int(lib().gemm_probe_mfma16(dtype, _addr(operands), operand_bytes, workgroups, iters, _addr(sink), sink_bytes,
                                     ctypes.byref(fl), _stream_addr(stream)))
    return rc, fl.value


def gemm_last_launch_error() -> str:
    return lib().gemm_last_launch_error().decode()
