"""Thin ctypes binding of ``include/conv_lineage.h`` (argument marshalling only).

Same rules as ``gemm.py``: every function has the name and meaning of the C entry point it calls, all
arithmetic runs in the HIP kernels of ``libgemm_lineage.so``, and there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Any, List

from . import gemm
from .gemm import _addr, _stream_addr

CONV_C0_DIRECT, CONV_C1_IM2COL_MFMA, CONV_C2_IMPLICIT_MFMA = 0, 1, 2
CONV_VARIANT_COUNT = 3
COND_BITS = {name: 1 << i for i, name in enumerate(
    ["ALIGN16_X", "ALIGN16_W", "ALIGN16_Y", "C_WHOLE_SLABS", "DTYPE_ON_FAST_KERNEL", "X_BELOW_2GIB", "SCRATCH_LENT"])}


class conv2d_desc_t(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64), ("C", ctypes.c_int64),
                ("F", ctypes.c_int64), ("R", ctypes.c_int64), ("S", ctypes.c_int64),
                ("stride_h", ctypes.c_int32), ("stride_w", ctypes.c_int32),
                ("pad_h", ctypes.c_int32), ("pad_w", ctypes.c_int32),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("bias", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p), ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class conv2d_query_t(ctypes.Structure):
    _fields_ = [("required", ctypes.c_uint32), ("violated", ctypes.c_uint32), ("holds", ctypes.c_uint32),
                ("P", ctypes.c_int64), ("Q", ctypes.c_int64),
                ("gemm_m", ctypes.c_int64), ("gemm_n", ctypes.c_int64), ("gemm_k", ctypes.c_int64),
                ("bm", ctypes.c_int32), ("bn", ctypes.c_int32), ("bk", ctypes.c_int32),
                ("threads", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
                ("grid", ctypes.c_int64), ("workspace_bytes", ctypes.c_size_t), ("path", ctypes.c_char * 64)]


_bound = False


def lib() -> ctypes.CDLL:
    global _bound
    L = gemm.lib()
    if not _bound:
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.conv2d_run.restype = ci
        L.conv2d_run.argtypes = [ci, ctypes.POINTER(conv2d_desc_t), vp, vp, vp]
        L.conv2d_query.restype = ci
        L.conv2d_query.argtypes = [ci, ctypes.POINTER(conv2d_desc_t), vp, vp, vp, ctypes.POINTER(conv2d_query_t)]
        L.conv2d_default_desc.restype = ci
        L.conv2d_default_desc.argtypes = [ctypes.POINTER(conv2d_desc_t)] + [i64] * 7 + [ci]
        for name in ("conv2d_variant_name", "conv2d_variant_intent"):
            getattr(L, name).restype = ctypes.c_char_p
            getattr(L, name).argtypes = [ci]
        L.conv2d_cond_name.restype = ctypes.c_char_p
        L.conv2d_cond_name.argtypes = [ctypes.c_uint32]
        L.conv2d_last_launch_error.restype = ctypes.c_char_p
        L.conv2d_last_launch_error.argtypes = []
        L.conv2d_variant_count.restype = ci
        _bound = True
    return L


def conv2d_default_desc(N: int, H: int, W: int, C: int, F: int, R: int, S: int, dtype: int) -> conv2d_desc_t:
    d = conv2d_desc_t()
    rc = lib().conv2d_default_desc(ctypes.byref(d), N, H, W, C, F, R, S, dtype)
    if rc != gemm.GEMM_OK:
        raise ValueError(gemm.gemm_status_string(rc))
    return d


def make_desc(N: int, H: int, W: int, C: int, F: int, R: int, S: int, in_dtype: int, out_dtype: int, *,
              stride=(1, 1), pad=(0, 0), bias: Any = None, workspace: Any = None, workspace_bytes: int = 0,
              stream: Any = None, flags: int = 0) -> conv2d_desc_t:
    d = conv2d_desc_t()
    d.N, d.H, d.W, d.C, d.F, d.R, d.S = N, H, W, C, F, R, S
    d.stride_h, d.stride_w = stride
    d.pad_h, d.pad_w = pad
    d.in_dtype, d.out_dtype = in_dtype, out_dtype
    d.bias, d.workspace, d.workspace_bytes = _addr(bias), _addr(workspace), workspace_bytes
    d.stream = _stream_addr(stream)
    d.flags, d.reserved = flags, 0
    return d


def conv2d_run(variant: int, d: conv2d_desc_t, x: Any, w: Any, y: Any) -> int:
    return int(lib().conv2d_run(variant, ctypes.byref(d), _addr(x), _addr(w), _addr(y)))


@dataclass
class Query:
    status: int
    required: int
    violated: int
    holds: int
    P: int
    Q: int
    gemm_m: int
    gemm_n: int
    gemm_k: int
    bm: int
    bn: int
    bk: int
    threads: int
    lds_bytes: int
    grid: int
    workspace_bytes: int
    path: str

    @staticmethod
    def names(mask: int) -> List[str]:
        return [n for n, b in COND_BITS.items() if mask & b]


def conv2d_query(variant: int, d: conv2d_desc_t, x: Any = None, w: Any = None, y: Any = None) -> Query:
    q = conv2d_query_t()
    rc = int(lib().conv2d_query(variant, ctypes.byref(d), _addr(x), _addr(w), _addr(y), ctypes.byref(q)))
    return Query(rc, q.required, q.violated, q.holds, q.P, q.Q, q.gemm_m, q.gemm_n, q.gemm_k, q.bm, q.bn, q.bk,
                 q.threads, q.lds_bytes, q.grid, q.workspace_bytes, q.path.decode())


def conv2d_variant_name(variant: int) -> str:
    return lib().conv2d_variant_name(variant).decode()


def conv2d_variant_intent(variant: int) -> str:
    return lib().conv2d_variant_intent(variant).decode()


def conv2d_cond_name(bit: int) -> str:
    return lib().conv2d_cond_name(bit).decode()


def conv2d_variant_count() -> int:
    return int(lib().conv2d_variant_count())


def conv2d_last_launch_error() -> str:
    return lib().conv2d_last_launch_error().decode()
