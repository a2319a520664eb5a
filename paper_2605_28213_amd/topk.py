"""Thin ctypes binding of ``include/topk_lineage.h`` (argument marshalling only; no CPU fallback)."""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Any, List

from . import gemm
from .gemm import _addr, _stream_addr

TOPK_T0_SELECTION, TOPK_T1_RADIX_SELECT, TOPK_T2_RESIDENT = 0, 1, 2
TOPK_VARIANT_COUNT = 3
COND_BITS = {name: 1 << i for i, name in enumerate(["ROW_IN_LDS", "ROW_IN_REGISTERS", "ALIGN16"])}


class topk_desc_t(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64), ("ld", ctypes.c_int64),
                ("stream", ctypes.c_void_p), ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class topk_query_t(ctypes.Structure):
    _fields_ = [("required", ctypes.c_uint32), ("violated", ctypes.c_uint32), ("holds", ctypes.c_uint32),
                ("threads", ctypes.c_int32), ("passes", ctypes.c_int32), ("lds_bytes", ctypes.c_int32),
                ("grid", ctypes.c_int64), ("path", ctypes.c_char * 64)]


_bound = False


def lib() -> ctypes.CDLL:
    global _bound
    L = gemm.lib()
    if not _bound:
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.topk_run.restype = ci
        L.topk_run.argtypes = [ci, ctypes.POINTER(topk_desc_t), vp, vp, vp]
        L.topk_query.restype = ci
        L.topk_query.argtypes = [ci, ctypes.POINTER(topk_desc_t), vp, ctypes.POINTER(topk_query_t)]
        for name in ("topk_variant_name", "topk_variant_intent"):
            getattr(L, name).restype = ctypes.c_char_p
            getattr(L, name).argtypes = [ci]
        L.topk_cond_name.restype = ctypes.c_char_p
        L.topk_cond_name.argtypes = [ctypes.c_uint32]
        L.topk_last_launch_error.restype = ctypes.c_char_p
        L.topk_last_launch_error.argtypes = []
        L.topk_variant_count.restype = ci
        _bound = True
    return L


def make_desc(batch: int, n: int, k: int, *, ld: int = 0, stream: Any = None, flags: int = 0) -> topk_desc_t:
    d = topk_desc_t()
    d.batch, d.n, d.k, d.ld = batch, n, k, ld or n
    d.stream = _stream_addr(stream)
    d.flags, d.reserved = flags, 0
    return d


def topk_run(variant: int, d: topk_desc_t, x: Any, idx: Any, val: Any) -> int:
    return int(lib().topk_run(variant, ctypes.byref(d), _addr(x), _addr(idx), _addr(val)))


@dataclass
class Query:
    status: int
    required: int
    violated: int
    holds: int
    threads: int
    passes: int
    lds_bytes: int
    grid: int
    path: str

    @staticmethod
    def names(mask: int) -> List[str]:
        return [n for n, b in COND_BITS.items() if mask & b]


def topk_query(variant: int, d: topk_desc_t, x: Any = None) -> Query:
    q = topk_query_t()
    rc = int(lib().topk_query(variant, ctypes.byref(d), _addr(x), ctypes.byref(q)))
    return Query(rc, q.required, q.violated, q.holds, q.threads, q.passes, q.lds_bytes, q.grid, q.path.decode())


def topk_variant_name(variant: int) -> str:
    return lib().topk_variant_name(variant).decode()


def topk_variant_intent(variant: int) -> str:
    return lib().topk_variant_intent(variant).decode()


def topk_cond_name(bit: int) -> str:
    return lib().topk_cond_name(bit).decode()


def topk_variant_count() -> int:
    return int(lib().topk_variant_count())


def topk_last_launch_error() -> str:
    return lib().topk_last_launch_error().decode()
