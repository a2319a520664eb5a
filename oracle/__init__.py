"""CPU oracle for the GEMM lineage and its convolution transfer -- TEST INFRASTRUCTURE ONLY.

ctypes wrapper around ``gemm_oracle.c``, ``conv_oracle.c`` (plain C, fp64 accumulation) and
``topk_oracle.c`` (rank counting).  Only the
test-suite, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library never does, and this package never imports the GPU
library.  See the headers of the two C files for the definitions they implement
and for the lists of pins that hold them in place.

Arrays are numpy; integer-coded dtypes are passed as their raw bit patterns
(``uint16`` for bf16/fp16, ``uint8`` for e4m3, ``float32`` for fp32).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

F32, BF16, F16, E4M3 = 0, 1, 2, 3
ROW_MAJOR, COL_MAJOR = 0, 1

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "gemm_oracle.c")
_SRC_CONV = os.path.join(_DIR, "conv_oracle.c")
_SRC_TOPK = os.path.join(_DIR, "topk_oracle.c")
_LIB = os.path.join(_DIR, "libgemm_oracle.so")

_NP_STORAGE = {F32: np.float32, BF16: np.uint16, F16: np.uint16, E4M3: np.uint8}

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: fp64 semantics are the point)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_CONV), os.path.getmtime(_SRC_TOPK))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
               "-ffp-contract=off", "-o", _LIB, _SRC, _SRC_CONV, _SRC_TOPK, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _bind(path: str):
    """Open an oracle shared object and declare its prototypes."""
    lib = ctypes.CDLL(path)
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    lib.oracle_decode.restype = ctypes.c_double
    lib.oracle_decode.argtypes = [ctypes.c_int, ctypes.c_uint32]
    lib.oracle_gemm.restype = ctypes.c_int
    lib.oracle_gemm.argtypes = ([ctypes.c_int] * 3 + [i64] * 4 + [vp, i64, i64, vp, i64, i64]
                                + [vp, vp, vp, vp, i64, i64])
    lib.oracle_gemm_points.restype = ctypes.c_int
    lib.oracle_gemm_points.argtypes = ([ctypes.c_int] * 3 + [i64] * 4 + [vp, i64, i64, vp, i64, i64]
                                       + [vp, vp, i64, vp, vp, vp, vp, vp])
    lib.oracle_num_threads.restype = ctypes.c_int
    if hasattr(lib, "oracle_conv2d"):                   # absent from a library built from gemm_oracle.c alone
        lib.oracle_conv2d_output_size.restype = None
        lib.oracle_conv2d_output_size.argtypes = [i64] * 8 + [vp, vp]
        lib.oracle_conv2d.restype = ctypes.c_int
        lib.oracle_conv2d.argtypes = [ctypes.c_int] + [i64] * 11 + [vp, vp, vp, vp]
        lib.oracle_conv2d_points.restype = ctypes.c_int
        lib.oracle_conv2d_points.argtypes = [ctypes.c_int] + [i64] * 11 + [vp, vp, i64, vp, vp, vp, vp, vp, vp]
    if hasattr(lib, "oracle_topk"):
        lib.oracle_topk.restype = ctypes.c_int
        lib.oracle_topk.argtypes = [i64, i64, i64, vp, i64, vp, vp]
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(_LIB)
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def decode(dtype: int, codes: np.ndarray) -> np.ndarray:
    """Decode an array of stored bit patterns to fp64 values, one C call per element
    for small arrays and a table lookup (built from those C calls) otherwise."""
    lib = _load()
    codes = np.asarray(codes)
    if dtype == F32:
        bits = codes.astype(np.float32).view(np.uint32) if codes.dtype.kind == "f" else codes.astype(np.uint32)
        flat = bits.ravel()
        if flat.size > 4096:
            # fp32 -> fp64 widening is exact; spot-checked against oracle_decode in the pins
            return flat.view(np.float32).astype(np.float64).reshape(codes.shape)
        return np.array([lib.oracle_decode(F32, int(c)) for c in flat], dtype=np.float64).reshape(codes.shape)
    nbits = 16 if dtype in (BF16, F16) else 8
    table = np.array([lib.oracle_decode(dtype, c) for c in range(1 << nbits)], dtype=np.float64)
    return table[codes.astype(np.int64)]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_storage(dtype: int, a: np.ndarray, name: str) -> np.ndarray:
    want = _NP_STORAGE[dtype]
    if a.dtype != want:
        raise TypeError(f"{name}: dtype code {dtype} is stored as {want}, got {a.dtype}")
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError(f"{name} must be a contiguous buffer (layout is described by ld/stride)")
    return a


def gemm(dtype: int, layout_a: int, layout_b: int, M: int, N: int, K: int,
         A: np.ndarray, lda: int, B: np.ndarray, ldb: int, *, batch: int = 1,
         stride_a: int = 0, stride_b: int = 0,
         scale_a: Optional[np.ndarray] = None, scale_b: Optional[np.ndarray] = None,
         bias: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Full oracle product.  Returns (C_ref, D), each fp64 of shape (batch, M, N).

    With `bias` (N fp32 values, the AddMM shape of the paper's App. D): C_ref[b,i,j] += bias[j] and
    D[b,i,j] += |bias[j]|, both in fp64, so that the acceptance metric stays a bound relative to the
    magnitude of the terms summed."""
    lib = _load()
    A = _check_storage(dtype, A, "A")
    B = _check_storage(dtype, B, "B")
    if scale_a is not None:
        scale_a = np.ascontiguousarray(scale_a, dtype=np.float32)
    if scale_b is not None:
        scale_b = np.ascontiguousarray(scale_b, dtype=np.float32)
    C = np.zeros((batch, M, N), dtype=np.float64)
    D = np.zeros((batch, M, N), dtype=np.float64)
    rc = lib.oracle_gemm(dtype, layout_a, layout_b, M, N, K, batch,
                         _ptr(A), lda, stride_a, _ptr(B), ldb, stride_b,
                         _ptr(scale_a), _ptr(scale_b), _ptr(C), _ptr(D), max(N, 1), M * N)
    if rc != 0:
        raise ValueError(f"oracle_gemm rejected its arguments (code {rc})")
    if bias is not None:
        bias64 = np.asarray(bias, dtype=np.float32).astype(np.float64).reshape(1, 1, N)
        C += bias64
        D += np.abs(bias64)
    return C, D


def gemm_points(dtype: int, layout_a: int, layout_b: int, M: int, N: int, K: int,
                A: np.ndarray, lda: int, B: np.ndarray, ldb: int,
                pb: np.ndarray, pi: np.ndarray, pj: np.ndarray, *, batch: int = 1,
                stride_a: int = 0, stride_b: int = 0,
                scale_a: Optional[np.ndarray] = None, scale_b: Optional[np.ndarray] = None,
                bias: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Oracle values at selected (batch, i, j) points.  Returns (C_ref, D), each fp64 of shape (n,).
    `bias` as in gemm()."""
    lib = _load()
    A = _check_storage(dtype, A, "A")
    B = _check_storage(dtype, B, "B")
    pb = np.ascontiguousarray(pb, dtype=np.int64)
    pi = np.ascontiguousarray(pi, dtype=np.int64)
    pj = np.ascontiguousarray(pj, dtype=np.int64)
    n = pb.size
    if pi.size != n or pj.size != n:
        raise ValueError("point index arrays differ in length")
    if scale_a is not None:
        scale_a = np.ascontiguousarray(scale_a, dtype=np.float32)
    if scale_b is not None:
        scale_b = np.ascontiguousarray(scale_b, dtype=np.float32)
    C = np.zeros(n, dtype=np.float64)
    D = np.zeros(n, dtype=np.float64)
    rc = lib.oracle_gemm_points(dtype, layout_a, layout_b, M, N, K, batch,
                                _ptr(A), lda, stride_a, _ptr(B), ldb, stride_b,
                                _ptr(scale_a), _ptr(scale_b), n, _ptr(pb), _ptr(pi), _ptr(pj),
                                _ptr(C), _ptr(D))
    if rc != 0:
        raise ValueError(f"oracle_gemm_points rejected its arguments (code {rc})")
    if bias is not None:
        bias64 = np.asarray(bias, dtype=np.float32).astype(np.float64)[pj]
        C += bias64
        D += np.abs(bias64)
    return C, D


def conv2d_output_size(H: int, W: int, R: int, S: int, stride: Tuple[int, int], pad: Tuple[int, int]) -> Tuple[int, int]:
    """(P, Q) as the C oracle defines them (one definition: the buffers below are sized by it)."""
    P, Q = ctypes.c_int64(0), ctypes.c_int64(0)
    _load().oracle_conv2d_output_size(H, W, R, S, stride[0], stride[1], pad[0], pad[1], ctypes.byref(P), ctypes.byref(Q))
    return int(P.value), int(Q.value)


def conv2d(dtype: int, x: np.ndarray, w: np.ndarray, *, stride: Tuple[int, int] = (1, 1),
           pad: Tuple[int, int] = (0, 0), bias: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Oracle convolution layer.  x: (N, H, W, C) stored codes, w: (F, R, S, C) stored codes.
    Returns (y_ref, D), each fp64 of shape (N, P, Q, F).  With `bias` (F fp32 values):
    y_ref[..., f] += bias[f] and D[..., f] += |bias[f]| in fp64."""
    lib = _load()
    x = _check_storage(dtype, x, "x")
    w = _check_storage(dtype, w, "w")
    N, H, W, C = x.shape
    F, R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("x and w disagree on the number of channels")
    if min(stride) < 1 or min(pad) < 0 or H + 2 * pad[0] < R or W + 2 * pad[1] < S:
        raise ValueError("oracle conv2d: stride, padding or filter size out of range")
    P, Q = conv2d_output_size(H, W, R, S, stride, pad)
    y = np.zeros((N, max(P, 0), max(Q, 0), F), dtype=np.float64)
    d = np.zeros_like(y)
    rc = lib.oracle_conv2d(dtype, N, H, W, C, F, R, S, stride[0], stride[1], pad[0], pad[1],
                           _ptr(x), _ptr(w), _ptr(y), _ptr(d))
    if rc != 0:
        raise ValueError(f"oracle_conv2d rejected its arguments (code {rc})")
    if bias is not None:
        b64 = np.asarray(bias, dtype=np.float32).astype(np.float64).reshape(1, 1, 1, F)
        y += b64
        d += np.abs(b64)
    return y, d


def conv2d_points(dtype: int, x: np.ndarray, w: np.ndarray, pn: np.ndarray, pp: np.ndarray, pq: np.ndarray,
                  pf: np.ndarray, *, stride: Tuple[int, int] = (1, 1), pad: Tuple[int, int] = (0, 0),
                  bias: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Oracle values at selected outputs (n, p, q, f).  Returns (y_ref, D), each fp64 of shape (npts,)."""
    lib = _load()
    x = _check_storage(dtype, x, "x")
    w = _check_storage(dtype, w, "w")
    N, H, W, C = x.shape
    F, R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("x and w disagree on the number of channels")
    idx = [np.ascontiguousarray(a, dtype=np.int64) for a in (pn, pp, pq, pf)]
    n = idx[0].size
    if any(a.size != n for a in idx):
        raise ValueError("point index arrays differ in length")
    y = np.zeros(n, dtype=np.float64)
    d = np.zeros(n, dtype=np.float64)
    rc = lib.oracle_conv2d_points(dtype, N, H, W, C, F, R, S, stride[0], stride[1], pad[0], pad[1],
                                  _ptr(x), _ptr(w), n, *[_ptr(a) for a in idx], _ptr(y), _ptr(d))
    if rc != 0:
        raise ValueError(f"oracle_conv2d_points rejected its arguments (code {rc})")
    if bias is not None:
        b64 = np.asarray(bias, dtype=np.float32).astype(np.float64)[idx[3]]
        y += b64
        d += np.abs(b64)
    return y, d


def topk(x: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Oracle top-k of each row of a 2-D fp32 array (rows may be a strided view along axis 0).
    Returns (idx int32, val fp32), each (batch, k): the k largest, ties towards lower indices,
    listed in increasing index order."""
    lib = _load()
    if x.dtype != np.float32 or x.ndim != 2 or x.strides[1] != 4 or x.strides[0] % 4 != 0:
        raise TypeError("oracle topk wants a 2-D fp32 array with contiguous rows")
    batch, n = x.shape
    ld = x.strides[0] // 4 if batch > 1 else max(n, 1)
    idx = np.zeros((batch, k), dtype=np.int32)
    val = np.zeros((batch, k), dtype=np.float32)
    rc = lib.oracle_topk(batch, n, k, x.ctypes.data_as(ctypes.c_void_p), ld, _ptr(idx), _ptr(val))
    if rc != 0:
        raise ValueError(f"oracle_topk rejected its arguments (code {rc})")
    return idx, val
