"""Seeded synthetic inputs for the GEMM lineage, the convolution layer and the top-k selection built
beside it (shared by the GPU tests and the CPU oracle tests).

This module holds none of their arithmetic: it only draws numbers, quantises them to
the storage format and describes the benchmark workloads.  Neither the HIP
library nor the oracle imports it; tests hand its arrays to both.

Generator.  Element ``n`` (linear position in the stored buffer) of tensor ``t``
under seed ``s`` is a pure function of ``(s, t, n)``: two 64-bit words come from
a SplitMix64-style finaliser applied to a counter, each gives a uniform in (0,1)
from its top 24 bits, and a normal deviate is the Box-Muller cosine branch of the
pair.  Generation is therefore independent of chunking and thread count.

Workloads.  ``CONFIGS`` lists the five shapes the validation gate is run on
(paper Sec. 4.1 measures GEMM at one square bf16 shape with unspecified values;
these synthetic shapes stand in for it and for the held-out GEMM-family shapes
of its App. D).  Smaller ``*_small`` variants keep the same dtype, layout, value
distribution and raggedness at sizes a CPU reference finishes in seconds.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

# dtype / layout codes: numerically equal to the enums of include/gemm_lineage.h
F32, BF16, F16, E4M3 = 0, 1, 2, 3
ROW_MAJOR, COL_MAJOR = 0, 1
DTYPE_NAMES = {F32: "f32", BF16: "bf16", F16: "f16", E4M3: "e4m3"}
STORAGE = {F32: np.float32, BF16: np.uint16, F16: np.uint16, E4M3: np.uint8}
ELEM_BYTES = {F32: 4, BF16: 2, F16: 2, E4M3: 1}

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def _mix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 output function (Steele, Lea, Flood 2014): a bijective 64-bit finaliser."""
    x = x.astype(np.uint64, copy=True)
    x ^= x >> np.uint64(30)
    x *= _C1
    x ^= x >> np.uint64(27)
    x *= _C2
    x ^= x >> np.uint64(31)
    return x


def _key(seed: int, tensor: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([np.uint64(seed) * _GOLDEN + np.uint64(1)], dtype=np.uint64))
        k = _mix64(k ^ (np.uint64(tensor) * _C1 + np.uint64(0x5851F42D4C957F2D)))
    return k[0]


def raw_words(seed: int, tensor: int, start: int, count: int, lane: int) -> np.ndarray:
    """64-bit word ``lane`` (0 or 1) for elements ``start .. start+count-1``."""
    with np.errstate(over="ignore"):
        n = np.arange(start, start + count, dtype=np.uint64)
        ctr = (n * np.uint64(2) + np.uint64(lane)) * _GOLDEN + _key(seed, tensor)
        return _mix64(ctr)


def unit_uniform(seed: int, tensor: int, start: int, count: int, lane: int = 0) -> np.ndarray:
    """Uniform on the open interval (0,1): (top 24 bits + 1/2) / 2^24, as fp64."""
    w = raw_words(seed, tensor, start, count, lane)
    return ((w >> np.uint64(40)).astype(np.float64) + 0.5) * (1.0 / 16777216.0)


def _chunked(fn, count: int, chunk: int = 1 << 22, threads: int = 8) -> np.ndarray:
    if count <= chunk:
        return fn(0, count)
    starts = list(range(0, count, chunk))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(lambda s: fn(s, min(chunk, count - s)), starts))
    return np.concatenate(parts)


def uniform_pm1(seed: int, tensor: int, count: int) -> np.ndarray:
    """iid uniform on (-1, 1), fp32."""
    return _chunked(lambda s, c: (2.0 * unit_uniform(seed, tensor, s, c) - 1.0).astype(np.float32), count)


def uniform_range(seed: int, tensor: int, count: int, lo: float, hi: float) -> np.ndarray:
    return _chunked(lambda s, c: (lo + (hi - lo) * unit_uniform(seed, tensor, s, c)).astype(np.float32), count)


def normal(seed: int, tensor: int, count: int, std: float = 1.0) -> np.ndarray:
    """iid N(0, std^2), fp32; Box-Muller on the element's two uniforms."""
    def part(s, c):
        u1 = unit_uniform(seed, tensor, s, c, 0)
        u2 = unit_uniform(seed, tensor, s, c, 1)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)
        return (std * z).astype(np.float32)
    return _chunked(part, count)


# ----------------------------------------------------------------------------
# storage quantisers (round to nearest, ties to even)
# ----------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), RNE; inputs must be finite."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def to_f16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> IEEE binary16 bit patterns (uint16), RNE (numpy's conversion)."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> OCP E4M3 codes (uint8), RNE, magnitudes clipped to the largest finite value 448."""
    x = np.ascontiguousarray(x, dtype=np.float32).astype(np.float64)
    sign = (np.signbit(x)).astype(np.uint8) << 7
    ax = np.minimum(np.abs(x), 448.0)
    frac, ex = np.frexp(ax)                  # ax = frac * 2^ex, frac in [0.5, 1)
    e = ex - 1                               # ax = (2 frac) * 2^e, 2 frac in [1, 2)
    sub = ax < 2.0 ** -6
    # subnormal grid: multiples of 2^-9; a result of 8 is the smallest normal and its code is 8 too
    q_sub = np.rint(ax * 512.0)
    m = np.rint((2.0 * frac - 1.0) * 8.0)
    carry = m == 8.0
    m = np.where(carry, 0.0, m)
    e = np.where(carry, e + 1, e)
    code_norm = ((e + 7).astype(np.int64) << 3) | m.astype(np.int64)
    code = np.where(sub, q_sub.astype(np.int64), code_norm)
    code = np.minimum(code, 0x7E)
    return (code.astype(np.uint8) | sign).astype(np.uint8)


def quantise(dtype: int, x: np.ndarray) -> np.ndarray:
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return to_bf16_bits(x)
    if dtype == F16:
        return to_f16_bits(x)
    if dtype == E4M3:
        return to_e4m3_bits(x)
    raise ValueError(f"unknown dtype code {dtype}")


# ----------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    M: int
    N: int
    K: int
    in_dtype: int
    out_dtype: int
    layout_a: int
    layout_b: int
    dist: str                 # "uniform" | "normal"
    std: float = 1.0          # for "normal"; the literal "rsqrtK" scale is folded in by make_inputs
    rsqrt_k: bool = False
    batch: int = 1
    scaled: bool = False      # per-problem scale_a[b], scale_b[b] ~ U[0.5, 2]
    biased: bool = False      # bias[j] ~ N(0, 1), fp32, added in the epilogue (AddMM)
    lda: int = 0              # 0 = tight
    ldb: int = 0
    ldc: int = 0

    @property
    def ld(self) -> Tuple[int, int, int]:
        lda = self.lda or (self.K if self.layout_a == ROW_MAJOR else self.M)
        ldb = self.ldb or (self.N if self.layout_b == ROW_MAJOR else self.K)
        ldc = self.ldc or self.N
        return lda, ldb, ldc

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K * self.batch

    @property
    def algorithmic_bytes(self) -> int:
        """Each operand read once, C written once, at storage width."""
        return self.batch * ((self.M * self.K + self.K * self.N) * ELEM_BYTES[self.in_dtype]
                             + self.M * self.N * ELEM_BYTES[self.out_dtype])


CONFIGS: Dict[str, Config] = {
    # the five gate workloads
    "C1": Config("C1", 256, 256, 256, F32, F32, ROW_MAJOR, ROW_MAJOR, "uniform"),
    "C2": Config("C2", 8192, 8192, 8192, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True),
    "C3": Config("C3", 4099, 4093, 4097, F16, F16, ROW_MAJOR, ROW_MAJOR, "uniform"),
    "C4": Config("C4", 16, 16384, 16384, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", std=0.02),
    "C5": Config("C5", 1024, 1024, 1024, E4M3, BF16, ROW_MAJOR, COL_MAJOR, "normal", batch=64, scaled=True),
    # the paper's own GEMM shape (Sec. 4.1, workload table) and the held-out GEMM-family shapes of its
    # App. D that are plain (batched) products; bf16, same layouts and value recipe as C2
    "P4096": Config("P4096", 4096, 4096, 4096, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True),
    "P2048": Config("P2048", 2048, 2048, 2048, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True),
    "PBMM16": Config("PBMM16", 2048, 2048, 2048, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True, batch=16),
    "PBMM32": Config("PBMM32", 1024, 1024, 1024, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True, batch=32),
    "PADDMM": Config("PADDMM", 4096, 4096, 4096, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True, biased=True),
    # decode-like shapes with more rows than C4 (its recipe): 32 and 64 rows still stream, 128 rows are
    # the split-K form's case
    "D32": Config("D32", 32, 16384, 16384, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", std=0.02),
    "D64": Config("D64", 64, 16384, 16384, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", std=0.02),
    "D128": Config("D128", 128, 16384, 16384, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", std=0.02),
    # C4's shape with e4m3 operands and C5's value recipe and scales: the streaming kernel on one-byte elements
    "D16_e4m3": Config("D16_e4m3", 16, 16384, 16384, E4M3, BF16, ROW_MAJOR, COL_MAJOR, "normal", scaled=True),
    # reduced-size counterparts: same dtype / layout / distribution / raggedness
    "C2_small": Config("C2_small", 512, 768, 640, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", rsqrt_k=True),
    "C3_small": Config("C3_small", 387, 301, 259, F16, F16, ROW_MAJOR, ROW_MAJOR, "uniform"),
    "C4_small": Config("C4_small", 16, 1024, 2048, BF16, BF16, ROW_MAJOR, COL_MAJOR, "normal", std=0.02),
    "C5_small": Config("C5_small", 256, 256, 256, E4M3, BF16, ROW_MAJOR, COL_MAJOR, "normal", batch=3, scaled=True),
}

TENSOR_A, TENSOR_B, TENSOR_SCALE_A, TENSOR_SCALE_B, TENSOR_BIAS = 1, 2, 3, 4, 5


def _draw(cfg: Config, seed: int, tensor: int, count: int) -> np.ndarray:
    if cfg.dist == "uniform":
        return uniform_pm1(seed, tensor, count)
    std = cfg.std * (1.0 / math.sqrt(cfg.K) if cfg.rsqrt_k else 1.0)
    x = normal(seed, tensor, count, std)
    if cfg.in_dtype == E4M3:
        np.clip(x, -448.0, 448.0, out=x)
    return x


@dataclass
class Inputs:
    cfg: Config
    seed: int
    A: np.ndarray                       # raw storage, 1-D, batch * stride_a elements
    B: np.ndarray
    lda: int
    ldb: int
    ldc: int
    stride_a: int
    stride_b: int
    stride_c: int
    scale_a: Optional[np.ndarray] = None    # fp32, one per batch item
    scale_b: Optional[np.ndarray] = None
    bias: Optional[np.ndarray] = None       # fp32, N values
    meta: dict = field(default_factory=dict)


def make_inputs(cfg: Config, seed: int) -> Inputs:
    """Draw, quantise and lay out the operands of one workload."""
    lda, ldb, ldc = cfg.ld
    rows_a = cfg.M if cfg.layout_a == ROW_MAJOR else cfg.K
    rows_b = cfg.K if cfg.layout_b == ROW_MAJOR else cfg.N
    stride_a, stride_b, stride_c = rows_a * lda, rows_b * ldb, cfg.M * ldc
    A = quantise(cfg.in_dtype, _draw(cfg, seed, TENSOR_A, cfg.batch * stride_a))
    B = quantise(cfg.in_dtype, _draw(cfg, seed, TENSOR_B, cfg.batch * stride_b))
    sa = sb = None
    if cfg.scaled:
        sa = uniform_range(seed, TENSOR_SCALE_A, cfg.batch, 0.5, 2.0)
        sb = uniform_range(seed, TENSOR_SCALE_B, cfg.batch, 0.5, 2.0)
    bias = normal(seed, TENSOR_BIAS, cfg.N, 1.0).astype(np.float32) if cfg.biased else None
    return Inputs(cfg, seed, A, B, lda, ldb, ldc, stride_a, stride_b, stride_c, sa, sb, bias)


# ----------------------------------------------------------------------------
# convolution layer (paper Sec. 4.1, workload table: Conv2d)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class ConvConfig:
    """x: N x H x W x C, w: F x R x S x C, y: N x P x Q x F; all dense, channels fastest.

    The paper gives the sizes and the dtype and no value distribution: activations are drawn uniform
    in [-1, 1], filters normal with standard deviation 1/sqrt(R*S*C) (outputs of order 1), the bias
    (where present) standard normal in fp32."""
    name: str
    N: int
    H: int
    W: int
    C: int
    F: int
    R: int
    S: int
    in_dtype: int
    out_dtype: int
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (1, 1)
    biased: bool = False

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad[0] - self.R) // self.stride[0] + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad[1] - self.S) // self.stride[1] + 1

    @property
    def flops(self) -> float:
        """2 x multiply-adds of the layer lowered to a matrix product (taps in the padding counted)."""
        return 2.0 * self.N * self.P * self.Q * self.F * self.R * self.S * self.C

    @property
    def algorithmic_bytes(self) -> int:
        """x and w read once, y written once, at storage width."""
        return ((self.N * self.H * self.W * self.C + self.F * self.R * self.S * self.C) * ELEM_BYTES[self.in_dtype]
                + self.N * self.P * self.Q * self.F * ELEM_BYTES[self.out_dtype])


CONV_CONFIGS: Dict[str, ConvConfig] = {
    # the paper's layer
    "CONV": ConvConfig("CONV", 8, 56, 56, 64, 128, 3, 3, F16, F16),
    # reduced and ragged counterparts: odd image sizes, strides, paddings, partial tiles in both directions
    "CONV_small": ConvConfig("CONV_small", 2, 13, 11, 64, 40, 3, 3, F16, F16),
    "CONV_stride2": ConvConfig("CONV_stride2", 3, 17, 15, 128, 136, 3, 3, BF16, BF16, stride=(2, 2), pad=(1, 1), biased=True),
    "CONV_5x3": ConvConfig("CONV_5x3", 1, 20, 9, 64, 24, 5, 3, F16, F32, stride=(1, 2), pad=(2, 0)),
    "CONV_1x1": ConvConfig("CONV_1x1", 2, 9, 9, 192, 130, 1, 1, BF16, BF16, pad=(0, 0)),
    "CONV_fp8": ConvConfig("CONV_fp8", 2, 10, 12, 128, 72, 3, 3, E4M3, BF16),
    # channels that are not whole 128-byte slabs: the implicit state refuses, im2col pads K
    "CONV_c24": ConvConfig("CONV_c24", 2, 12, 10, 24, 20, 3, 3, F16, F16),
    "CONV_c3": ConvConfig("CONV_c3", 1, 16, 16, 3, 8, 7, 7, BF16, BF16, stride=(2, 2), pad=(3, 3)),
}

TENSOR_X, TENSOR_W, TENSOR_CONV_BIAS = 11, 12, 13


@dataclass
class ConvInputs:
    cfg: ConvConfig
    seed: int
    x: np.ndarray                       # raw storage, shape (N, H, W, C)
    w: np.ndarray                       # raw storage, shape (F, R, S, C)
    bias: Optional[np.ndarray] = None   # fp32, F values


def make_conv_inputs(cfg: ConvConfig, seed: int) -> ConvInputs:
    nx, nw = cfg.N * cfg.H * cfg.W * cfg.C, cfg.F * cfg.R * cfg.S * cfg.C
    xv = uniform_pm1(seed, TENSOR_X, nx)
    wv = normal(seed, TENSOR_W, nw, 1.0 / math.sqrt(cfg.R * cfg.S * cfg.C))
    if cfg.in_dtype == E4M3:
        wv = wv * 16.0      # keep the filters clear of e4m3's subnormal range; the metric is scale-invariant
    x = quantise(cfg.in_dtype, xv).reshape(cfg.N, cfg.H, cfg.W, cfg.C)
    w = quantise(cfg.in_dtype, wv).reshape(cfg.F, cfg.R, cfg.S, cfg.C)
    bias = normal(seed, TENSOR_CONV_BIAS, cfg.F, 1.0).astype(np.float32) if cfg.biased else None
    return ConvInputs(cfg, seed, x, w, bias)


# ----------------------------------------------------------------------------
# row-wise top-k (paper Sec. 4.1, workload table: Top-K)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class TopkConfig:
    """x: batch rows of n fp32 values, ld elements apart.  The paper gives the shape only; values are
    standard normal ("normal"), or standard normal rounded to multiples of 1/4 so that many elements tie,
    also at the threshold ("ties")."""
    name: str
    batch: int
    n: int
    k: int
    ld: int = 0               # 0 = tight
    dist: str = "normal"

    @property
    def algorithmic_bytes(self) -> int:
        """The rows read once, indices and values written once."""
        return self.batch * (self.n * 4 + self.k * 8)


TOPK_CONFIGS: Dict[str, TopkConfig] = {
    "TOPK": TopkConfig("TOPK", 64, 4096, 512),                       # the paper's shape
    "TOPK_ties": TopkConfig("TOPK_ties", 64, 4096, 512, dist="ties"),
    "TOPK_small": TopkConfig("TOPK_small", 5, 1000, 37, ld=1004),
    "TOPK_ragged": TopkConfig("TOPK_ragged", 3, 4099, 4000, ld=4100, dist="ties"),
    "TOPK_wide": TopkConfig("TOPK_wide", 2, 16384, 2048, dist="ties"),
    "TOPK_long": TopkConfig("TOPK_long", 2, 70001, 300),             # beyond what T0 and T2 hold: both refuse
}

TENSOR_TOPK = 21


def make_topk_inputs(cfg: TopkConfig, seed: int) -> np.ndarray:
    """Returns the (batch, ld) fp32 buffer; the row is its first n columns, the rest is padding (huge
    values, which a kernel that read past n would select)."""
    ld = cfg.ld or cfg.n
    x = normal(seed, TENSOR_TOPK, cfg.batch * ld, 1.0).astype(np.float32).reshape(cfg.batch, ld)
    if cfg.dist == "ties":
        x = (np.round(x * 4.0) / 4.0).astype(np.float32)
    x[:, cfg.n:] = 1.0e30
    return x
