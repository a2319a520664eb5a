"""Pins for the CPU oracle: everything here runs without a GPU and without the HIP library.

The paper prints no GEMM output value (Sec. 4.1 only says correctness is checked at three
seeds), so the oracle is held in place by what mathematics fixes: library dtype conversions
and the OCP FP8 spec's named values for the decoders; closed forms (identity, all-ones = K,
rank-1), exact integer products against numpy's int64 matmul, exact rational brute force on
tiny ragged shapes, and algebraic identities (transpose, permutation, power-of-two scaling).
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2605_28213_amd import inputs as gen

F32, BF16, F16, E4M3 = 0, 1, 2, 3
ROW, COL = 0, 1
ALL_DTYPES = [F32, BF16, F16, E4M3]


# ---------------------------------------------------------------- decoders
def test_decode_bf16_every_code(oracle):
    codes = np.arange(65536, dtype=np.uint32)
    want = (codes << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    got = oracle.decode(BF16, codes)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    assert np.signbit(got[0x8000]) and got[0x8000] == 0.0


def test_decode_f16_every_code(oracle):
    codes = np.arange(65536, dtype=np.uint16)
    want = codes.view(np.float16).astype(np.float64)
    got = oracle.decode(F16, codes)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    assert got[0x7BFF] == 65504.0 and got[0x0001] == 2.0 ** -24 and got[0x0400] == 2.0 ** -14


def test_decode_e4m3_every_code_vs_torch_and_spec(oracle):
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = oracle.decode(E4M3, codes)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    # values named in the OCP 8-bit floating point specification (E4M3 column)
    assert got[0x7E] == 448.0 and got[0xFE] == -448.0          # max normal S.1111.110
    assert got[0x08] == 2.0 ** -6                               # min normal
    assert got[0x07] == 0.875 * 2.0 ** -6                       # max subnormal
    assert got[0x01] == 2.0 ** -9                               # min subnormal
    assert got[0x38] == 1.0 and got[0x00] == 0.0
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF])          # only NaN codes; no infinities
    assert np.all(np.isfinite(got[ok]))


def test_decode_f32_samples(oracle):
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 2 ** 32, size=2000, dtype=np.uint64).astype(np.uint32)
    bits = np.concatenate([bits, np.array([0, 1, 0x007FFFFF, 0x00800000, 0x3F800000, 0x7F7FFFFF, 0x80000000],
                                          dtype=np.uint32)])
    want = bits.view(np.float32).astype(np.float64)
    got = oracle.decode(F32, bits)          # < 4096 elements: goes through the C decoder
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))


def test_quantisers_roundtrip_through_oracle_decode(oracle):
    """encode(decode(code)) == code for every finite code; RNE at exact midpoints."""
    for dt, nb, enc in [(BF16, 16, gen.to_bf16_bits), (F16, 16, gen.to_f16_bits), (E4M3, 8, gen.to_e4m3_bits)]:
        codes = np.arange(1 << nb, dtype=np.uint32)
        vals = oracle.decode(dt, codes)
        fin = np.isfinite(vals)
        back = enc(vals[fin].astype(np.float32))
        np.testing.assert_array_equal(back.astype(np.uint32), codes[fin])
    # e4m3 midpoints: halfway between neighbours goes to the even code, saturation at 448
    vals = oracle.decode(E4M3, np.arange(0x7F, dtype=np.uint32))
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    enc = gen.to_e4m3_bits(mids).astype(np.int64)
    lo = np.arange(0x7E, dtype=np.int64)
    want = np.where(lo % 2 == 0, lo, lo + 1)
    np.testing.assert_array_equal(enc, want)
    assert gen.to_e4m3_bits(np.array([1e9, -1e9, 449.0, 464.0], np.float32)).tolist() == [0x7E, 0xFE, 0x7E, 0x7E]
    # bf16 midpoint: 1 + 2^-8 is halfway between 1 (even) and 1+2^-7
    assert gen.to_bf16_bits(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)).tolist() == [0x3F80, 0x3F82]


# ---------------------------------------------------------------- helpers
def _small_ints(rng, shape, lo=-2, hi=2):
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def _store(dt, logical, layout, ld=None, pad_value=None):
    """Lay a logical (rows x cols) fp32 matrix out in storage; returns (raw 1-D buffer, ld)."""
    r, c = logical.shape
    major, minor = (r, c) if layout == ROW else (c, r)
    ld = ld or max(minor, 1)
    buf = np.full((major, ld), 7.0 if pad_value is None else pad_value, dtype=np.float32)
    buf[:, :minor] = logical if layout == ROW else logical.T
    return gen.quantise(dt, buf.ravel()), ld


def _run(oracle, dt, la, lb, Al, Bl, **kw):
    M, K = Al.shape
    K2, N = Bl.shape
    assert K == K2
    A, lda = _store(dt, Al, la, kw.pop("lda", None))
    B, ldb = _store(dt, Bl, lb, kw.pop("ldb", None))
    C, D = oracle.gemm(dt, la, lb, M, N, K, A, lda, B, ldb, **kw)
    return C[0], D[0]


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("dt", ALL_DTYPES)
@pytest.mark.parametrize("la,lb", [(ROW, ROW), (ROW, COL), (COL, ROW), (COL, COL)])
def test_identity(oracle, dt, la, lb):
    rng = np.random.default_rng(1)
    n, m = 9, 5
    X = _small_ints(rng, (n, m), -3, 3) * 0.5          # exactly representable in every dtype
    I = np.eye(n, dtype=np.float32)
    C, D = _run(oracle, dt, la, lb, I, X)
    np.testing.assert_array_equal(C, X.astype(np.float64))
    np.testing.assert_array_equal(D, np.abs(X).astype(np.float64))
    Y = X.T.copy()
    C, _ = _run(oracle, dt, la, lb, Y, I)
    np.testing.assert_array_equal(C, Y.astype(np.float64))


@pytest.mark.parametrize("dt", ALL_DTYPES)
@pytest.mark.parametrize("K", [1, 7, 256, 4097])
def test_all_ones_gives_K(oracle, dt, K):
    C, D = _run(oracle, dt, ROW, COL, np.ones((3, K), np.float32), np.ones((K, 4), np.float32))
    assert np.all(C == K) and np.all(D == K)


def test_all_ones_K16384(oracle):
    C, D = _run(oracle, BF16, ROW, COL, np.ones((1, 16384), np.float32), np.ones((16384, 2), np.float32))
    assert np.all(C == 16384) and np.all(D == 16384)


@pytest.mark.parametrize("dt", ALL_DTYPES)
def test_rank_one(oracle, dt):
    u = np.array([1.0, -2.0, 0.5, 3.0, -0.25], np.float32)
    v = np.array([2.0, 0.5, -1.5, 4.0], np.float32)
    C, D = _run(oracle, dt, ROW, ROW, u[:, None], v[None, :])
    np.testing.assert_array_equal(C, np.outer(u, v).astype(np.float64))
    np.testing.assert_array_equal(D, np.abs(np.outer(u, v)).astype(np.float64))
    K = 37
    C, _ = _run(oracle, dt, ROW, COL, np.repeat(u[:, None], K, 1), np.repeat(v[None, :], K, 0))
    np.testing.assert_array_equal(C, K * np.outer(u, v).astype(np.float64))


@pytest.mark.parametrize("dt", ALL_DTYPES)
@pytest.mark.parametrize("la,lb", [(ROW, ROW), (ROW, COL), (COL, ROW), (COL, COL)])
def test_integer_valued_exact_vs_int64_matmul(oracle, dt, la, lb):
    """Entries in {-2..2}: every partial sum is a small integer, so the product is exact; numpy's
    integer matmul is an independent exact routine.  Non-square and ragged on purpose."""
    rng = np.random.default_rng(2 + dt)
    M, N, K = 23, 17, 301
    Al, Bl = _small_ints(rng, (M, K)), _small_ints(rng, (K, N))
    C, D = _run(oracle, dt, la, lb, Al, Bl, lda=(K if la == ROW else M) + 3, ldb=(N if lb == ROW else K) + 5)
    want = Al.astype(np.int64) @ Bl.astype(np.int64)
    wantD = np.abs(Al).astype(np.int64) @ np.abs(Bl).astype(np.int64)
    np.testing.assert_array_equal(C, want.astype(np.float64))
    np.testing.assert_array_equal(D, wantD.astype(np.float64))


# ---------------------------------------------------------------- exact brute force
def _frac(x):
    return Fraction(float(x))


@pytest.mark.parametrize("dt", ALL_DTYPES)
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 5), (5, 2, 17), (3, 17, 2), (17, 5, 3)])
@pytest.mark.parametrize("la,lb", [(ROW, ROW), (ROW, COL), (COL, ROW), (COL, COL)])
def test_exact_rational_brute_force(oracle, dt, M, N, K, la, lb):
    """Random non-integer values; the reference sums exact rationals in pure Python, rounding once."""
    rng = np.random.default_rng(1000 * dt + 100 * M + 10 * N + K)
    Al = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    Bl = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    A, lda = _store(dt, Al, la)
    B, ldb = _store(dt, Bl, lb)
    # decode the stored codes with library conversions, not with the oracle
    if dt == F32:
        Av, Bv = A.astype(np.float64), B.astype(np.float64)
    elif dt == BF16:
        Av = (A.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        Bv = (B.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    elif dt == F16:
        Av, Bv = A.view(np.float16).astype(np.float64), B.view(np.float16).astype(np.float64)
    else:
        Av = torch.from_numpy(A.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
        Bv = torch.from_numpy(B.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    a = (lambda i, k: Av[i * lda + k]) if la == ROW else (lambda i, k: Av[k * lda + i])
    b = (lambda k, j: Bv[k * ldb + j]) if lb == ROW else (lambda k, j: Bv[j * ldb + k])
    C, D = oracle.gemm(dt, la, lb, M, N, K, A, lda, B, ldb)
    for i in range(M):
        for j in range(N):
            exact = sum((_frac(a(i, k)) * _frac(b(k, j)) for k in range(K)), Fraction(0))
            mag = sum((abs(_frac(a(i, k)) * _frac(b(k, j))) for k in range(K)), Fraction(0))
            assert abs(Fraction(float(C[0, i, j])) - exact) <= Fraction(1, 2 ** 50) * mag + Fraction(1, 2 ** 1000)
            assert abs(Fraction(float(D[0, i, j])) - mag) <= Fraction(1, 2 ** 50) * mag


# ---------------------------------------------------------------- algebra
@pytest.mark.parametrize("dt", ALL_DTYPES)
def test_transpose_identity(oracle, dt):
    """(A B)^T = B^T A^T, evaluated by swapping operands and layout flags on the same buffers."""
    cfg_rng = np.random.default_rng(5)
    M, N, K = 11, 7, 29
    Al = cfg_rng.uniform(-1, 1, (M, K)).astype(np.float32)
    Bl = cfg_rng.uniform(-1, 1, (K, N)).astype(np.float32)
    A, lda = _store(dt, Al, ROW)
    B, ldb = _store(dt, Bl, ROW)
    C, D = oracle.gemm(dt, ROW, ROW, M, N, K, A, lda, B, ldb)
    # B row-major K x N read as column-major is B^T (N x K); same for A
    Ct, Dt = oracle.gemm(dt, COL, COL, N, M, K, B, ldb, A, lda)
    np.testing.assert_array_equal(Ct[0], C[0].T)
    np.testing.assert_array_equal(Dt[0], D[0].T)


def test_permutation_and_pow2_scaling(oracle):
    rng = np.random.default_rng(6)
    M, N, K = 6, 8, 8
    Al = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    perm = rng.permutation(K)
    P = np.zeros((K, N), np.float32)
    P[perm, np.arange(N)] = 1.0
    C, _ = _run(oracle, F32, ROW, ROW, Al, P)
    np.testing.assert_array_equal(C, Al[:, perm].astype(np.float64))
    Bl = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    C1, D1 = _run(oracle, F32, ROW, COL, Al, Bl)
    C2, D2 = _run(oracle, F32, ROW, COL, Al * 8.0, Bl * 0.25)
    np.testing.assert_array_equal(C2, 2.0 * C1)
    np.testing.assert_array_equal(D2, 2.0 * D1)


def test_sign_and_operand_order_matter(oracle):
    """A planted transposition or sign slip would survive symmetric inputs; these are neither."""
    Al = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]], np.float32)           # 2 x 3
    Bl = np.array([[1.0, -1.0], [0.5, 2.0], [-2.0, 0.25]], np.float32)      # 3 x 2
    C, D = _run(oracle, F32, ROW, ROW, Al, Bl)
    np.testing.assert_array_equal(C, np.array([[-4.0, 3.75], [-5.5, 7.5]]))
    np.testing.assert_array_equal(D, np.array([[8.0, 5.75], [18.5, 15.5]]))


# ---------------------------------------------------------------- batch, scales, strides, points
def test_batch_scales_and_points(oracle):
    rng = np.random.default_rng(7)
    M, N, K, nb = 5, 6, 19, 3
    A = gen.quantise(E4M3, rng.normal(0, 1, nb * M * K).astype(np.float32))
    B = gen.quantise(E4M3, rng.normal(0, 1, nb * N * K).astype(np.float32))
    sa = np.array([0.5, -2.0, 1.25], np.float32)
    sb = np.array([2.0, 0.5, 1.5], np.float32)
    C, D = oracle.gemm(E4M3, ROW, COL, M, N, K, A, K, B, K, batch=nb, stride_a=M * K, stride_b=N * K,
                       scale_a=sa, scale_b=sb)
    C0, D0 = oracle.gemm(E4M3, ROW, COL, M, N, K, A, K, B, K, batch=nb, stride_a=M * K, stride_b=N * K)
    for b in range(nb):
        s = float(sa[b]) * float(sb[b])
        np.testing.assert_array_equal(C[b], s * C0[b])
        np.testing.assert_array_equal(D[b], abs(s) * D0[b])
        # each batch item equals the single-problem product on its slice
        Cb, _ = oracle.gemm(E4M3, ROW, COL, M, N, K, A[b * M * K:(b + 1) * M * K], K, B[b * N * K:(b + 1) * N * K], K)
        np.testing.assert_array_equal(C0[b], Cb[0])
    assert np.all(D >= np.abs(C))
    pb, pi, pj = np.meshgrid(np.arange(nb), np.arange(M), np.arange(N), indexing="ij")
    Cp, Dp = oracle.gemm_points(E4M3, ROW, COL, M, N, K, A, K, B, K, pb.ravel(), pi.ravel(), pj.ravel(),
                                batch=nb, stride_a=M * K, stride_b=N * K, scale_a=sa, scale_b=sb)
    np.testing.assert_array_equal(Cp.reshape(nb, M, N), C)
    np.testing.assert_array_equal(Dp.reshape(nb, M, N), D)


def test_padding_is_never_read_and_empty_K(oracle):
    rng = np.random.default_rng(8)
    Al = rng.uniform(-1, 1, (4, 6)).astype(np.float32)
    Bl = rng.uniform(-1, 1, (6, 3)).astype(np.float32)
    ref, _ = _run(oracle, F32, ROW, ROW, Al, Bl)
    A, lda = _store(F32, Al, ROW, ld=11, pad_value=np.nan)
    B, ldb = _store(F32, Bl, ROW, ld=9, pad_value=np.nan)
    C, _ = oracle.gemm(F32, ROW, ROW, 4, 3, 6, A, lda, B, ldb)
    np.testing.assert_array_equal(C[0], ref)
    C, D = oracle.gemm(F32, ROW, ROW, 4, 3, 0, np.zeros(0, np.float32), 1, np.zeros(0, np.float32), 3)
    assert C.shape == (1, 4, 3) and np.all(C == 0) and np.all(D == 0)
    with pytest.raises(ValueError):
        oracle.gemm(F32, ROW, ROW, 4, 3, 6, A, 5, B, ldb)          # lda < K


def test_matches_numpy_fp64_matmul_within_rounding(oracle):
    """Special case that reduces to a library routine: fp64 BLAS on the decoded operands."""
    cfg = gen.CONFIGS["C3_small"]
    inp = gen.make_inputs(cfg, 0)
    C, D = oracle.gemm(cfg.in_dtype, cfg.layout_a, cfg.layout_b, cfg.M, cfg.N, cfg.K, inp.A, inp.lda, inp.B, inp.ldb)
    Av = inp.A.view(np.float16).astype(np.float64).reshape(cfg.M, cfg.K)
    Bv = inp.B.view(np.float16).astype(np.float64).reshape(cfg.K, cfg.N)
    assert np.max(np.abs(C[0] - Av @ Bv) / D[0]) < 1e-13
    assert np.max(np.abs(D[0] - np.abs(Av) @ np.abs(Bv)) / D[0]) < 1e-13


def test_output_rounding_probe_fits_tolerance(oracle):
    """All-ones, K=4097, fp16 output: 4097 is not representable, RNE gives 4096, and the
    normalised error 1/4097 sits well inside the 1e-2 half-precision tolerance."""
    C, D = _run(oracle, F16, ROW, ROW, np.ones((1, 4097), np.float32), np.ones((4097, 1), np.float32))
    stored = np.array([4097.0], np.float32).astype(np.float16).view(np.uint16)
    back = oracle.decode(F16, stored)
    assert back[0] == 4096.0
    assert abs(back[0] - C[0, 0]) / D[0, 0] == pytest.approx(1 / 4097) and 1 / 4097 < 1e-2


def test_bias_term_closed_forms(oracle):
    """With A = 0 the result is the bias alone, exactly, and D = |bias|; with all-ones operands
    C = K + bias[j] exactly; the point form agrees with the full form; the bias is shared by a batch."""
    M, N, K, nb = 5, 7, 9, 2
    bias = (np.arange(N, dtype=np.float32) - 3.0) * 0.25
    zero = np.zeros(nb * M * K, dtype=np.float32)
    ones_a, ones_b = np.ones(nb * M * K, dtype=np.float32), np.ones(nb * K * N, dtype=np.float32)
    C, D = oracle.gemm(oracle.F32, 0, 0, M, N, K, zero, K, ones_b, N, batch=nb, stride_a=M * K, stride_b=K * N, bias=bias)
    assert np.array_equal(C, np.broadcast_to(bias.astype(np.float64), (nb, M, N))) and np.array_equal(D, np.abs(C))
    C, D = oracle.gemm(oracle.F32, 0, 0, M, N, K, ones_a, K, ones_b, N, batch=nb, stride_a=M * K, stride_b=K * N, bias=bias)
    assert np.array_equal(C, K + np.broadcast_to(bias.astype(np.float64), (nb, M, N)))
    assert np.array_equal(D, K + np.abs(np.broadcast_to(bias.astype(np.float64), (nb, M, N))))
    pb, pi, pj = np.array([0, 1, 1]), np.array([0, 4, 2]), np.array([6, 0, 3])
    Cp, Dp = oracle.gemm_points(oracle.F32, 0, 0, M, N, K, ones_a, K, ones_b, N, pb, pi, pj, batch=nb, stride_a=M * K,
                                stride_b=K * N, bias=bias)
    assert np.array_equal(Cp, C[pb, pi, pj]) and np.array_equal(Dp, D[pb, pi, pj])
