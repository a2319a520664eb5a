"""Seeded random GEMM calls against the oracle (GPU): shapes, layouts, leading dimensions, batch,
scales, bias, output types and scratch lending drawn at random inside the documented limits, so that
combinations no hand-written case names still get run.  The draw is fixed by its seed; every case runs
K4 (whatever path its planner picks) and one earlier state.
"""
import numpy as np
import pytest

from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util
from tests.test_parity_gpu import oracle_for

pytestmark = pytest.mark.gpu

ROW, COL = gen.ROW_MAJOR, gen.COL_MAJOR


def draw_case(rng, i):
    dtype = int(rng.choice([gen.F32, gen.BF16, gen.F16, gen.E4M3], p=[0.1, 0.35, 0.3, 0.25]))
    kind = rng.choice(["ragged", "aligned", "small_m", "thin_tail", "tiny"], p=[0.3, 0.3, 0.2, 0.1, 0.1])
    la, lb = int(rng.choice([ROW, COL])), int(rng.choice([ROW, COL]))
    batch = int(rng.choice([1, 1, 2, 3]))
    if kind == "small_m":
        M, N, K = int(rng.integers(1, 17)), int(rng.choice([40, 500, 8200])), int(rng.integers(1, 40)) * 8
        la, lb = ROW, COL
    elif kind == "thin_tail":
        M, N, K = 256 * int(rng.integers(1, 3)) + int(rng.integers(1, 17)), int(rng.integers(100, 400)), int(rng.integers(60, 300))
    elif kind == "tiny":
        M, N, K = (int(rng.integers(0, 9)) for _ in range(3))
    else:
        M, N, K = int(rng.integers(1, 600)), int(rng.integers(1, 600)), int(rng.integers(1, 700))
    es = gen.ELEM_BYTES[dtype]
    if kind in ("aligned", "small_m"):
        K = max(128 // es, K // (128 // es) * (128 // es)) if kind == "aligned" else K
        la, lb = (ROW, COL) if rng.random() < 0.7 else (la, lb)
        pad = lambda n: (n + 15) // 16 * 16
    else:
        pad = lambda n: n + int(rng.integers(0, 5))
    out = int(rng.choice({gen.F32: [gen.F32], gen.BF16: [gen.BF16, gen.F32], gen.F16: [gen.F16, gen.F32], gen.E4M3: [gen.BF16, gen.F32]}[dtype]))
    cfg = gen.Config(f"fuzz{i}", M, N, K, dtype, out, la, lb, str(rng.choice(["uniform", "normal"])),
                     batch=batch, scaled=bool(rng.random() < 0.3), biased=bool(rng.random() < 0.3),
                     lda=max(1, pad(K if la == ROW else M)), ldb=max(1, pad(N if lb == ROW else K)), ldc=max(1, pad(N)))
    return cfg, bool(rng.random() < 0.6)


CASES = [draw_case(np.random.default_rng(1000 + i), i) for i in range(48)]


@pytest.mark.parametrize("i", range(len(CASES)))
def test_random_case(i):
    cfg, lend = CASES[i]
    inp = gen.make_inputs(cfg, 100 + i)
    C_ref, D = oracle_for(inp)
    rng = np.random.default_rng(i)
    variants = [gemm.GEMM_K4_MFMA, int(rng.integers(0, 4))]
    for v in variants:
        rc, C, _ = util.run_config(v, inp, lend_workspace=lend)
        q = gemm.gemm_query(v, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b,
                                              lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch))
        assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_variant_name(v), gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
        if cfg.M * cfg.N == 0:
            continue
        err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
        assert err <= util.TOL[cfg.in_dtype], (cfg, gemm.gemm_variant_name(v), q.path, err)


def draw_rows_case(rng, i):
    """17..96 rows on the streaming kernel: few wide strips per problem, enough problems to pass its rule."""
    dtype = int(rng.choice([gen.BF16, gen.F16, gen.E4M3]))
    M = int(rng.integers(17, 97))
    cols = 32 if M <= 32 else 64
    strips = int(rng.integers(1, 7))
    batch = -(-128 // strips) + int(rng.integers(0, 4))
    N = cols * (strips - 1) + int(rng.integers(1, cols + 1))
    K = 16 * int(rng.integers(1, 100))
    pad = lambda n: n + 16 * int(rng.integers(0, 4))
    out = int(rng.choice([gen.BF16 if dtype == gen.E4M3 else dtype, gen.F32]))
    return gen.Config(f"rows{i}", M, N, K, dtype, out, ROW, COL, str(rng.choice(["uniform", "normal"])), batch=batch,
                      scaled=bool(rng.random() < 0.3), biased=bool(rng.random() < 0.3), lda=pad(K), ldb=pad(K), ldc=N + int(rng.integers(0, 5)))


ROWS_CASES = [draw_rows_case(np.random.default_rng(2000 + i), i) for i in range(24)]


def draw_cols_case(rng, i):
    """Few columns on the streaming kernel's transposed form: the rows case with M and N exchanged."""
    c = draw_rows_case(rng, i)
    n = int(rng.integers(1, 97))
    cols = 16 if n <= 16 else 32 if n <= 32 else 64
    strips = int(rng.integers(1, 7))
    batch = 1 if n <= 16 and rng.random() < 0.5 else -(-128 // strips) + int(rng.integers(0, 3))
    M = max(97, cols * (strips - 1) + int(rng.integers(1, cols + 1)))       # more rows than the row forms take
    return gen.Config(f"cols{i}", M, n, c.K, c.in_dtype, c.out_dtype, ROW, COL, c.dist, batch=batch, scaled=c.scaled, biased=c.biased,
                      lda=c.ld[0], ldb=c.ld[1], ldc=n + int(rng.integers(0, 5)))


def draw_long_k_few_tiles_case(rng, i):
    """At most 256 tiles of 128 x 128 and K of 32 to 70 slabs, aligned operands, B column-major, 128-tiles asked for:
    the nine-region ring of the small-tile kernel (first slab, trips of nine, tails of every length)."""
    dtype = int(rng.choice([gen.BF16, gen.F16, gen.E4M3]))
    es = gen.ELEM_BYTES[dtype]
    batch = int(rng.choice([1, 1, 2, 3]))
    tm, tn = int(rng.integers(1, 7)), int(rng.integers(1, 7))
    M = 128 * (tm - 1) + int(rng.integers(97, 129))
    N = 128 * (tn - 1) + int(rng.integers(97, 129))
    K = 128 // es * int(rng.integers(32, 71))
    lda = K + 16 // es * int(rng.integers(0, 3))
    ldb = K + 16 // es * int(rng.integers(0, 3))
    out = int(rng.choice([gen.BF16 if dtype == gen.E4M3 else dtype, gen.F32]))
    return gen.Config(f"deep{i}", M, N, K, dtype, out, ROW, COL, str(rng.choice(["uniform", "normal"])), batch=batch,
                      scaled=bool(rng.random() < 0.3), biased=bool(rng.random() < 0.3), lda=lda, ldb=ldb, ldc=N + int(rng.integers(0, 3)))


DEEP_CASES = [draw_long_k_few_tiles_case(np.random.default_rng(8000 + i), i) for i in range(16)]


@pytest.mark.parametrize("i", range(len(DEEP_CASES)))
def test_random_case_for_the_nine_region_ring(i):
    cfg = DEEP_CASES[i]
    inp = gen.make_inputs(cfg, 800 + i)
    C_ref, D = oracle_for(inp)
    q = gemm.gemm_query(4, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, COL, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc,
                                          batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c,
                                          flags=gemm.GEMM_FLAG_TILE_128))
    assert (q.path, q.bm, q.stages) == ("mfma32-direct-to-lds", 128, 4), (cfg, q)
    rc, C, _ = util.run_config(4, inp, flags=gemm.GEMM_FLAG_TILE_128)
    assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg, err)


COLS_CASES = [draw_cols_case(np.random.default_rng(2500 + i), i) for i in range(24)]


def draw_many_tiles_case(rng, i):
    """At least 256 tiles of 256 x 256 with a short K: the persistent forms of the tiled kernel.  B column-major with
    aligned operands and whole slabs (all three types), or A and B row-major with anything (bf16, fp16: read in place)."""
    row_major_b = bool(rng.random() < 0.5)
    dtype = int(rng.choice([gen.BF16, gen.F16] if row_major_b else [gen.BF16, gen.F16, gen.E4M3]))
    es = gen.ELEM_BYTES[dtype]
    tm, tn = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    batch = -(-256 // (tm * tn)) + int(rng.integers(0, 3))
    M = 256 * (tm - 1) + int(rng.integers(97, 257))        # (more than 96 rows and columns: not the streaming kernel's)
    N = 256 * (tn - 1) + int(rng.integers(97, 257))
    if row_major_b:
        K = int(rng.integers(2 * 128 // es + 1, 6 * 128 // es))
        lda, ldb = K + int(rng.integers(0, 4)), N + int(rng.integers(0, 4))
    else:
        K = 128 // es * int(rng.integers(3, 8))
        lda = ldb = K + 16 // es * int(rng.integers(0, 3))
    out = int(rng.choice([gen.BF16 if dtype == gen.E4M3 else dtype, gen.F32]))
    return gen.Config(f"tiles{i}", M, N, K, dtype, out, ROW, ROW if row_major_b else COL, str(rng.choice(["uniform", "normal"])),
                      batch=batch, scaled=bool(rng.random() < 0.3), biased=bool(rng.random() < 0.3), lda=lda, ldb=ldb,
                      ldc=N + int(rng.integers(0, 3)))


TILES_CASES = [draw_many_tiles_case(np.random.default_rng(3000 + i), i) for i in range(24)]


@pytest.mark.parametrize("i", range(len(TILES_CASES)))
def test_random_case_with_many_tiles(i):
    cfg = TILES_CASES[i]
    inp = gen.make_inputs(cfg, 300 + i)
    C_ref, D = oracle_for(inp)
    q = gemm.gemm_query(4, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, cfg.layout_b, lda=inp.lda, ldb=inp.ldb,
                                          ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c))
    if cfg.layout_b == ROW:
        assert q.path in ("mfma32-direct-to-lds(persistent,B-row-major)", "mfma32-direct-to-lds(persistent,B-row-major)+thin(M-tail)") and q.grid == 256, (cfg, q)
    else:   # (the tile rule may prefer 128-tiles, which have no persistent form)
        assert q.path in ("mfma32-direct-to-lds(persistent)", "mfma32-direct-to-lds"), (cfg, q)
    rc, C, _ = util.run_config(4, inp)
    assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg, err)


@pytest.mark.parametrize("i", range(len(COLS_CASES)))
def test_random_case_with_few_columns(i):
    cfg = COLS_CASES[i]
    inp = gen.make_inputs(cfg, 250 + i)
    C_ref, D = oracle_for(inp)
    q = gemm.gemm_query(4, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, COL, lda=inp.lda, ldb=inp.ldb,
                                          ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c))
    assert q.path == "mfma16-stream(small-N)", (cfg, q)
    rc, C, _ = util.run_config(4, inp)
    assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg, err)


@pytest.mark.parametrize("i", range(len(ROWS_CASES)))
def test_random_case_with_17_to_96_rows(i):
    cfg = ROWS_CASES[i]
    inp = gen.make_inputs(cfg, 200 + i)
    C_ref, D = oracle_for(inp)
    q = gemm.gemm_query(4, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, COL, lda=inp.lda, ldb=inp.ldb,
                                          ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c))
    assert q.path == "mfma16-stream(small-M)", (cfg, q)
    rc, C, _ = util.run_config(4, inp)
    assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg, err)


def draw_conv_case(rng, i):
    """A random layer inside the documented limits: image and filter sizes, strides and paddings drawn
    independently per axis, channel counts that are whole 128-byte slabs (every state) or not (C0, C1)."""
    dtype = int(rng.choice([gen.F16, gen.BF16, gen.E4M3]))
    es = gen.ELEM_BYTES[dtype]
    slab = 128 // es
    C = int(rng.choice([slab, 2 * slab, slab, int(rng.integers(1, 40))]))
    R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    pad = (int(rng.integers(0, R)), int(rng.integers(0, S)))
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    H = int(rng.integers(max(1, R - 2 * pad[0]), 24)) + 1
    W = int(rng.integers(max(1, S - 2 * pad[1]), 24)) + 1
    out = int(rng.choice([gen.BF16 if dtype == gen.E4M3 else dtype, gen.F32]))
    return gen.ConvConfig(f"convfuzz{i}", int(rng.integers(1, 4)), H, W, C, int(rng.integers(1, 200)), R, S, dtype, out,
                          stride=stride, pad=pad, biased=bool(rng.random() < 0.4))


CONV_CASES = [draw_conv_case(np.random.default_rng(3000 + i), i) for i in range(24)]


@pytest.mark.parametrize("i", range(len(CONV_CASES)))
def test_random_convolution_layer(i):
    from paper_2605_28213_amd import conv
    from tests.test_conv_gpu import reference, run_state
    cfg = CONV_CASES[i]
    inp = gen.make_conv_inputs(cfg, 300 + i)
    y_ref, D = reference(inp)
    whole = (cfg.C * gen.ELEM_BYTES[cfg.in_dtype]) % 128 == 0
    for variant in range(3):
        rc, y, q, _ = run_state(variant, inp)
        if variant == 2 and not whole:
            assert rc == gemm.GEMM_ERR_PRECONDITION, (cfg, q)
            continue
        assert rc == gemm.GEMM_OK, (cfg, variant, gemm.gemm_status_string(rc), conv.conv2d_last_launch_error(), q)
        err = util.norm_err(y, y_ref, D)
        assert err <= util.TOL[cfg.in_dtype], (cfg, variant, q.path, err)


def draw_topk_case(rng, i):
    """Row length, k, leading dimension and value distribution at random: normal, heavily tied (multiples of
    1/4), or a handful of distinct values; k from 0 to n."""
    n = int(rng.choice([int(rng.integers(1, 300)), int(rng.integers(300, 5000)), int(rng.integers(5000, 17000))]))
    k = int(rng.choice([0, 1, n, int(rng.integers(0, n + 1)), max(1, n // 8)]))
    batch = int(rng.integers(1, 6))
    # mostly a multiple of 4 (the resident state loads 16 bytes per lane and refuses other rows), sometimes not
    ld = (n + 3) // 4 * 4 + 4 * int(rng.choice([0, 0, 1])) if rng.random() < 0.7 else n + int(rng.choice([0, 7]))
    kind = str(rng.choice(["normal", "quarters", "few"]))
    return batch, n, k, ld, kind


TOPK_CASES = [draw_topk_case(np.random.default_rng(4000 + i), i) for i in range(24)]


@pytest.mark.parametrize("i", range(len(TOPK_CASES)))
def test_random_selection(i):
    import oracle
    from paper_2605_28213_amd import topk
    from tests.test_topk_gpu import run_state
    batch, n, k, ld, kind = TOPK_CASES[i]
    v = gen.normal(400 + i, 0, batch * ld, 1.0).reshape(batch, ld)
    if kind == "quarters":
        v = np.round(v * 4) / 4
    elif kind == "few":
        v = np.round(v)                                      # about seven distinct values, both zeros among them
    x = v.astype(np.float32)
    ridx, rval = oracle.topk(x[:, :n], k)
    for variant in range(3):
        q = topk.topk_query(variant, topk.make_desc(batch, n, k, ld=ld))
        rc, idx, val, _ = run_state(variant, x, n, k)
        if q.status != gemm.GEMM_OK:
            assert rc == q.status == gemm.GEMM_ERR_PRECONDITION, (TOPK_CASES[i], variant, q)
            continue
        assert rc == gemm.GEMM_OK, (TOPK_CASES[i], variant, topk.topk_last_launch_error())
        np.testing.assert_array_equal(idx, ridx)
        np.testing.assert_array_equal(val.view(np.uint32), rval.view(np.uint32))


def draw_thin_case(rng, i):
    """At most 64 rows with both operands row-major (two-byte types): the thin kernel, as a product of its own or,
    for the second half of the family, as the remainder of a product the persistent kernel reads in place."""
    dtype = int(rng.choice([gen.BF16, gen.F16]))
    rows = int(rng.integers(1, 65))
    if i % 2 == 0:
        M, N, K, batch = rows, int(rng.integers(1, 3000)), int(rng.integers(1, 2500)), int(rng.choice([1, 1, 2, 5]))
    else:       # whole rounds of 256-tiles plus a thin remainder that would cost one more
        tn = int(rng.integers(1, 5))
        batch = 256 // tn // 2 + int(rng.integers(0, 2))
        M, N, K = 512 + rows, 256 * (tn - 1) + int(rng.integers(97, 257)), int(rng.integers(130, 400))
    out = int(rng.choice([dtype, gen.F32]))
    return gen.Config(f"thin{i}", M, N, K, dtype, out, ROW, ROW, str(rng.choice(["uniform", "normal"])), batch=batch,
                      scaled=bool(rng.random() < 0.3), biased=bool(rng.random() < 0.3), lda=K + int(rng.integers(0, 4)),
                      ldb=N + int(rng.integers(0, 4)), ldc=N + int(rng.integers(0, 3)))


THIN_CASES = [draw_thin_case(np.random.default_rng(4000 + i), i) for i in range(24)]


@pytest.mark.parametrize("i", range(len(THIN_CASES)))
def test_random_case_for_the_thin_kernel(i):
    cfg = THIN_CASES[i]
    inp = gen.make_inputs(cfg, 400 + i)
    C_ref, D = oracle_for(inp)
    q = gemm.gemm_query(4, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, ROW, lda=inp.lda, ldb=inp.ldb,
                                          ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c))
    if i % 2 == 0:
        assert q.path == "mfma16-thin(B-row-major)", (cfg, q.path)
    else:       # (the remainder is split off only where it saves a round of tiles; either way B is read in place)
        assert q.path.startswith("mfma32-direct-to-lds(persistent,B-row-major)"), (cfg, q.path)
    rc, C, _ = util.run_config(4, inp)
    assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg, err)


def draw_pipelined_case(rng, i):
    """K3 on operands its asynchronous form takes (K contiguous in both, rows 16-byte aligned, K whole 64-byte slabs):
    every input type, both tile sizes, ragged M and N, padded leading dimensions, batch, scales, bias."""
    dtype = int(rng.choice([gen.F32, gen.BF16, gen.F16, gen.E4M3]))
    es = gen.ELEM_BYTES[dtype]
    K = 64 // es * int(rng.integers(1, 14))
    big = bool(rng.random() < 0.4)          # at least 256 tiles of 128 x 128: the large-tile form
    if big:
        M, N, batch = int(rng.integers(1500, 2300)), int(rng.integers(1900, 2300)), 1
    else:
        M, N, batch = int(rng.integers(1, 500)), int(rng.integers(1, 500)), int(rng.choice([1, 2, 3]))
    ld = K + 16 // es * int(rng.integers(0, 3))
    out = int(rng.choice({gen.F32: [gen.F32], gen.BF16: [gen.BF16, gen.F32], gen.F16: [gen.F16, gen.F32], gen.E4M3: [gen.BF16, gen.F32]}[dtype]))
    return gen.Config(f"pipe{i}", M, N, K, dtype, out, ROW, COL, str(rng.choice(["uniform", "normal"])), batch=batch,
                      scaled=bool(rng.random() < 0.3), biased=bool(rng.random() < 0.3), lda=ld, ldb=ld, ldc=N + int(rng.integers(0, 3)))


PIPE_CASES = [draw_pipelined_case(np.random.default_rng(5000 + i), i) for i in range(24)]


@pytest.mark.parametrize("i", range(len(PIPE_CASES)))
def test_random_case_for_the_pipelined_state(i):
    cfg = PIPE_CASES[i]
    inp = gen.make_inputs(cfg, 500 + i)
    C_ref, D = oracle_for(inp)
    q = gemm.gemm_query(3, gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, COL, lda=inp.lda, ldb=inp.ldb,
                                          ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c))
    # (a batch stride that is not a multiple of 16 bytes breaks the alignment condition: then the register-staged form runs)
    aligned = cfg.batch == 1 or ((cfg.M * inp.lda * gen.ELEM_BYTES[cfg.in_dtype]) % 16 == 0 and (cfg.N * inp.ldb * gen.ELEM_BYTES[cfg.in_dtype]) % 16 == 0)
    assert (q.path == "vec16-direct-to-lds(3 stages)") == aligned, (cfg, q.path)
    rc, C, _ = util.run_config(3, inp)
    assert rc == gemm.GEMM_OK, (cfg, gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    err = util.norm_err(C[:, :, : cfg.N], C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg, err)
