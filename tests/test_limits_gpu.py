"""GEMM calls at the addressing limits the planner states (GPU): leading dimensions at and just past the
fast kernel's 4 MiB rows and the streaming kernel's 2^24 elements, operands and outputs that span more
than 4 GiB, the largest batch count.  Dense seeded operands are placed into zero-filled strided device
buffers; the oracle works on the dense copies.
"""
import numpy as np
import pytest
import torch

from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util
from tests.test_parity_gpu import oracle_for

pytestmark = pytest.mark.gpu

ROW, COL = gen.ROW_MAJOR, gen.COL_MAJOR


def place(arr, rows, cols, ld, es):
    """rows x cols dense raw storage -> device bytes of a rows x ld matrix (the gaps are zero)."""
    raw = torch.from_numpy(np.ascontiguousarray(arr).reshape(-1).view(np.uint8).reshape(rows, cols * es).copy()).cuda()
    buf = torch.zeros(rows * ld * es, dtype=torch.uint8, device="cuda")
    buf.view(rows, ld * es)[:, : cols * es] = raw
    return buf


def run_strided(variant, cfg, seed, lda, ldb, ldc, expect_path=None):
    """cfg is dense (tight leading dimensions, batch 1, A row-major, B column-major)."""
    assert cfg.batch == 1 and cfg.layout_a == ROW and cfg.layout_b == COL
    inp = gen.make_inputs(cfg, seed)
    C_ref, D = oracle_for(inp)
    es, eo = gen.ELEM_BYTES[cfg.in_dtype], util.OUT_BYTES[cfg.out_dtype]
    dA = place(inp.A, cfg.M, cfg.K, lda, es)
    dB = place(inp.B, cfg.N, cfg.K, ldb, es)
    dC = torch.full((cfg.M * ldc * eo,), util.POISON, dtype=torch.uint8, device="cuda")
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, ROW, COL, lda=lda, ldb=ldb, ldc=ldc)
    q = gemm.gemm_query(variant, d, dA, dB, dC)
    if expect_path is not None:
        assert q.path.startswith(expect_path), (q.path, expect_path)
    print(f"[limits] {cfg.name} variant {variant} lda {lda} ldb {ldb} ldc {ldc}: {q.path}", flush=True)
    rc = gemm.gemm_run_ex(variant, d, dA, dB, dC)
    torch.cuda.synchronize()
    assert rc == gemm.GEMM_OK, (gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    rows = dC.view(cfg.M, ldc * eo)
    C = util.decode_out(rows[:, : cfg.N * eo].contiguous().reshape(-1), cfg.out_dtype).reshape(1, cfg.M, cfg.N)
    err = util.norm_err(C, C_ref, D)
    assert err <= util.TOL[cfg.in_dtype], (cfg.name, variant, q.path, err)
    if ldc > cfg.N:   # the gap right of the last column keeps its poison bytes
        gap = rows[:, cfg.N * eo : min(ldc, cfg.N + 16) * eo]
        assert torch.all(gap == util.POISON)
    del dA, dB, dC
    torch.cuda.empty_cache()


def test_rows_of_4_mib_are_the_fast_kernels_limit():
    """bf16, leading dimensions of 2^21 elements: the direct-to-LDS kernel's 32-bit offsets span a 1 GiB tile;
    eight elements more and the planner hands the call to the masked kernel."""
    cfg = gen.Config("ld4MiB", 300, 260, 192, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True)
    run_strided(4, cfg, 31, 1 << 21, 1 << 21, 264, expect_path="mfma32-direct-to-lds")
    run_strided(4, cfg, 31, (1 << 21) + 8, 1 << 21, 264, expect_path="mfma32-vec16-masked")
    run_strided(4, cfg, 31, 1 << 21, (1 << 21) + 8, 264, expect_path="mfma32-vec16-masked")


def test_leading_dimensions_of_2_to_the_24_are_the_streaming_kernels_limit():
    cfg = gen.Config("ld2p24", 16, 40, 264, gen.BF16, gen.BF16, ROW, COL, "normal", std=0.02)
    run_strided(4, cfg, 32, 1 << 24, 1 << 24, 40, expect_path="mfma16-stream")
    cfg64 = gen.Config("ld2p24rows64", 64, 8192, 72, gen.F16, gen.F16, ROW, COL, "normal", std=0.02)
    run_strided(4, cfg64, 33, 1 << 24, 72, 8192, expect_path="mfma16-stream")
    # past the limit the streaming kernel is not offered
    d = gemm.make_desc(16, 40, 264, gen.BF16, gen.BF16, ROW, COL, lda=(1 << 24) + 8, ldb=1 << 24, ldc=40)
    assert "stream" not in gemm.gemm_query(4, d).path


@pytest.mark.parametrize("variant", [0, 2, 4])
def test_output_and_operand_beyond_4_gib(variant):
    """70 000 rows 80 000 bytes apart: C, then A, spans 5.6 GB, so row offsets need 64 bits in every state."""
    cfg = gen.Config("big_c", 70000, 64, 64, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True)
    run_strided(variant, cfg, 34, 64, 64, 40000)
    cfg = gen.Config("big_a", 70000, 64, 128, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True)
    run_strided(variant, cfg, 35, 40000, 128, 64)


def test_largest_batch_count():
    """65 535 problems.  On the streaming kernel (8 rows, or 8 columns and 104 rows) one strip each, every
    problem with operands of its own.  On the direct-to-LDS kernel (K = 64) and on the masked one (K = 40)
    one 104 x 104 tile each; there all problems share one pair of operands (batch strides of zero), so the
    65 535 outputs must equal the first one bit for bit and the first one the oracle."""
    for M, N, K, path in ((8, 8, 40, "mfma16-stream(small-M)"), (104, 8, 40, "mfma16-stream(small-N)")):
        cfg = gen.Config("batch65535", M, N, K, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True, batch=65535)
        inp = gen.make_inputs(cfg, 36)
        d = gemm.make_desc(M, N, K, gen.BF16, gen.BF16, ROW, COL, batch=65535)
        assert gemm.gemm_query(4, d).path.startswith(path)
        C_ref, D = oracle_for(inp)
        rc, C, _ = util.run_config(4, inp)
        assert rc == gemm.GEMM_OK
        assert util.norm_err(C[:, :, :N], C_ref, D) <= util.TOL[gen.BF16]
    M = N = 104
    for K, path in ((64, "mfma32-direct-to-lds"), (40, "mfma32-vec16-masked")):
        cfg = gen.Config("batch65535_shared", M, N, K, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True)
        inp = gen.make_inputs(cfg, 37)
        C_ref, D = oracle_for(inp)
        dA, dB = util.dev(inp.A), util.dev(inp.B)
        dC = torch.full((65535 * M * N * 2,), util.POISON, dtype=torch.uint8, device="cuda")
        d = gemm.make_desc(M, N, K, gen.BF16, gen.BF16, ROW, COL, batch=65535, stride_a=0, stride_b=0)
        assert gemm.gemm_query(4, d, dA, dB, dC).path == path
        assert gemm.gemm_run_ex(4, d, dA, dB, dC) == gemm.GEMM_OK
        torch.cuda.synchronize()
        items = dC.view(65535, M * N * 2)
        assert bool((items == items[0]).all())
        first = util.decode_out(items[0].contiguous(), gen.BF16).reshape(1, M, N)
        assert util.norm_err(first, C_ref, D) <= util.TOL[gen.BF16]
        del dC
        torch.cuda.empty_cache()
    d = gemm.make_desc(8, 8, 64, gen.BF16, gen.BF16, ROW, COL, batch=65536)
    assert gemm.gemm_query(4, d).status == gemm.GEMM_ERR_BAD_ARG


def test_gather_with_activations_just_below_2_gib():
    """The implicit-GEMM state addresses the activations with 32-bit byte offsets and needs them below
    2^31 bytes: 255 images of 256 x 256 x 64 fp16 are 2 139 095 040 bytes.  Every image is the same seeded
    one, so the oracle evaluates sampled outputs (all images, image corners included) on a single image."""
    import oracle
    from paper_2605_28213_amd import conv
    N, H, C, F = 255, 256, 64, 64
    one = gen.make_conv_inputs(gen.ConvConfig("below2GiB", 1, H, H, C, F, 3, 3, gen.F16, gen.F16), 41)
    img = util.dev(one.x)
    dx = img.repeat(N)
    assert dx.numel() == N * H * H * C * 2 < 1 << 31
    dw = util.dev(one.w)
    dy = torch.full((N * H * H * F * 2,), util.POISON, dtype=torch.uint8, device="cuda")
    d = conv.make_desc(N, H, H, C, F, 3, 3, gen.F16, gen.F16, stride=(1, 1), pad=(1, 1))
    q = conv.conv2d_query(conv.CONV_C2_IMPLICIT_MFMA, d, dx, dw, dy)
    assert q.status == gemm.GEMM_OK and q.violated == 0, q
    rc = conv.conv2d_run(conv.CONV_C2_IMPLICIT_MFMA, d, dx, dw, dy)
    torch.cuda.synchronize()
    assert rc == gemm.GEMM_OK, conv.conv2d_last_launch_error()
    rng = np.random.default_rng(7)
    npts = 4000
    pn = rng.integers(0, N, npts); pn[:200] = N - 1; pn[200:300] = 0
    pp = rng.integers(0, H, npts); pq = rng.integers(0, H, npts); pf = rng.integers(0, F, npts)
    pp[:50], pq[:50] = H - 1, H - 1                        # the last pixel of the last image: the largest offsets
    pp[50:100], pq[50:100] = 0, 0
    y_ref, D = oracle.conv2d_points(gen.F16, one.x, one.w, np.zeros(npts, dtype=np.int64), pp, pq, pf, stride=(1, 1), pad=(1, 1))
    idx = torch.from_numpy((((pn * H + pp) * H + pq) * F + pf).astype(np.int64)).cuda()
    got = dy.view(torch.int16)[idx].cpu().numpy().view(np.float16).astype(np.float64)
    assert util.norm_err(got, y_ref, D) <= util.TOL[gen.F16]
    # one image more and the state is refused
    d = conv.make_desc(N + 1, H, H, C, F, 3, 3, gen.F16, gen.F16, stride=(1, 1), pad=(1, 1))
    q = conv.conv2d_query(conv.CONV_C2_IMPLICIT_MFMA, d)
    assert q.status == gemm.GEMM_ERR_PRECONDITION and conv.Query.names(q.violated) == ["X_BELOW_2GIB"]


def test_radix_select_on_rows_of_five_million():
    """Rows far beyond what the oracle's rank count can walk: the selection is checked against its
    definition (the k largest, ties at the threshold to the lower indices, indices increasing, values
    bit for bit), which holds at any size.  Values are standard normal rounded to multiples of 1/1024, so
    thousands of elements tie at the threshold; the second row sits ld - n elements after the first."""
    from paper_2605_28213_amd import topk
    n, k, ld = 5_000_003, 100_000, 5_000_008
    x = np.zeros((2, ld), np.float32)
    x[:, :n] = np.round(gen.normal(43, 0, 2 * n, 1.0).reshape(2, n) * 1024) / 1024
    x[:, n:] = 99.0                                          # past the row: must never be selected
    dx = torch.from_numpy(x.reshape(-1)).cuda()
    didx = torch.full((2 * k,), -7, dtype=torch.int32, device="cuda")
    dval = torch.full((2 * k,), -7.0, dtype=torch.float32, device="cuda")
    d = topk.make_desc(2, n, k, ld=ld)
    for refused in (topk.TOPK_T0_SELECTION, topk.TOPK_T2_RESIDENT):
        assert topk.topk_query(refused, d, dx).status == gemm.GEMM_ERR_PRECONDITION
    rc = topk.topk_run(topk.TOPK_T1_RADIX_SELECT, d, dx, didx, dval)
    torch.cuda.synchronize()
    assert rc == gemm.GEMM_OK, topk.topk_last_launch_error()
    idx, val = didx.cpu().numpy().reshape(2, k), dval.cpu().numpy().reshape(2, k)
    for b in range(2):
        row = x[b, :n]
        assert np.all(np.diff(idx[b]) > 0) and idx[b][0] >= 0 and idx[b][-1] < n
        np.testing.assert_array_equal(val[b].view(np.uint32), row[idx[b]].view(np.uint32))
        t = val[b].min()
        chosen = np.zeros(n, bool)
        chosen[idx[b]] = True
        assert np.all(row[~chosen] <= t) and np.all(chosen[row > t])
        at = np.flatnonzero(row == t)                        # the tie at the threshold goes to the lower indices
        taken = chosen[at]
        assert taken.sum() == k - int((row > t).sum()) and np.all(taken[: taken.sum()]) and not np.any(taken[taken.sum():])
