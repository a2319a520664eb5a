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
    """65 535 problems: one workgroup tile each on the direct-to-LDS kernel (K = 64) and on the masked one
    (K = 40) with 72 rows, one strip each on the streaming kernel with 8 rows."""
    for M, K, path in ((72, 64, "mfma32-direct-to-lds"), (72, 40, "mfma32-"), (8, 40, "mfma16-stream")):
        cfg = gen.Config("batch65535", M, 8, K, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True, batch=65535)
        inp = gen.make_inputs(cfg, 36)
        d = gemm.make_desc(M, 8, K, gen.BF16, gen.BF16, ROW, COL, batch=65535)
        assert gemm.gemm_query(4, d).path.startswith(path)
        C_ref, D = oracle_for(inp)
        rc, C, _ = util.run_config(4, inp)
        assert rc == gemm.GEMM_OK
        assert util.norm_err(C[:, :, :8], C_ref, D) <= util.TOL[gen.BF16]
    d = gemm.make_desc(8, 8, 64, gen.BF16, gen.BF16, ROW, COL, batch=65536)
    assert gemm.gemm_query(4, d).status == gemm.GEMM_ERR_BAD_ARG
