"""gemm_run_static, the entry point that allocates nothing: its results against gemm_run_ex with lent scratch.

Both entry points run the same kernels, so their outputs must be equal byte for byte.  Each case makes
two calls in a row on the library's fixed scratch array, the second with a smaller input (the array
then still holds the first call's contents), on K4's split-K form (fp32 partial products in scratch) and
on its packed path (operand copies in scratch); one case also checks the result against the CPU oracle.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util

pytestmark = pytest.mark.gpu

ROW, COL = gen.ROW_MAJOR, gen.COL_MAJOR
K4 = gemm.GEMM_K4_MFMA


def both_ways(cfg, seed, expect_in_path):
    """Returns (raw output of gemm_run_static, raw output of gemm_run_ex with lent scratch, inputs)."""
    inp = gen.make_inputs(cfg, seed)
    dA, dB = util.dev(inp.A), util.dev(inp.B)
    bias = torch.from_numpy(inp.bias).cuda() if inp.bias is not None else None
    kw = dict(lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
              stride_c=inp.stride_c, bias=bias)
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, **kw)
    need = gemm.gemm_query(K4, d, dA, dB).workspace_bytes
    assert 0 < need <= gemm.gemm_static_scratch_bytes(), need
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    lent = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, workspace=ws,
                          workspace_bytes=need, **kw)
    assert expect_in_path in gemm.gemm_query(K4, lent, dA, dB).path
    C_static = util.out_buffer(cfg.batch * inp.stride_c, cfg.out_dtype)
    C_lent = util.out_buffer(cfg.batch * inp.stride_c, cfg.out_dtype)
    torch.cuda.synchronize()
    rc = gemm.gemm_run_static(K4, d, dA, dB, C_static)
    assert rc == gemm.GEMM_OK, (gemm.gemm_status_string(rc), gemm.gemm_last_launch_error())
    assert gemm.gemm_run_ex(K4, lent, dA, dB, C_lent) == gemm.GEMM_OK
    torch.cuda.synchronize()
    return C_static, C_lent, inp


def test_split_k_on_the_static_scratch_twice_the_second_call_smaller():
    big = gen.Config("static_splitk_big", 128, 4096, 8192, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True, biased=True)
    small = gen.Config("static_splitk_small", 100, 300, 4096, gen.BF16, gen.BF16, ROW, COL, "normal", rsqrt_k=True)
    for cfg, seed in ((big, 0), (small, 1)):
        got, want, inp = both_ways(cfg, seed, "splitK")
        assert torch.equal(got, want), cfg.name
    # the second (smaller) call against the oracle as well
    C_ref, D = oracle.gemm(small.in_dtype, ROW, COL, small.M, small.N, small.K, inp.A, inp.lda, inp.B, inp.ldb)
    C = util.decode_out(got, small.out_dtype)[: small.M * small.N].reshape(1, small.M, small.N)
    assert util.norm_err(C, C_ref, D) <= util.TOL[small.in_dtype]


def test_packed_path_on_the_static_scratch_twice_the_second_call_smaller():
    big = gen.Config("static_packed_big", 1500, 1203, 1999, gen.F16, gen.F16, ROW, ROW, "uniform", lda=2001, ldb=1205, ldc=1207)
    small = gen.Config("static_packed_small", 300, 270, 203, gen.E4M3, gen.BF16, COL, ROW, "uniform", batch=2, lda=303, ldb=275)
    for cfg, seed in ((big, 2), (small, 3)):
        got, want, inp = both_ways(cfg, seed, "packed")
        assert torch.equal(got, want), cfg.name
        C_ref, D = oracle.gemm(cfg.in_dtype, cfg.layout_a, cfg.layout_b, cfg.M, cfg.N, cfg.K, inp.A, inp.lda, inp.B, inp.ldb,
                               batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b)
        C = util.decode_out(got, cfg.out_dtype)[: cfg.batch * inp.stride_c].reshape(cfg.batch, cfg.M, inp.ldc)[:, :, : cfg.N]
        assert util.norm_err(C, C_ref, D) <= util.TOL[cfg.in_dtype]


def test_paths_without_scratch_run_as_in_gemm_run_ex_and_every_state_is_accepted():
    inp = gen.make_inputs(gen.CONFIGS["C2_small"], 0)
    c = inp.cfg
    dA, dB = util.dev(inp.A), util.dev(inp.B)
    d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, c.layout_a, c.layout_b)
    for v in range(gemm.GEMM_VARIANT_COUNT):
        a, b = util.out_buffer(c.M * c.N, c.out_dtype), util.out_buffer(c.M * c.N, c.out_dtype)
        assert gemm.gemm_run_static(v, d, dA, dB, a) == gemm.GEMM_OK
        assert gemm.gemm_run_ex(v, d, dA, dB, b) == gemm.GEMM_OK
        torch.cuda.synchronize()
        assert torch.equal(a, b)


def test_requests_beyond_the_array_and_lent_workspaces_are_refused():
    # the ragged fp16 workload's sizes with A column-major (no kernel reads that in place): the packed copies take
    # 68 MB, more than the array
    cfg = gen.CONFIGS["C3"]
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, COL, cfg.layout_b)
    assert gemm.gemm_query(K4, d).workspace_bytes > gemm.gemm_static_scratch_bytes()
    es = gen.ELEM_BYTES[cfg.in_dtype]
    dA = torch.zeros(cfg.M * cfg.K * es, dtype=torch.uint8, device="cuda")
    dB = torch.zeros(cfg.K * cfg.N * es, dtype=torch.uint8, device="cuda")
    dC = util.out_buffer(cfg.M * cfg.N, cfg.out_dtype)
    assert gemm.gemm_run_static(K4, d, dA, dB, dC) == gemm.GEMM_ERR_WORKSPACE
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    small = gemm.make_desc(64, 64, 64, gen.BF16, gen.BF16, ROW, COL, workspace=ws, workspace_bytes=1 << 20)
    assert gemm.gemm_run_static(K4, small, dA, dB, dC) == gemm.GEMM_ERR_BAD_ARG
    torch.cuda.synchronize()
    assert torch.all(dC == util.POISON), "a refused call must leave C untouched"
