"""The pipelined state (K3) in its asynchronous form: slabs travel global -> LDS without registers, three stages
deep, operands kept in storage format in LDS and decoded on read (Table 1 "cp.async + pipeline").

Integer-valued operands with fp32 output must match the CPU oracle bit for bit (every partial sum is an integer
below 2^24 in any order), which pins the stage rotation, the swizzled landing of the direct loads, the in-register
decode of every input type and the edges (rows past M or N come back as zeros from the range check).  A second test
sends every e4m3 code through the kernel's decode.  Where the form's conditions fail the state must say so and run
its register-staged form.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util
from tests.test_exact_gpu import int_inputs, oracle_for

pytestmark = pytest.mark.gpu

ROW, COL = gen.ROW_MAJOR, gen.COL_MAJOR
K3 = gemm.GEMM_K3_PIPELINED
ASYNC = "vec16-direct-to-lds(3 stages)"

CASES = [  # (M, N, slabs of 64 bytes, batch, padding of the leading dimensions in 16-byte units, tile)
    (2048, 2100, 7, 1, 0, 128),      # 16 x 17 tiles of 128: the ring of three stages goes round twice and stops mid-way
    (2050, 2048, 1, 1, 1, 128),      # a single slab (prologue only), a row of tiles with two valid rows
    (1024, 1024, 2, 4, 0, 128),      # two slabs, batched
    (300, 260, 9, 2, 3, 64),         # small problem: 64 x 64 tiles, every edge ragged
    (16, 4100, 12, 1, 0, 64),        # a decode-like shape: one row of tiles, 16 valid rows in 64
    (64, 64, 3, 1, 0, 64),           # one tile, exactly the ring's length
]


def query(inp, out=gen.F32, flags=0):
    c = inp.cfg
    d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, out, c.layout_a, c.layout_b, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=c.batch,
                       stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c, flags=flags)
    return gemm.gemm_query(K3, d)


@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16, gen.F16, gen.E4M3])
@pytest.mark.parametrize("case", CASES, ids=["%dx%dx%dslabs_b%d_pad%d_t%d" % c for c in CASES])
def test_asynchronous_form_is_exact(dtype, case):
    M, N, ns, nb, pad, tile = case
    es = gen.ELEM_BYTES[dtype]
    K = ns * 64 // es
    ld = K + pad * 16 // es
    inp = int_inputs(dtype, M, N, K, ROW, COL, batch=nb, lda=ld, ldb=ld, seed=ns + M, biased=(ns == 9))
    q = query(inp)
    assert q.path == ASYNC and q.violated == 0 and (q.bm, q.bn, q.bk) == (tile, tile, 64 // es) and q.stages == 3, (q.path, q.bm)
    C_ref, _ = oracle_for(inp)
    rc, C, _ = util.run_config(K3, inp)
    assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
    np.testing.assert_array_equal(C[:, :, :N], C_ref)


def test_every_e4m3_code_decodes_as_the_oracle_says():
    """A holds all 254 finite e4m3 codes (0x7F and 0xFF are NaN), B is a 0/1 selection matrix: C[i][j] = A[i][j]."""
    M, N, K = 64, 64, 256
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    A = np.resize(codes, (M, K)).copy()
    A[:, :64] = np.resize(np.roll(codes, 17), (M, 64))
    B = np.zeros((N, K), dtype=np.uint8)            # column-major B: row j holds column j of the K x N matrix
    for j in range(N):
        B[j, (3 * j) % K] = 0x38                    # 1.0 in e4m3
    cfg = gen.Config("codes", M, N, K, gen.E4M3, gen.F32, ROW, COL, "uniform")
    inp = gen.Inputs(cfg, 0, A.reshape(-1), B.reshape(-1), K, K, N, M * K, N * K, M * N, None, None, None)
    assert query(inp).path == ASYNC
    C_ref, _ = oracle.gemm(gen.E4M3, ROW, COL, M, N, K, inp.A, K, inp.B, K)
    rc, C, _ = util.run_config(K3, inp)
    assert rc == gemm.GEMM_OK
    np.testing.assert_array_equal(C[0], C_ref[0])
    assert len(np.unique(C_ref)) > 100              # (the selection really reads many different codes)


@pytest.mark.parametrize("name", ["C2_small", "C4_small", "C5_small"])
def test_generated_workloads_with_scales_and_rounded_output(name):
    """Generated values, per-problem scales (e4m3), two-byte output: the acceptance metric against the oracle."""
    inp = gen.make_inputs(gen.CONFIGS[name], 5)
    c = inp.cfg
    assert query(inp, out=c.out_dtype).path == ASYNC
    C_ref, D = oracle.gemm(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, inp.A, inp.lda, inp.B, inp.ldb, batch=c.batch,
                           stride_a=inp.stride_a, stride_b=inp.stride_b, scale_a=inp.scale_a, scale_b=inp.scale_b, bias=inp.bias)
    rc, C, _ = util.run_config(K3, inp)
    assert rc == gemm.GEMM_OK
    assert util.norm_err(C[:, :, : c.N], C_ref, D) <= util.TOL[c.in_dtype]


def test_where_the_conditions_fail_the_state_says_so_and_runs_its_register_staged_form():
    for (la, lb, K, pad, missing) in [(ROW, ROW, 256, 0, "K_CONTIG_B"), (ROW, COL, 250, 0, "TILE_DIV_K"), (ROW, COL, 256, 1, "LD16_A")]:
        inp = int_inputs(gen.BF16, 300, 200, K, la, lb, lda=K + pad, seed=K)
        q = query(inp)
        assert q.path != ASYNC and missing in gemm.Query.names(q.violated), (q.path, gemm.Query.names(q.violated))
        strict = query(inp, flags=gemm.GEMM_FLAG_STRICT)
        assert strict.status == gemm.GEMM_ERR_PRECONDITION
        C_ref, _ = oracle_for(inp)
        rc, C, _ = util.run_config(K3, inp)
        assert rc == gemm.GEMM_OK
        np.testing.assert_array_equal(C[:, :, :200], C_ref)
    # the vector-load simplification takes the state back to its register-staged form
    inp = int_inputs(gen.BF16, 256, 256, 256, ROW, COL)
    assert query(inp, flags=gemm.GEMM_FLAG_DEOPT_NO_VECTOR).path == "elementwise-masked(-novec)"
