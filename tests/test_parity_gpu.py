"""GPU parity: every lineage variant against the CPU oracle, element by element, through the C ABI.

Sizes here are ones the oracle finishes in seconds while still spanning several workgroup tiles of
every variant (the largest tile is 256 x 256 x 128 B of K) and ending in ragged tails.  Full-size
workloads are covered by tests/test_gate_gpu.py.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util

pytestmark = pytest.mark.gpu

VARIANTS = list(range(gemm.GEMM_VARIANT_COUNT))
ROW, COL = gen.ROW_MAJOR, gen.COL_MAJOR


def variants_for(dtype):
    return list(VARIANTS)


def oracle_for(inp):
    c = inp.cfg
    return oracle.gemm(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, inp.A, inp.lda, inp.B, inp.ldb,
                       batch=c.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
                       scale_a=inp.scale_a, scale_b=inp.scale_b, bias=inp.bias)


def check(variant, inp, ref=None, out_dtype=None, lend_workspace=False):
    c = inp.cfg
    C_ref, D = ref if ref is not None else oracle_for(inp)
    rc, C, _ = util.run_config(variant, inp, out_dtype=out_dtype, lend_workspace=lend_workspace)
    assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
    err = util.norm_err(C[:, :, : c.N], C_ref, D)
    assert err <= util.TOL[c.in_dtype], f"{gemm.gemm_variant_name(variant)} on {c.name}: normalised error {err:.3e}"
    return err


@pytest.mark.parametrize("name", ["C1", "C2_small", "C3_small", "C4_small", "C5_small"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_small_workloads_three_seeds(name, seed):
    """The five workload families at reduced size (C1 is already small), all variants, seeds 0..2."""
    cfg = gen.CONFIGS[name]
    inp = gen.make_inputs(cfg, seed)
    ref = oracle_for(inp)
    for v in variants_for(cfg.in_dtype):
        check(v, inp, ref)


@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16, gen.F16, gen.E4M3])
@pytest.mark.parametrize("la,lb", [(ROW, ROW), (ROW, COL), (COL, ROW), (COL, COL)])
@pytest.mark.parametrize("aligned", [True, False])
def test_all_layouts_ragged_multi_tile(dtype, la, lb, aligned):
    """M, N, K cross tile edges of every variant with a tail; leading dimensions either padded to a
    16-byte multiple (fast paths) or tight and odd (masked paths)."""
    M, N, K = 300, 270, 203
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    pad = (lambda n: (n + 15) // 16 * 16) if aligned else (lambda n: n)
    cfg = gen.Config("ragged", M, N, K, dtype, out, la, lb, "uniform",
                     lda=pad(K if la == ROW else M), ldb=pad(N if lb == ROW else K), ldc=pad(N))
    inp = gen.make_inputs(cfg, 11)
    ref = oracle_for(inp)
    for v in variants_for(dtype):
        q = gemm.gemm_query(v, gemm.make_desc(M, N, K, dtype, out, la, lb, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc))
        if v >= 2 and aligned and not (v == 4 and (la != ROW or lb != COL)):
            assert "elementwise" not in q.path
        if v >= 2 and not aligned and dtype != gen.E4M3:
            assert "elementwise" in q.path
        check(v, inp, ref)


@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16, gen.F16, gen.E4M3])
def test_integer_inputs_give_bitwise_exact_fp32_output(dtype):
    """Entries in {-2..2}, K <= 4096: every partial sum is an integer below 2^24, so any correct
    fp32-accumulating kernel equals the exact product bit for bit, whatever its summation order."""
    rng = np.random.default_rng(5)
    M, N, K = 259, 130, 1000
    la, lb = ROW, COL
    A = gen.quantise(dtype, rng.integers(-2, 3, M * K).astype(np.float32))
    B = gen.quantise(dtype, rng.integers(-2, 3, N * K).astype(np.float32))
    cfg = gen.Config("ints", M, N, K, dtype, gen.F32, la, lb, "uniform")
    inp = gen.Inputs(cfg, 0, A, B, K, K, N, M * K, N * K, M * N)
    C_ref, D = oracle_for(inp)
    for v in variants_for(dtype):
        rc, C, _ = util.run_config(v, inp)
        assert rc == gemm.GEMM_OK
        np.testing.assert_array_equal(C, C_ref, err_msg=gemm.gemm_variant_name(v))


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (1, 7, 5), (16, 33, 64), (17, 16, 8), (5, 3, 0), (2, 600, 9), (33, 1, 4100)])
@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16, gen.E4M3])
def test_degenerate_shapes(M, N, K, dtype):
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    for la, lb in [(ROW, ROW), (ROW, COL)]:
        cfg = gen.Config("tiny", M, N, K, dtype, out, la, lb, "uniform")
        inp = gen.make_inputs(cfg, 3)
        ref = oracle_for(inp)
        for v in variants_for(dtype):
            check(v, inp, ref)
            if K == 0:
                rc, C, _ = util.run_config(v, inp)
                assert np.all(C == 0)


def test_skinny_path_edges():
    """The small-M streaming path: M below 16, N not a multiple of its column block, K a multiple of
    16 bytes only, all three types, fp32 output."""
    for dtype in (gen.BF16, gen.F16, gen.E4M3):
        out = gen.BF16 if dtype == gen.E4M3 else dtype
        cases = [(16, 512, 1024), (7, 100, 144), (1, 33, 16), (16, 2049, 4112)] if dtype == gen.E4M3 else \
                [(16, 512, 1024), (7, 100, 136), (1, 33, 8), (16, 2049, 4104)]
        for (M, N, K) in cases:
            cfg = gen.Config("skinny", M, N, K, dtype, out, ROW, COL, "normal", std=0.02 if dtype != gen.E4M3 else 1.0)
            inp = gen.make_inputs(cfg, 4)
            d = gemm.make_desc(M, N, K, dtype, out, ROW, COL)
            assert gemm.gemm_query(4, d).path.startswith("mfma16-stream")
            check(4, inp)
            check(4, inp, out_dtype=gen.F32)
    # batched, with a ragged last K tile in every wave's share of K and padded leading dimensions
    cfg = gen.Config("skinny_batched", 13, 75, 1320, gen.BF16, gen.BF16, ROW, COL, "normal", std=0.02, batch=3,
                     lda=1328, ldb=1336, ldc=80)
    inp = gen.make_inputs(cfg, 5)
    check(4, inp)


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
def test_streaming_path_with_17_to_96_rows(dtype):
    """Two to six groups of 16 rows of A per workgroup: every group boundary, a ragged last group, a
    ragged last strip of columns, a ragged last K tile for every wave, batches, padded leading dimensions,
    scales and bias; and the rule that hands such a product to the tiled kernel when its strips are few."""
    cases = [(17, 4100, 520, {}), (32, 4096, 1024, {}), (33, 8200, 264, {}), (47, 520, 1160, dict(batch=16, scaled=True)),
             (48, 8192, 128, dict(biased=True)), (49, 8256, 392, {}), (64, 8192, 2048, {}), (65, 8200, 392, {}),
             (81, 530, 1160, dict(batch=16, scaled=True, biased=True)), (96, 8192, 1024, {}),
             (20, 130, 1320, dict(batch=32, lda=1328, ldb=1336, ldc=136)), (64, 70, 776, dict(batch=70, scaled=True))]
    for (M, N, K, kw) in cases:
        out = gen.BF16 if dtype == gen.E4M3 else dtype
        if dtype == gen.E4M3:
            K = (K + 15) // 16 * 16
            kw = {k_: (v_ + 15) // 16 * 16 if k_ in ("lda", "ldb") else v_ for k_, v_ in kw.items()}
        cfg = gen.Config("rows", M, N, K, dtype, out, ROW, COL, "normal", std=0.02 if dtype != gen.E4M3 else 1.0, **kw)
        inp = gen.make_inputs(cfg, 6)
        d = gemm.make_desc(M, N, K, dtype, out, ROW, COL, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch,
                           stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c)
        q = gemm.gemm_query(4, d)
        assert q.path == "mfma16-stream(small-M)" and q.bm == (16 * ((M + 15) // 16) if M <= 64 else 96) and q.bn == (32 if M <= 32 else 64), (M, N, K, q)
        ref = oracle_for(inp)
        check(4, inp, ref)
        check(4, inp, ref, out_dtype=gen.F32)
    # too few strips for the chip: the tiled kernel keeps the product
    for (M, N) in ((17, 4064), (64, 8128), (33, 4096), (96, 8128), (97, 16384)):
        assert gemm.gemm_query(4, gemm.make_desc(M, N, 1024, dtype, out, ROW, COL)).path.startswith("mfma32-direct-to-lds")


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
def test_streaming_path_with_few_columns(dtype):
    """Up to 64 columns and many rows: the streaming kernel multiplies the transposed product (B's columns as
    its rows, strips along M) and writes C transposed back; bias per column of C, scales, ragged strips,
    ragged K tiles, padded leading dimensions, batches, fp32 output."""
    cases = [(200, 16, 1024, {}), (4100, 7, 136, dict(biased=True)), (300, 1, 8, {}), (4100, 17, 520, dict(biased=True)),
             (8200, 33, 264, {}), (8192, 64, 2048, dict(biased=True, ldc=72)), (530, 48, 1160, dict(batch=16, scaled=True, biased=True)),
             (8200, 80, 392, dict(biased=True)),
             (70, 16, 1320, dict(batch=3, lda=1328, ldb=1336, ldc=24))]
    for (M, N, K, kw) in cases:
        out = gen.BF16 if dtype == gen.E4M3 else dtype
        if dtype == gen.E4M3:
            K = (K + 15) // 16 * 16
            kw = {k_: (v_ + 15) // 16 * 16 if k_ in ("lda", "ldb") else v_ for k_, v_ in kw.items()}
        cfg = gen.Config("cols", M, N, K, dtype, out, ROW, COL, "normal", std=0.02 if dtype != gen.E4M3 else 1.0, **kw)
        inp = gen.make_inputs(cfg, 13)
        d = gemm.make_desc(M, N, K, dtype, out, ROW, COL, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch,
                           stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c)
        q = gemm.gemm_query(4, d)
        assert q.path == "mfma16-stream(small-N)" and q.bn == (16 * ((N + 15) // 16) if N <= 64 else 96), (M, N, K, q)
        ref = oracle_for(inp)
        check(4, inp, ref)
        check(4, inp, ref, out_dtype=gen.F32)
    # 17..64 columns and too few strips along M for the chip: the tiled kernel keeps the product
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    for (M, N) in ((4064, 17), (8128, 64)):
        assert gemm.gemm_query(4, gemm.make_desc(M, N, 1024, dtype, out, ROW, COL)).path.startswith("mfma32-direct-to-lds")


def test_batched_strides_scales_and_padding_untouched():
    """Batch strides larger than the matrices, ldc > N: the gaps keep their poison bytes."""
    M, N, K, nb = 70, 50, 96, 3
    cfg = gen.Config("batched", M, N, K, gen.E4M3, gen.BF16, ROW, COL, "normal", batch=nb, scaled=True,
                     lda=K + 16, ldb=K + 32, ldc=N + 6)
    inp = gen.make_inputs(cfg, 9)
    inp.scale_a[1] = -1.5                                   # a negative scale must carry its sign
    ref = oracle_for(inp)
    for v in VARIANTS:
        rc, C, raw = util.run_config(v, inp)
        assert rc == gemm.GEMM_OK
        assert util.norm_err(C[:, :, :N], ref[0], ref[1]) <= util.TOL[gen.E4M3]
        pad = raw.cpu().numpy().view(np.uint16)[: nb * inp.stride_c].reshape(nb, M, inp.ldc)[:, :, N:]
        assert np.all(pad == 0xFFFF), "bytes between rows of C were overwritten"


def test_refusal_leaves_C_untouched_and_is_not_a_fallback():
    """A variant asked to run outside its preconditions in strict mode returns an error and writes
    nothing (it must not quietly run something else)."""
    inp = gen.make_inputs(gen.CONFIGS["C3_small"], 0)
    for v in (2, 3, 4):
        rc, _, raw = util.run_config(v, inp, flags=gemm.GEMM_FLAG_STRICT)
        assert rc == gemm.GEMM_ERR_PRECONDITION
        assert torch.all(raw == util.POISON)


def test_success_overwrites_every_output_and_is_deterministic():
    inp = gen.make_inputs(gen.CONFIGS["C2_small"], 1)
    for v in VARIANTS:
        rc, C1, raw1 = util.run_config(v, inp)
        rc2, C2, raw2 = util.run_config(v, inp)
        assert rc == rc2 == gemm.GEMM_OK
        assert np.all(np.isfinite(C1))                       # no poison left anywhere
        assert torch.equal(raw1, raw2)                       # no atomics: run-to-run bitwise equal


def test_gemm_run_short_form_uses_default_layouts():
    M, N, K = 96, 80, 72
    for dtype, lb in [(gen.F32, ROW), (gen.F16, ROW), (gen.BF16, COL), (gen.E4M3, COL)]:
        out = gen.BF16 if dtype == gen.E4M3 else dtype
        cfg = gen.Config("short", M, N, K, dtype, out, ROW, lb, "uniform")
        inp = gen.make_inputs(cfg, 2)
        C_ref, D = oracle_for(inp)
        dA, dB = util.dev(inp.A), util.dev(inp.B)
        for v in variants_for(dtype):
            dC = util.out_buffer(M * N, out)
            assert gemm.gemm_run(v, M, N, K, dtype, dA, dB, dC) == gemm.GEMM_OK
            torch.cuda.synchronize()
            C = util.decode_out(dC, out).reshape(1, M, N)
            assert util.norm_err(C, C_ref, D) <= util.TOL[dtype]


def test_launch_on_a_side_stream():
    inp = gen.make_inputs(gen.CONFIGS["C2_small"], 0)
    c = inp.cfg
    C_ref, D = oracle_for(inp)
    s = torch.cuda.Stream()
    dA, dB = util.dev(inp.A), util.dev(inp.B)
    dC = util.out_buffer(c.M * c.N, c.out_dtype)
    torch.cuda.synchronize()
    d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, c.layout_a, c.layout_b, stream=s)
    assert gemm.gemm_run_ex(4, d, dA, dB, dC) == gemm.GEMM_OK
    s.synchronize()
    C = util.decode_out(dC, c.out_dtype).reshape(1, c.M, c.N)
    assert util.norm_err(C, C_ref, D) <= util.TOL[c.in_dtype]


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
@pytest.mark.parametrize("la,lb,tag", [(ROW, ROW, "(B)"), (COL, COL, "(A)"), (COL, ROW, "")])
def test_packed_path_leaves_a_conforming_operand_in_place(dtype, la, lb, tag):
    """Aligned operands and K in whole slabs, but K strided in one or both operands: only the operand that
    breaks the fast kernel's conditions is packed; the scratch asked for covers that operand alone."""
    M, N, K, nb = 392, 264, 384, 2
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    es = gen.ELEM_BYTES[dtype]
    cfg = gen.Config("halfpacked", M, N, K, dtype, out, la, lb, "normal", rsqrt_k=True, batch=nb, biased=True)
    inp = gen.make_inputs(cfg, 12)
    d = gemm.make_desc(M, N, K, dtype, out, la, lb, batch=nb)
    q = gemm.gemm_query(4, d)
    rows = {"(B)": N, "(A)": M, "": M + N}[tag]
    assert q.workspace_bytes == nb * rows * K * es and "packed" not in q.path
    d.workspace, d.workspace_bytes = 256, q.workspace_bytes
    assert gemm.gemm_query(4, d).path == "mfma32-packed%s+direct-to-lds" % tag
    check(4, inp, lend_workspace=True)
    check(4, inp, out_dtype=gen.F32, lend_workspace=True)


def test_host_threads_and_streams_side_by_side():
    """The library keeps no state between calls (the launch-error slot is per thread): four host threads,
    each on a stream of its own, launch different paths of K4 and an earlier state at the same time, many
    times over, into buffers of their own; every result must equal the one the same call gives alone."""
    import threading
    jobs = []
    for name, variant, lend in (("C2_small", 4, False), ("C4_small", 4, False), ("C3_small", 4, True), ("C5_small", 2, False)):
        inp = gen.make_inputs(gen.CONFIGS[name], 1)
        c = inp.cfg
        dA, dB = util.dev(inp.A), util.dev(inp.B)
        sa = torch.from_numpy(inp.scale_a).cuda() if inp.scale_a is not None else None
        sb = torch.from_numpy(inp.scale_b).cuda() if inp.scale_b is not None else None
        stream = torch.cuda.Stream()
        kw = dict(lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=c.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
                  stride_c=inp.stride_c, scale_a=sa, scale_b=sb)
        d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, c.layout_a, c.layout_b, stream=stream, **kw)
        ws = None
        if lend:
            need = gemm.gemm_query(variant, d, dA, dB).workspace_bytes
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            d.workspace, d.workspace_bytes = ws.data_ptr(), need
        alone = util.out_buffer(c.batch * inp.stride_c, c.out_dtype)
        assert gemm.gemm_run_ex(variant, d, dA, dB, alone) == gemm.GEMM_OK
        stream.synchronize()
        outs = [util.out_buffer(c.batch * inp.stride_c, c.out_dtype) for _ in range(3)]
        jobs.append(dict(variant=variant, d=d, dA=dA, dB=dB, alone=alone, outs=outs, stream=stream, keep=(sa, sb, ws), rcs=[]))
    torch.cuda.synchronize()

    def work(j):
        for i in range(60):
            j["rcs"].append(gemm.gemm_run_ex(j["variant"], j["d"], j["dA"], j["dB"], j["outs"][i % 3]))

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for j in jobs:
        assert all(rc == gemm.GEMM_OK for rc in j["rcs"]) and len(j["rcs"]) == 60
        for o in j["outs"]:
            assert torch.equal(o, j["alone"])


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
@pytest.mark.parametrize("la,lb", [(ROW, ROW), (ROW, COL), (COL, ROW), (COL, COL)])
def test_packed_path_with_lent_workspace(dtype, la, lb):
    """K4 with scratch lent: operands that violate the fast path's conditions (odd leading dimensions,
    K strided, ragged K) are packed and multiplied by the fast kernel; the query names that path."""
    M, N, K = 300, 270, 203
    cfg = gen.Config("packed", M, N, K, dtype, gen.BF16 if dtype == gen.E4M3 else dtype, la, lb, "uniform", batch=2,
                     lda=(K if la == ROW else M) + 3, ldb=(N if lb == ROW else K) + 5, ldc=N + 1)
    inp = gen.make_inputs(cfg, 11)
    ref = oracle_for(inp)
    d = gemm.make_desc(M, N, K, dtype, cfg.out_dtype, la, lb, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=2)
    q = gemm.gemm_query(4, d)
    assert q.workspace_bytes > 0 and q.path.startswith("mfma32-") and "packed" not in q.path
    d.workspace, d.workspace_bytes = 256, q.workspace_bytes          # any non-null address: query only
    assert gemm.gemm_query(4, d).path.startswith("mfma32-packed+direct-to-lds")
    check(4, inp, ref, lend_workspace=True)
    check(4, inp, ref, out_dtype=gen.F32, lend_workspace=True)
    check(4, inp, ref)                                               # and the masked path without scratch


def test_lent_workspace_too_small_or_misaligned_is_refused():
    cfg = gen.CONFIGS["C3_small"]
    inp = gen.make_inputs(cfg, 0)
    dA, dB = util.dev(inp.A), util.dev(inp.B)
    dC = util.out_buffer(cfg.M * inp.ldc, cfg.out_dtype)
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b)
    need = gemm.gemm_query(4, d).workspace_bytes
    ws = torch.empty(need + 32, dtype=torch.uint8, device="cuda")
    before = dC.clone()
    d.workspace, d.workspace_bytes = ws.data_ptr(), need - 1
    assert gemm.gemm_run_ex(4, d, dA, dB, dC) == gemm.GEMM_ERR_WORKSPACE
    d.workspace, d.workspace_bytes = ws.data_ptr() + 2, need
    assert gemm.gemm_run_ex(4, d, dA, dB, dC) == gemm.GEMM_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.equal(before, dC), "a refused call must leave C untouched"


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
@pytest.mark.parametrize("rem", [3, 16, 17, 48, 64, 65])
def test_thin_row_remainder_goes_to_the_streaming_kernel(dtype, rem):
    """M a few rows past 16 whole rows of 256-tiles, 16 tile columns: the seventeenth row of tiles would be
    a second round of the chip, so a remainder of up to 64 rows is multiplied by the streaming kernel
    instead (all of its row-group forms); both parts must agree with the oracle, in the aligned fast path
    and in the packed path.  A remainder whose tiles fit the round that runs anyway stays with the tiles."""
    M, N, K = 4096 + rem, 4096, 256
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    cfg = gen.Config("mtail", M, N, K, dtype, out, ROW, COL, "normal", rsqrt_k=True)
    inp = gen.make_inputs(cfg, 6)
    ref = oracle_for(inp)
    d = gemm.make_desc(M, N, K, dtype, out, ROW, COL)
    # (at least 256 whole tiles; K = 256 elements is 4 slabs for the two-byte types, which the persistent form of the
    # tiled kernel takes, and 2 slabs for e4m3, which it does not)
    form = "" if dtype == gen.E4M3 else "(persistent)"
    assert gemm.gemm_query(4, d).path == "mfma32-direct-to-lds" + form + ("+stream(M-tail)" if rem <= 64 else "")
    check(4, inp, ref)
    if rem in (3, 48):
        ragged = gen.Config("mtail_packed", M, N, K - 5, dtype, out, ROW, ROW, "normal", rsqrt_k=True, biased=True)
        rinp = gen.make_inputs(ragged, 7)
        need = gemm.gemm_query(4, gemm.make_desc(M, N, K - 5, dtype, out, ROW, ROW)).workspace_bytes
        lent = gemm.make_desc(M, N, K - 5, dtype, out, ROW, ROW, workspace=256, workspace_bytes=need)
        # (two-byte types with both operands row-major are read in place, the remainder by the thin kernel, scratch or
        # not; e4m3 has no such form and is packed)
        assert gemm.gemm_query(4, lent).path == ("mfma32-packed+direct-to-lds+stream(M-tail)" if dtype == gen.E4M3 else
                                                 "mfma32-direct-to-lds(persistent,B-row-major)+thin(M-tail)")
        check(4, rinp, lend_workspace=True)
    # 2 x 2 tiles per problem: one round with or without the remainder
    small = gemm.make_desc(256 + rem, 300, K, dtype, out, ROW, COL, batch=2)
    assert "M-tail" not in gemm.gemm_query(4, small).path
    scfg = gen.Config("mtail_small", 256 + rem, 300, K, dtype, out, ROW, COL, "normal", rsqrt_k=True, batch=2)
    check(4, gen.make_inputs(scfg, 8))


@pytest.mark.parametrize("flags", [gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE, gemm.GEMM_FLAG_DEOPT_NO_OVERLAP,
                                   gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE | gemm.GEMM_FLAG_DEOPT_NO_OVERLAP])
@pytest.mark.parametrize("dtype", [gen.BF16, gen.E4M3])
def test_simplified_expert_states_compute_the_same_product(flags, dtype):
    """The validated simplifications of the fast kernel (no LDS swizzle, no load/MFMA overlap) on a ragged
    multi-tile shape with enough slabs to go round the LDS ring."""
    M, N, K = 300, 520, 1024
    cfg = gen.Config("deopt", M, N, K, dtype, gen.BF16, ROW, COL, "normal", rsqrt_k=True, batch=2)
    inp = gen.make_inputs(cfg, 12)
    c = inp.cfg
    C_ref, D = oracle_for(inp)
    rc, C, _ = util.run_config(4, inp, flags=flags)
    assert rc == gemm.GEMM_OK
    assert util.norm_err(C[:, :, :N], C_ref, D) <= util.TOL[dtype]


@pytest.mark.parametrize("tile_flag", [gemm.GEMM_FLAG_TILE_256, gemm.GEMM_FLAG_TILE_128])
@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
def test_both_tile_configurations_on_ragged_shapes(tile_flag, dtype):
    """The fast kernel with 256- and with 128-tiles forced, on shapes whose M and N end inside a tile
    (rows past the end come from outside the buffer resource), with a batch, both output types, and
    with K long enough to go round the LDS ring and to leave it through the tail loop."""
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    for (M, N, K, nb) in [(300, 520, 1024, 2), (257, 129, 896, 1), (100, 700, 128, 3)]:
        cfg = gen.Config("tiles", M, N, K, dtype, out, ROW, COL, "normal", rsqrt_k=True, batch=nb)
        inp = gen.make_inputs(cfg, 13)
        C_ref, D = oracle_for(inp)
        for od in (out, gen.F32):
            rc, C, _ = util.run_config(4, inp, flags=tile_flag, out_dtype=od)
            assert rc == gemm.GEMM_OK
            assert util.norm_err(C[:, :, :N], C_ref, D) <= util.TOL[dtype], (M, N, K, nb, od)
    d = gemm.make_desc(300, 520, 1024, dtype, out, ROW, COL, flags=tile_flag)
    assert gemm.gemm_query(4, d).bm == (256 if tile_flag == gemm.GEMM_FLAG_TILE_256 else 128)


@pytest.mark.parametrize("tile_flag", [0, gemm.GEMM_FLAG_TILE_256, gemm.GEMM_FLAG_TILE_128])
def test_row_major_tile_walk_computes_the_same_product(tile_flag):
    """GEMM_FLAG_DEOPT_NO_RASTER: a different order of the same tiles, with either tile size, batched and ragged."""
    for dtype, (M, N, K, nb) in ((gen.BF16, (700, 520, 512, 3)), (gen.E4M3, (257, 1100, 256, 2)), (gen.F16, (1024, 768, 128, 1))):
        out = gen.BF16 if dtype == gen.E4M3 else dtype
        cfg = gen.Config("walk", M, N, K, dtype, out, ROW, COL, "normal", rsqrt_k=True, batch=nb)
        inp = gen.make_inputs(cfg, 17)
        C_ref, D = oracle_for(inp)
        flags = tile_flag | gemm.GEMM_FLAG_DEOPT_NO_RASTER
        rc, C, _ = util.run_config(4, inp, flags=flags)
        assert rc == gemm.GEMM_OK
        assert util.norm_err(C[:, :, :N], C_ref, D) <= util.TOL[dtype], (dtype, M, N, K, nb)
        q = gemm.gemm_query(4, gemm.make_desc(M, N, K, dtype, out, ROW, COL, batch=nb, flags=flags))
        assert q.path.endswith("-noraster")


@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16, gen.F16, gen.E4M3])
@pytest.mark.parametrize("la,lb", [(ROW, ROW), (ROW, COL), (COL, COL)])
def test_vector_loads_removed_from_k2_and_k3(dtype, la, lb):
    """GEMM_FLAG_DEOPT_NO_VECTOR: both states fetch element by element and still compute the product, on
    aligned operands (where they would otherwise use 16-byte loads), large and small tile forms."""
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    for (M, N, K) in ((300, 272, 208), (2100, 2064, 64)):
        cfg = gen.Config("novec", M, N, K, dtype, out, la, lb, "uniform", lda=(K if la == ROW else M) + 16 - (K if la == ROW else M) % 16,
                         ldb=(N if lb == ROW else K) + 16 - (N if lb == ROW else K) % 16)
        inp = gen.make_inputs(cfg, 19)
        C_ref, D = oracle_for(inp)
        for v in (gemm.GEMM_K2_VECTORIZED, gemm.GEMM_K3_PIPELINED):
            rc, C, _ = util.run_config(v, inp, flags=gemm.GEMM_FLAG_DEOPT_NO_VECTOR)
            assert rc == gemm.GEMM_OK
            assert util.norm_err(C[:, :, :N], C_ref, D) <= util.TOL[dtype], (v, dtype, M, N, K)
    rc, _, raw = util.run_config(gemm.GEMM_K1_LDS_TILED, inp, flags=gemm.GEMM_FLAG_DEOPT_NO_VECTOR)
    assert rc == gemm.GEMM_ERR_BAD_ARG and torch.all(raw == util.POISON)


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
def test_split_k_with_lent_scratch(dtype):
    """Few tiles and a long K: with scratch lent, K4 cuts K into ranges that run side by side and adds the
    fp32 partial products in a second pass (scale, bias and the single rounding happen there)."""
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    es = gen.ELEM_BYTES[dtype]
    for (M, N, nslab, kw) in ((100, 300, 64, dict(biased=True)), (33, 130, 48, dict(scaled=True)), (200, 257, 32, {}), (64, 1024, 128, dict(ldc=1032))):
        K = nslab * 128 // es
        cfg = gen.Config("splitk", M, N, K, dtype, out, ROW, COL, "normal", rsqrt_k=True, **kw)
        inp = gen.make_inputs(cfg, 23)
        ref = oracle_for(inp)
        d = gemm.make_desc(M, N, K, dtype, out, ROW, COL, ldc=inp.ldc)
        q = gemm.gemm_query(4, d)
        assert q.workspace_bytes > 0 and "splitK" not in q.path             # offered, not taken without scratch
        check(4, inp, ref)                                                  # the unsplit kernel
        d.workspace, d.workspace_bytes = 4096, q.workspace_bytes
        assert "splitK" in gemm.gemm_query(4, d).path
        check(4, inp, ref, lend_workspace=True)
        check(4, inp, ref, out_dtype=gen.F32, lend_workspace=True)
    # the scratch must be big enough
    dA, dB = util.dev(inp.A), util.dev(inp.B)
    dC = util.out_buffer(inp.stride_c, out)
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, dtype, out, ROW, COL, ldc=inp.ldc, workspace=ws, workspace_bytes=4096)
    assert gemm.gemm_run_ex(4, d, dA, dB, dC) == gemm.GEMM_ERR_WORKSPACE and torch.all(dC == util.POISON)


def test_launches_are_capturable_and_replayable_in_a_hip_graph():
    """The library allocates nothing and only launches kernels on the given stream, so a sequence of
    calls can be captured into a HIP graph.  Three different states and shapes are captured once and
    replayed several times with eager work in between; every replay must reproduce the eager result
    bit for bit."""
    stream = torch.cuda.Stream()
    jobs = []
    for variant, name in ((gemm.GEMM_K4_MFMA, "C2_small"), (gemm.GEMM_K4_MFMA, "C4_small"), (gemm.GEMM_K1_LDS_TILED, "C1")):
        cfg = gen.CONFIGS[name]
        inp = gen.make_inputs(cfg, 5)
        dA, dB = util.dev(inp.A), util.dev(inp.B)
        dC = util.out_buffer(cfg.batch * inp.stride_c, cfg.out_dtype)
        d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, lda=inp.lda,
                           ldb=inp.ldb, ldc=inp.ldc, stream=stream)
        jobs.append((variant, d, dA, dB, dC))
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        for variant, d, dA, dB, dC in jobs:
            assert gemm.gemm_run_ex(variant, d, dA, dB, dC) == gemm.GEMM_OK
    stream.synchronize()
    eager = [dC.clone() for *_, dC in jobs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for variant, d, dA, dB, dC in jobs:
            assert gemm.gemm_run_ex(variant, d, dA, dB, dC) == gemm.GEMM_OK
    for replay in range(3):
        for *_, dC in jobs:
            dC.fill_(0xFF)                                   # eager work between replays (a fill kernel)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for want, (*_, dC) in zip(eager, jobs):
            assert torch.equal(want, dC), f"replay {replay} differs from the eager result"


@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16, gen.F16, gen.E4M3])
def test_bias_is_added_before_the_rounding_in_every_state(dtype):
    """AddMM: C = round(s * A.B + bias[j]).  Every state, ragged multi-tile shapes in the aligned and
    in the masked / packed paths, a batch (the bias is shared), the streaming path, both tile sizes."""
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    shapes = [(300, 270, 256, 2, ROW, COL, 0), (130, 70, 203, 1, ROW, ROW, 3), (9, 100, 264, 2, ROW, COL, 0)]
    for (M, N, K, nb, la, lb, pad) in shapes:
        cfg = gen.Config("addmm", M, N, K, dtype, out, la, lb, "normal", rsqrt_k=True, batch=nb, scaled=dtype == gen.E4M3,
                         biased=True, lda=(K if la == ROW else M) + pad, ldb=(N if lb == ROW else K) + pad, ldc=N + pad)
        inp = gen.make_inputs(cfg, 21)
        ref = oracle_for(inp)
        assert np.max(np.abs(ref[0])) > 1.0                         # the bias dominates: a dropped bias cannot pass
        for v in variants_for(dtype):
            check(v, inp, ref)
        if dtype != gen.F32:
            check(4, inp, ref, lend_workspace=True)
            if la == ROW and lb == COL and pad == 0 and M > 16:
                for flag in (gemm.GEMM_FLAG_TILE_256, gemm.GEMM_FLAG_TILE_128):
                    rc, C, _ = util.run_config(4, inp, flags=flag)
                    assert rc == gemm.GEMM_OK and util.norm_err(C[:, :, :N], ref[0], ref[1]) <= util.TOL[dtype]


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16, gen.E4M3])
def test_persistent_form_of_the_tiled_kernel(dtype):
    """At least 256 tiles of 256 x 256 and 3..64 slabs of K: one workgroup per CU walks several tiles with the LDS
    ring running across the tile boundaries.  Ragged edges in M and N (masked epilogue beside the unmasked one),
    per-problem scales, a bias, both output types, workgroups with unequal numbers of tiles."""
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    es = gen.ELEM_BYTES[dtype]
    for (M, N, ns, nb, kw) in [(700, 520, 5, 29, dict(scaled=True, biased=True)), (512, 300, 3, 70, {}), (1100, 1030, 9, 11, dict(biased=True))]:
        K = ns * 128 // es
        cfg = gen.Config("ring", M, N, K, dtype, out, ROW, COL, "normal", rsqrt_k=True, batch=nb, **kw)
        inp = gen.make_inputs(cfg, 31)
        if inp.scale_a is not None:
            inp.scale_a[1] = -0.75
        d = gemm.make_desc(M, N, K, dtype, out, ROW, COL, batch=nb, flags=gemm.GEMM_FLAG_TILE_256)
        q = gemm.gemm_query(4, d)
        assert q.path == "mfma32-direct-to-lds(persistent)" and q.grid == 256, q
        ref = oracle_for(inp)
        for od in (out, gen.F32):
            rc, C, _ = util.run_config(4, inp, flags=gemm.GEMM_FLAG_TILE_256, out_dtype=od)
            assert rc == gemm.GEMM_OK
            assert util.norm_err(C[:, :, :N], ref[0], ref[1]) <= util.TOL[dtype], (M, N, K, nb, od)
    # fewer tiles than workgroups, or fewer than three slabs: the one-tile-per-workgroup kernel keeps the product
    assert gemm.gemm_query(4, gemm.make_desc(700, 520, 5 * 128 // es, dtype, out, ROW, COL, batch=20, flags=gemm.GEMM_FLAG_TILE_256)).path == "mfma32-direct-to-lds"
    assert gemm.gemm_query(4, gemm.make_desc(700, 520, 2 * 128 // es, dtype, out, ROW, COL, batch=29, flags=gemm.GEMM_FLAG_TILE_256)).path == "mfma32-direct-to-lds"
