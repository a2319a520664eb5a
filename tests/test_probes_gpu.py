"""The measurement probes: argument checks and one small launch each (their results are rates, read by bench.py)."""
import pytest
import torch

from paper_2605_28213_amd import gemm

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("probe,per_iter", [(gemm.gemm_probe_mfma, 32 * 2.0 * 32 * 32 * 16), (gemm.gemm_probe_mfma16, 128 * 2.0 * 16 * 16 * 32)])
def test_matrix_pipe_probes_run_and_report_their_flops(probe, per_iter):
    wgs, iters = 8, 3
    need = gemm.gemm_probe_mfma_operand_bytes(gemm.GEMM_BF16, wgs)
    assert need == wgs * 256 * 16 * 16                  # 16 chunks of 16 bytes per lane; the 16x16x32 loop holds twice that
    if probe is gemm.gemm_probe_mfma16:
        need *= 2
    ops = torch.ones(need // 2, dtype=torch.bfloat16, device="cuda")
    sink = torch.full((wgs * 256,), -1.0, dtype=torch.float32, device="cuda")
    rc, flops = probe(gemm.GEMM_BF16, ops, need, wgs, iters, sink, sink.numel() * 4)
    torch.cuda.synchronize()
    assert rc == gemm.GEMM_OK and flops == wgs * 4 * iters * per_iter
    # all-ones operands: every accumulator element is the number of k it summed; the sink holds a lane's sum of them
    assert torch.all(sink > 0) and torch.all(sink == sink[0])
    assert probe(gemm.GEMM_BF16, ops, need - 16, wgs, iters, sink, sink.numel() * 4)[0] == gemm.GEMM_ERR_BAD_ARG
    assert probe(gemm.GEMM_BF16, ops, need, wgs, 0, sink, sink.numel() * 4)[0] == gemm.GEMM_ERR_BAD_ARG
    assert probe(gemm.GEMM_F32, ops, need, wgs, iters, sink, sink.numel() * 4)[0] == gemm.GEMM_ERR_UNSUPPORTED_DTYPE


def test_16x16_probe_is_for_two_byte_types_only():
    ops = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")      # (1 workgroup needs 128 KB)
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    assert gemm.gemm_probe_mfma16(gemm.GEMM_FP8_E4M3, ops, ops.numel(), 1, 1, sink, 1024)[0] == gemm.GEMM_ERR_UNSUPPORTED_DTYPE
