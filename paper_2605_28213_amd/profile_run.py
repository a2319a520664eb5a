"""Launches one lineage state on one workload a few times, for a profiler to watch.

The gate's profile leg (paper Sec. 3.1; Sec. 3.3: profile deltas feed the skill record) takes hardware
counters from rocprofv3, which must start the measured program itself, with the program directly after
`--` and one counter group per run:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -o fetch -- python3 -m paper_2605_28213_amd.profile_run --variant 4 --workload C2
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d DIR -o write -- python3 -m paper_2605_28213_amd.profile_run --variant 4 --workload C2
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_LDS_BANK_CONFLICT SQ_INSTS_LDS SQ_INSTS_VALU SQ_INSTS_VMEM_RD SQ_WAIT_INST_ANY \\
              --output-format csv -d DIR -o sq -- python3 -m paper_2605_28213_amd.profile_run --variant 4 --workload C2

`gate.read_counters(DIR, patterns)` then averages each counter over the dispatches of the state's
kernels.  Besides the state, the program launches the copy probe once (256 MiB read, 256 MiB written):
the known size that calibrates the byte counters in the same file.  No result is checked here (the
gate's correctness leg does that); inputs are the workload's seeded synthetic operands.
"""
from __future__ import annotations

import argparse


def main() -> None:
    import numpy as np
    import torch

    from . import gate, gemm
    from . import inputs as gen

    ap = argparse.ArgumentParser()
    ap.add_argument("--variant", type=int, required=True)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--launches", type=int, default=5)
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--no-workspace", action="store_true")
    args = ap.parse_args()
    cfg = gen.CONFIGS[args.workload]
    inp = gen.make_inputs(cfg, 0)
    stream = torch.cuda.Stream()
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a).reshape(-1).view(np.uint8)).cuda()
    sets = [(up(inp.A), up(inp.B), torch.empty(max(1, cfg.batch * inp.stride_c) * 4, dtype=torch.uint8, device="cuda"))
            for _ in range(gate.OPERAND_SETS)]
    sa = torch.from_numpy(inp.scale_a).cuda() if inp.scale_a is not None else None
    sb = torch.from_numpy(inp.scale_b).cuda() if inp.scale_b is not None else None
    bias = torch.from_numpy(inp.bias).cuda() if inp.bias is not None else None
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, lda=inp.lda, ldb=inp.ldb,
                       ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c,
                       scale_a=sa, scale_b=sb, bias=bias, stream=stream, flags=args.flags)
    ws = None
    if not args.no_workspace:
        need = gemm.gemm_query(args.variant, d, *sets[0]).workspace_bytes
        if need:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            d.workspace, d.workspace_bytes = ws.data_ptr(), need
    q = gemm.gemm_query(args.variant, d, *sets[0])
    print(f"{gemm.gemm_variant_name(args.variant)} on {cfg.name}: path {q.path}, grid {q.grid}", flush=True)
    n = max(1, args.launches if cfg.flops / 1e12 < 0.5 or args.variant > 0 else 1)
    torch.cuda.synchronize()
    for i in range(n):
        rc = gemm.gemm_run_ex(args.variant, d, *sets[i % len(sets)])
        assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
    stream.synchronize()
    src = torch.empty(gate.PROBE_COPY_BYTES, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty(gate.PROBE_COPY_BYTES, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    assert gemm.gemm_probe_copy(dst, src, gate.PROBE_COPY_BYTES, stream) == gemm.GEMM_OK
    stream.synchronize()
    print("done", flush=True)


if __name__ == "__main__":
    main()
