"""Tile sweep for the expert state ("autotune" in the paper's Table 1: the expression-level skill that
needs a templatized kernel; App. D notes that the tile configuration is what a hand-written carrier
contributes beyond the idiom).

The fast kernel of K4 exists in two tile configurations, 256 x 256 (one workgroup per CU) and
128 x 128 (two per CU), each with the XCD-aware tile walk or a plain row-major one: four points.  The
library's default choice is a frozen rule (128-tiles when 256-tiles would not fill the CUs once, always
the XCD-aware walk); this module measures all points on a workload so that the rule can be checked
against the hardware, and prints the table.

    python -m paper_2605_28213_amd.tune C2 C5 P2048
"""
from __future__ import annotations

import json
import sys
from typing import Dict, Iterable

import numpy as np

from . import gemm
from . import inputs as gen

CHOICES = {"default": 0, "tile256": gemm.GEMM_FLAG_TILE_256, "tile128": gemm.GEMM_FLAG_TILE_128,
           "tile256-rowmajor": gemm.GEMM_FLAG_TILE_256 | gemm.GEMM_FLAG_DEOPT_NO_RASTER,
           "tile128-rowmajor": gemm.GEMM_FLAG_TILE_128 | gemm.GEMM_FLAG_DEOPT_NO_RASTER}


def sweep(cfg: gen.Config, *, seed: int = 0, warmup: int = 10, reps: int = 50) -> Dict[str, dict]:
    """Median launch time of K4 on `cfg` for the default tile choice and for each forced one."""
    import torch

    inp = gen.make_inputs(cfg, seed)
    dA = torch.from_numpy(np.ascontiguousarray(inp.A).reshape(-1).view(np.uint8)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(inp.B).reshape(-1).view(np.uint8)).cuda()
    sa = torch.from_numpy(inp.scale_a).cuda() if inp.scale_a is not None else None
    sb = torch.from_numpy(inp.scale_b).cuda() if inp.scale_b is not None else None
    bias = torch.from_numpy(inp.bias).cuda() if inp.bias is not None else None
    dC = torch.empty(max(1, cfg.batch * inp.stride_c) * 4, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    out = {}
    for name, flag in CHOICES.items():
        d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, lda=inp.lda,
                           ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
                           stride_c=inp.stride_c, scale_a=sa, scale_b=sb, bias=bias, stream=stream, flags=flag)
        q = gemm.gemm_query(gemm.GEMM_K4_MFMA, d, dA, dB, dC)
        if q.status != gemm.GEMM_OK:
            out[name] = {"status": gemm.gemm_status_string(q.status)}
            continue
        torch.cuda.synchronize()
        for _ in range(warmup):
            gemm.gemm_run_ex(gemm.GEMM_K4_MFMA, d, dA, dB, dC)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record(stream)
            gemm.gemm_run_ex(gemm.GEMM_K4_MFMA, d, dA, dB, dC)
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        med = ms[len(ms) // 2]
        out[name] = {"path": q.path, "tile": [q.bm, q.bn], "grid": q.grid, "median_us": 1e3 * med,
                     "TFLOP/s": cfg.flops / (med * 1e-3) / 1e12}
    return out


def report(names: Iterable[str]) -> str:
    points = [k for k in CHOICES if k != "default"]
    rows = ["workload   default tile  default us   " + "   ".join("%-16s" % (p + " us") for p in points) + "   best"]
    for n in names:
        r = sweep(gen.CONFIGS[n])
        t = {k: v.get("median_us") for k, v in r.items()}
        best = min((k for k in points if t.get(k)), key=lambda k: t[k], default="-")
        fmt = lambda x: ("%.1f" % x) if x else "-"
        rows.append("%-10s %-13s %-12s " % (n, "x".join(map(str, r["default"].get("tile", []))) or "-", fmt(t.get("default")))
                    + "   ".join("%-16s" % fmt(t.get(p)) for p in points) + "   " + best)
    return "\n".join(rows)


if __name__ == "__main__":
    names = sys.argv[1:] or ["C2", "C5", "P4096", "P2048", "PBMM16", "PBMM32"]
    print(report(names))
