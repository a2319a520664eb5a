"""Configuration sweep for the expert state ("autotune" in the paper's Table 1: the expression-level skill that
needs a templatized kernel; App. D notes that the tile configuration is what a hand-written carrier
contributes beyond the idiom).

What the library freezes, and what this module measures against it on a workload:

  tiled kernel      tile side 256 (one workgroup per CU) or 128 (two per CU)  x  XCD-aware or row-major tile walk
                    x  persistent (one workgroup per CU walks several tiles, the LDS ring runs across tile
                    boundaries) or one tile per workgroup: up to 8 points, those that apply to the product
  streaming kernel  its six compiled forms (waves per workgroup x columns per strip x K run x row groups:
                    1x16x512B/16 rows, 4x16x512B/16, 2x32x512B/32, 4x64x256B/48, /64, /96), those with at
                    least the product's rows

Every point is launched on operands rotated over three buffer sets (a sweep on one set keeps products of up
to ~100 MB in the Infinity Cache between launches and then favours whatever re-reads most).  The library's
default choice is a frozen rule; `sweep` returns the default beside every point so that the rule can be
checked against the hardware (tests/test_gate_gpu.py does), and `report` prints the table.

    python3 -m paper_2605_28213_amd.tune C2 C4 C5 D32 D64 P2048 PBMM32
"""
from __future__ import annotations

import sys
from typing import Dict, Iterable

import numpy as np

from . import gemm
from . import inputs as gen

G = gemm
TILED_POINTS = {
    "tile256": G.GEMM_FLAG_TILE_256,
    "tile256-onetile": G.GEMM_FLAG_TILE_256 | G.GEMM_FLAG_DEOPT_NO_PERSISTENT,
    "tile256-rowmajor": G.GEMM_FLAG_TILE_256 | G.GEMM_FLAG_DEOPT_NO_RASTER,
    "tile256-mfma32x32": G.GEMM_FLAG_TILE_256 | G.GEMM_FLAG_MFMA_32X32,
    "tile128": G.GEMM_FLAG_TILE_128,
    "tile128-rowmajor": G.GEMM_FLAG_TILE_128 | G.GEMM_FLAG_DEOPT_NO_RASTER,
}
STREAM_FORMS = ["1w x 16col x 512B / 16 rows", "4w x 16col x 512B / 16 rows", "2w x 32col x 512B / 32 rows",
                "4w x 64col x 256B / 48 rows", "4w x 64col x 256B / 64 rows", "4w x 64col x 256B / 96 rows"]
STREAM_POINTS = {"form%d" % f: G.GEMM_FLAG_STREAM_FORM(f) for f in range(6)}
OPERAND_SETS = 3


def sweep(cfg: gen.Config, *, seed: int = 0, warmup: int = 10, reps: int = 50, ramp_s: float = 0.5) -> Dict[str, dict]:
    """Median launch time of K4 on `cfg` for the default choice ("default") and for every point that applies.
    The default configuration is first launched for `ramp_s` seconds untimed: from idle the GPU takes some
    tenths of a second to settle at the clock its power limit allows, and the first point measured would
    otherwise be timed on a different clock than the rest."""
    import time

    import torch

    inp = gen.make_inputs(cfg, seed)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a).reshape(-1).view(np.uint8)).cuda()
    sets = [(up(inp.A), up(inp.B), torch.empty(max(1, cfg.batch * inp.stride_c) * 4, dtype=torch.uint8, device="cuda"))
            for _ in range(OPERAND_SETS)]
    sa = torch.from_numpy(inp.scale_a).cuda() if inp.scale_a is not None else None
    sb = torch.from_numpy(inp.scale_b).cuda() if inp.scale_b is not None else None
    bias = torch.from_numpy(inp.bias).cuda() if inp.bias is not None else None
    stream = torch.cuda.Stream()

    def desc(flags):
        return gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, lda=inp.lda,
                              ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
                              stride_c=inp.stride_c, scale_a=sa, scale_b=sb, bias=bias, stream=stream, flags=flags)
    streaming = "stream(small" in gemm.gemm_query(gemm.GEMM_K4_MFMA, desc(0), *sets[0]).path
    points = dict(default=0, **(STREAM_POINTS if streaming else TILED_POINTS))
    out = {}
    d0, t0 = desc(0), time.perf_counter()
    while time.perf_counter() - t0 < ramp_s:
        for i in range(20):
            assert gemm.gemm_run_ex(gemm.GEMM_K4_MFMA, d0, *sets[i % OPERAND_SETS]) == gemm.GEMM_OK
        stream.synchronize()
    for name, flag in points.items():
        d = desc(flag)
        q = gemm.gemm_query(gemm.GEMM_K4_MFMA, d, *sets[0])
        if q.status != gemm.GEMM_OK:
            out[name] = {"status": gemm.gemm_status_string(q.status)}
            continue
        torch.cuda.synchronize()
        for i in range(warmup):
            assert gemm.gemm_run_ex(gemm.GEMM_K4_MFMA, d, *sets[i % OPERAND_SETS]) == gemm.GEMM_OK
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record(stream)
            gemm.gemm_run_ex(gemm.GEMM_K4_MFMA, d, *sets[i % OPERAND_SETS])
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        med = ms[len(ms) // 2]
        out[name] = {"path": q.path, "tile": [q.bm, q.bn], "threads": q.threads, "grid": q.grid, "median_us": 1e3 * med,
                     "TFLOP/s": cfg.flops / (med * 1e-3) / 1e12, "GB/s": cfg.algorithmic_bytes / (med * 1e-3) / 1e9}
    return out


def best_point(result: Dict[str, dict]) -> str:
    timed = {k: v["median_us"] for k, v in result.items() if k != "default" and "median_us" in v}
    return min(timed, key=timed.get)


def report(names: Iterable[str]) -> str:
    rows = []
    for n in names:
        r = sweep(gen.CONFIGS[n])
        b = best_point(r)
        rows.append("%s: default %s [%s, grid %d] %.1f us; best point %s %.1f us" % (
            n, "x".join(map(str, r["default"]["tile"])), r["default"]["path"], r["default"]["grid"], r["default"]["median_us"],
            b, r[b]["median_us"]))
        for k, v in r.items():
            if k != "default":
                rows.append("    %-18s %s" % (k, ("%8.1f us  %-44s grid %d" % (v["median_us"], v["path"], v["grid"])) if "median_us" in v
                                              else "(" + v["status"] + ")"))
    return "\n".join(rows)


if __name__ == "__main__":
    names = sys.argv[1:] or ["C2", "C4", "C5", "D32", "D64", "P4096", "P2048", "PBMM16", "PBMM32"]
    print(report(names))
