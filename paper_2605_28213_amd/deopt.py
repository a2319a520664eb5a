"""Guided deoptimisation trace of the expert GEMM state (paper Sec. 3.2 and the deoptimisation-trace
figure of Sec. 4.5: the expert kernel is walked backwards, one optimisation removed per edge, every
intermediate state re-validated, the latency of each recorded; the inverse edges are the lineage's
forward skills).

The walk on gfx950, every state through the gate (three seeds, 100 timed launches unless the state is
slow):

    expert K4 -> -XCD raster -> -LDS swizzle -> -load/MFMA overlap -> -MFMA (= K3) -> -pipeline (= K2)
              -> -vectorised loads (= K2 without them) -> smaller tile, no register tile reuse (= K1)
              -> -LDS staging (= K0, naive)

and two off-lineage orders the forward lineage never visits: swizzle and overlap removed together, and
"pipeline without vectorised loads" (K3 with the vector loads taken out).  Like the gate, this module
never imports the oracle: the caller hands in the reference (tests/test_gate_gpu.py does).
"""
from __future__ import annotations

from typing import Callable, List, Optional

from . import gate, gemm
from . import inputs as gen

F = gemm
# (label, variant, extra flags, on the main backward walk?)
STATES = [
    ("expert (K4)", F.GEMM_K4_MFMA, 0, True),
    ("- XCD raster", F.GEMM_K4_MFMA, F.GEMM_FLAG_DEOPT_NO_RASTER, True),
    ("- LDS swizzle", F.GEMM_K4_MFMA, F.GEMM_FLAG_DEOPT_NO_RASTER | F.GEMM_FLAG_DEOPT_NO_SWIZZLE, True),
    ("- load/MFMA overlap", F.GEMM_K4_MFMA,
     F.GEMM_FLAG_DEOPT_NO_RASTER | F.GEMM_FLAG_DEOPT_NO_SWIZZLE | F.GEMM_FLAG_DEOPT_NO_OVERLAP, True),
    ("- MFMA (K3)", F.GEMM_K3_PIPELINED, 0, True),
    ("- pipeline (K2)", F.GEMM_K2_VECTORIZED, 0, True),
    ("- vector loads", F.GEMM_K2_VECTORIZED, F.GEMM_FLAG_DEOPT_NO_VECTOR, True),
    ("- register tile 8x8 -> 4x4 (K1)", F.GEMM_K1_LDS_TILED, 0, True),
    ("- LDS staging (K0)", F.GEMM_K0_NAIVE, 0, True),
    ("expert - swizzle only", F.GEMM_K4_MFMA, F.GEMM_FLAG_DEOPT_NO_SWIZZLE, False),
    ("expert - overlap only", F.GEMM_K4_MFMA, F.GEMM_FLAG_DEOPT_NO_OVERLAP, False),
    ("K3 - vector loads (off-lineage)", F.GEMM_K3_PIPELINED, F.GEMM_FLAG_DEOPT_NO_VECTOR, False),
]


def trace(cfg: gen.Config, reference: Callable, *, seeds=(0, 1, 2), ledger_path: Optional[str] = None,
          time_budget_s: float = 1.0) -> List[dict]:
    """Run every state of the walk through the gate on `cfg`; returns the ledger entries, labelled."""
    cache: dict = {}
    out = []
    for label, variant, flags, main in STATES:
        e = gate.run_gate(variant, cfg, reference, seeds=seeds, inputs_cache=cache, extra_flags=flags,
                          ledger_path=ledger_path, time_budget_s=time_budget_s)
        e["deopt_label"], e["deopt_main_walk"] = label, main
        out.append(e)
    return out


def format_trace(entries: List[dict]) -> str:
    rows = ["state                               verdict   path                                         median us    x expert"]
    base = None
    for e in entries:
        med = e.get("profile", {}).get("median_us")
        if base is None and med:
            base = med
        rows.append("%-35s %-9s %-44s %-12s %s" % (
            ("  " if not e["deopt_main_walk"] else "") + e["deopt_label"], e["verdict"][:9], e.get("query", {}).get("path", "")[:44],
            ("%.1f" % med) if med else "-", ("%.2f" % (med / base)) if med and base else "-"))
    return "\n".join(rows)
