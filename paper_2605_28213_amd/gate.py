"""The validation gate applied to one lineage state on one workload (paper Sec. 3.1, Sec. 4.1).

The paper accepts a kernel state only after it passes a compile / correctness / profile gate, with
correctness checked at three random seeds and latency taken as the median of 100 launches after 25
warm-ups.  This module is that gate for the GEMM lineage, minus any judgement of its own about what
the right answer is: reference values are handed in by the caller (the test-suite hands in the CPU
oracle's), so the package itself stays free of any second implementation of the product.

Legs, in order, each recorded in the ledger entry:
  compile      the shared library is built from source (when absent, or stale under `rebuild`) and
               loads; ABI version recorded
  query        conditions the state relies on / holds / violates, the code path, launch geometry
  correctness  per seed: max |C - C_ref| / D over the reference outputs, no NaN/Inf anywhere in C
  profile      HIP-event time of every launch on the launch stream: median, mean, min, p10, p90

A state whose conditions are violated is not an error of the gate: without GEMM_FLAG_STRICT its own
masked path runs (and the entry says which); with it the call is refused and the entry records the
violated conditions, which is the evidence the paper files under a skill's `risk` field.
"""
from __future__ import annotations

import json
import os
import time
from dataclasses import dataclass
from typing import Callable, Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

from . import gemm
from . import inputs as gen

TOLERANCE = {gen.F32: 1e-5, gen.BF16: 1e-2, gen.F16: 1e-2, gen.E4M3: 6e-2}
_OUT_BYTES = {gen.F32: 4, gen.BF16: 2, gen.F16: 2}


@dataclass
class Reference:
    """Reference outputs for one generated workload: either the full product (points is None,
    C_ref and D shaped (batch, M, N)) or sampled outputs (points = (b, i, j) index arrays)."""
    C_ref: np.ndarray
    D: np.ndarray
    points: Optional[Tuple[np.ndarray, np.ndarray, np.ndarray]] = None


def normalised_error(C: np.ndarray, C_ref: np.ndarray, D: np.ndarray) -> float:
    """max |C - C_ref| / D; +inf for a non-finite output or a non-zero error where D == 0."""
    if not np.all(np.isfinite(C)):
        return float("inf")
    num = np.abs(C - C_ref)
    zero = D == 0
    if np.any(num[zero] != 0):
        return float("inf")
    if np.all(zero):
        return 0.0
    return float(np.max(num[~zero] / D[~zero]))


def _decode(raw: np.ndarray, out_dtype: int) -> np.ndarray:
    if out_dtype == gen.F32:
        return raw.view(np.float32).astype(np.float64)
    if out_dtype == gen.F16:
        return raw.view(np.float16).astype(np.float64)
    return (raw.view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _stats(ms: Sequence[float]) -> Dict[str, float]:
    s = sorted(ms)
    n = len(s)
    return {"median_us": 1e3 * s[n // 2], "mean_us": 1e3 * sum(s) / n, "min_us": 1e3 * s[0],
            "p10_us": 1e3 * s[n // 10], "p90_us": 1e3 * s[(9 * n) // 10], "launches": n}


def run_gate(variant: int, cfg: gen.Config, reference: Callable[[gen.Inputs], Reference], *,
             seeds: Iterable[int] = (0, 1, 2), warmup: int = 25, reps: int = 100, strict: bool = False,
             time_budget_s: float = 3.0, inputs_cache: Optional[Dict[int, gen.Inputs]] = None,
             rebuild: bool = False, lend_workspace: bool = True, extra_flags: int = 0,
             ledger_path: Optional[str] = None) -> dict:
    """Run the gate for (variant, cfg) and return the ledger entry (also appended to ledger_path).

    `reference(inputs)` supplies the values C is compared against.  `reps` is cut down for states so
    slow that 100 launches would exceed `time_budget_s` (the entry records the number used).
    `extra_flags` are GEMM_FLAG_DEOPT_* bits: the gate applied to a simplification of the expert state.
    `rebuild` recompiles stale objects first; otherwise the compile leg only builds when no library
    is present and records that the existing one loaded.
    """
    import torch

    from . import build as gl_build

    entry: dict = {"variant": variant, "workload": cfg.name, "time": time.time(),
                   "shape": [cfg.M, cfg.N, cfg.K, cfg.batch], "in_dtype": gen.DTYPE_NAMES[cfg.in_dtype],
                   "strict": strict, "flags": extra_flags}
    # ---- compile ---------------------------------------------------------------------------------
    try:
        prebuilt = os.path.exists(gemm.LIB_PATH) and not rebuild
        lib_path = gemm.LIB_PATH if prebuilt else gl_build.build()
        entry["compile"] = {"ok": True, "library": os.path.basename(lib_path), "abi": gemm.gemm_abi_version(),
                            "built_now": not prebuilt}
    except Exception as e:  # a failed build is a gate verdict, not a crash of the gate
        entry["compile"] = {"ok": False, "error": str(e)[-2000:]}
        entry["verdict"] = "failed(compile)"
        return _finish(entry, ledger_path)
    entry["variant_name"] = gemm.gemm_variant_name(variant)
    entry["intent"] = gemm.gemm_variant_intent(variant)

    if not torch.cuda.is_available():
        raise RuntimeError("the gate's correctness and profile legs need a GPU")
    stream = torch.cuda.Stream()
    flags = (gemm.GEMM_FLAG_STRICT if strict else 0) | extra_flags
    tol = TOLERANCE[cfg.in_dtype]
    seed_results: List[dict] = []
    timing = None
    verdict = "passed"
    for seed in seeds:
        inp = inputs_cache[seed] if inputs_cache is not None and seed in inputs_cache else gen.make_inputs(cfg, seed)
        if inputs_cache is not None:
            inputs_cache[seed] = inp
        dA = torch.from_numpy(np.ascontiguousarray(inp.A).reshape(-1).view(np.uint8)).cuda()
        dB = torch.from_numpy(np.ascontiguousarray(inp.B).reshape(-1).view(np.uint8)).cuda()
        sa = torch.from_numpy(inp.scale_a).cuda() if inp.scale_a is not None else None
        sb = torch.from_numpy(inp.scale_b).cuda() if inp.scale_b is not None else None
        bias = torch.from_numpy(inp.bias).cuda() if inp.bias is not None else None
        n_out = max(1, cfg.batch * inp.stride_c)
        dC = torch.full((n_out * _OUT_BYTES[cfg.out_dtype],), 0xFF, dtype=torch.uint8, device="cuda")
        d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b,
                           lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a,
                           stride_b=inp.stride_b, stride_c=inp.stride_c, scale_a=sa, scale_b=sb, bias=bias, stream=stream,
                           flags=flags)
        # lend the scratch the state's packed path asks for (K4 on operands that break its fast path)
        ws = None
        if lend_workspace:
            need = gemm.gemm_query(variant, d, dA, dB, dC).workspace_bytes
            if need:
                ws = torch.empty(need, dtype=torch.uint8, device="cuda")
                d.workspace, d.workspace_bytes = ws.data_ptr(), need
        torch.cuda.synchronize()            # uploads and the poison fill ran on another stream
        # ---- query (once) ------------------------------------------------------------------------
        if "query" not in entry:
            q = gemm.gemm_query(variant, d, dA, dB, dC)
            entry["query"] = {"status": gemm.gemm_status_string(q.status), "path": q.path,
                              "required": gemm.Query.names(q.required), "violated": gemm.Query.names(q.violated),
                              "holds": gemm.Query.names(q.holds), "tile": [q.bm, q.bn, q.bk], "threads": q.threads,
                              "stages": q.stages, "lds_bytes": q.lds_bytes, "grid": q.grid,
                              "workspace_bytes": q.workspace_bytes, "workspace_lent": ws is not None}
            if q.status == gemm.GEMM_ERR_PRECONDITION:
                entry["verdict"] = "refused(precondition: " + ",".join(gemm.Query.names(q.violated)) + ")"
                return _finish(entry, ledger_path)
            if q.status != gemm.GEMM_OK:
                entry["verdict"] = f"failed(query: {gemm.gemm_status_string(q.status)})"
                return _finish(entry, ledger_path)
        # ---- correctness ---------------------------------------------------------------------------
        rc = gemm.gemm_run_ex(variant, d, dA, dB, dC)
        stream.synchronize()
        if rc != gemm.GEMM_OK:
            entry["verdict"] = f"failed(launch: {gemm.gemm_status_string(rc)})"
            return _finish(entry, ledger_path)
        C = _decode(dC.cpu().numpy(), cfg.out_dtype)[: cfg.batch * inp.stride_c]
        C = C.reshape(cfg.batch, cfg.M, inp.ldc)[:, :, : cfg.N]
        ref = reference(inp)
        finite = bool(np.all(np.isfinite(C)))
        got = C[ref.points] if ref.points is not None else C
        err = normalised_error(got, ref.C_ref, ref.D) if finite else float("inf")
        ok = err <= tol
        seed_results.append({"seed": seed, "error": err, "tolerance": tol, "outputs_checked": int(ref.C_ref.size),
                             "all_outputs_finite": finite, "pass": ok})
        if not ok:
            verdict = "failed(correctness)"
        # ---- profile (on the last seed's operands) ---------------------------------------------------
        last = seed == list(seeds)[-1]
        if last and verdict == "passed":
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            gemm.gemm_run_ex(variant, d, dA, dB, dC)
            e1.record(stream)
            stream.synchronize()
            one = e0.elapsed_time(e1) * 1e-3
            n = int(max(3, min(reps, time_budget_s / max(one, 1e-6))))
            w = int(min(warmup, max(1, n // 4)))
            for _ in range(w):
                gemm.gemm_run_ex(variant, d, dA, dB, dC)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for a, b in ev:
                a.record(stream)
                gemm.gemm_run_ex(variant, d, dA, dB, dC)
                b.record(stream)
            stream.synchronize()
            timing = _stats([a.elapsed_time(b) for a, b in ev])
            timing["warmup"] = w
            timing["cache_state"] = "same operands every launch"
            med = timing["median_us"] * 1e-6
            timing["TFLOP/s"] = cfg.flops / med / 1e12
            timing["GB/s"] = cfg.algorithmic_bytes / med / 1e9
        del dA, dB, dC, ws
    entry["correctness"] = seed_results
    entry["profile"] = timing
    entry["verdict"] = verdict
    return _finish(entry, ledger_path)


def _finish(entry: dict, ledger_path: Optional[str]) -> dict:
    if ledger_path:
        os.makedirs(os.path.dirname(os.path.abspath(ledger_path)), exist_ok=True)
        with open(ledger_path, "a") as f:
            f.write(json.dumps(entry) + "\n")
    return entry


def pass_rate(entries: Sequence[dict]) -> dict:
    """Gate pass rate over (state, workload, seed) triples; refusals are counted apart."""
    attempted = passed = 0
    refused = []
    for e in entries:
        if e.get("verdict", "").startswith("refused"):
            refused.append((e.get("variant_name", e["variant"]), e["workload"], e["verdict"]))
            continue
        for s in e.get("correctness", []):
            attempted += 1
            passed += bool(s["pass"])
    return {"attempted": attempted, "passed": passed, "rate": passed / attempted if attempted else None,
            "refused": refused}


def format_table(entries: Sequence[dict]) -> str:
    """Plain-text table of a ledger: one line per (state, workload)."""
    rows = ["state          workload  verdict   path                                   max err    median us   TFLOP/s    GB/s"]
    for e in entries:
        errs = [s["error"] for s in e.get("correctness", [])]
        p = e.get("profile") or {}
        rows.append("%-14s %-9s %-9s %-38s %-10s %-11s %-10s %s" % (
            e.get("variant_name", e["variant"]), e["workload"], e["verdict"][:9], e.get("query", {}).get("path", "")[:38],
            ("%.2e" % max(errs)) if errs else "-", ("%.1f" % p["median_us"]) if p else "-",
            ("%.2f" % p["TFLOP/s"]) if p else "-", ("%.0f" % p["GB/s"]) if p else "-"))
    return "\n".join(rows)
