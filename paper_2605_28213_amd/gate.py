"""The validation gate applied to one lineage state on one workload (paper Sec. 3.1, Sec. 4.1), and the
skill record it fills in.

The paper accepts a kernel state only after it passes a compile / correctness / profile gate, with
correctness checked at three random seeds and latency taken as the median of 100 launches after 25
warm-ups; the profile deltas between neighbouring states feed the skill record (Sec. 3.3), whose fields
are intent, anchor, carrier, pre, effect, evidence, risk, scope and ver (Sec. 3.1).  This module is
that gate for the GEMM lineage, minus any judgement of its own about what the right answer is:
reference values are handed in by the caller (the test-suite hands in the CPU oracle's), so the package
itself stays free of any second implementation of the product.

Legs, in order, each recorded in the ledger entry:
  compile      the library is brought up to date with its sources (every call: a stale binary cannot
               pass); the entry keeps the digest of the sources, which translation units were compiled
               now, and the registers / spills / scratch / LDS / occupancy of the kernels this state
               launches, as the compiler reported them
  query        conditions the state relies on / holds / violates, the code path, launch geometry (`pre`)
  correctness  per seed: max |C - C_ref| / D over the reference outputs, no NaN/Inf anywhere in C (`ver`)
  profile      HIP-event time of every launch on the launch stream, operands rotated over three sets
               (median, mean, min, p10, p90), plus hardware counters per launch when the caller hands in
               a counter file written by `python3 -m paper_2605_28213_amd.profile_run` under rocprofv3
               (`evidence`)
and, from those: `effect` (latency and counter deltas against the predecessor state's entry, with a flag
when a forward step is slower), `risk` (what the state does on a workload that violates its conditions:
refusal mask under GEMM_FLAG_STRICT, slow path and measured slowdown otherwise; see `risk_probe`),
`scope` (platform, language, the intents already applied).

A state whose conditions are violated is not an error of the gate: without GEMM_FLAG_STRICT its own
masked path runs (and the entry says which); with it the call is refused and the entry records the
violated conditions.
"""
from __future__ import annotations

import csv
import glob
import json
import os
import re
import time
from dataclasses import dataclass
from typing import Callable, Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

from . import gemm
from . import inputs as gen

TOLERANCE = {gen.F32: 1e-5, gen.BF16: 1e-2, gen.F16: 1e-2, gen.E4M3: 6e-2}
_OUT_BYTES = {gen.F32: 4, gen.BF16: 2, gen.F16: 2}
_DT = {gen.F32: "F32", gen.BF16: "BF16", gen.F16: "F16", gen.E4M3: "E4M3"}
OPERAND_SETS = 3          # the profile leg rotates its launches over this many copies of the operands
SCOPE = {"platform": "AMD Instinct MI355X (gfx950, CDNA4)", "language": "HIP C++", "workload": "dense GEMM, fp32 accumulation"}


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


# ---- compile leg -------------------------------------------------------------------------------------
def kernel_patterns(variant: int, in_dtype: int, path: str, bm: int, bn: int, threads: int, flags: int = 0, stages: int = 2) -> List[str]:
    """Regular expressions (on demangled names) of the kernels a state launches on the path the query names."""
    dt = "gl::" + _DT[in_dtype]
    if variant == gemm.GEMM_K0_NAIVE:
        return [r"k0_naive<%s>" % dt]
    if variant in (gemm.GEMM_K1_LDS_TILED, gemm.GEMM_K2_VECTORIZED, gemm.GEMM_K3_PIPELINED):
        vec = "false" if variant == gemm.GEMM_K1_LDS_TILED or (flags & gemm.GEMM_FLAG_DEOPT_NO_VECTOR) else "true"
        dbuf = "true" if variant == gemm.GEMM_K3_PIPELINED else "false"
        if variant == gemm.GEMM_K3_PIPELINED and path.startswith("vec16-direct-to-lds"):
            return [r"valu_async<%s, %d>" % (dt, bm // 16)]
        return [r"valu_tiled<%s, gl::ValuCfg<%d, %d, \d+, \d+, \d+, %s, %s>" % (dt, bm, bn, vec, dbuf)]
    pats = []
    if "stream(small" in path:
        return [r"k4_stream<gl::StreamCfg<%s, %d, " % (dt, threads // 64)]
    if path.startswith("mfma16-thin"):
        return [r"k4_thin_brow<gl::ThinCfg<%s, %d, %d, " % (dt, 1 if bm <= 16 else 2 if bm <= 32 else 4, bn)]
    if "direct-to-lds" in path:
        swz = "false" if flags & gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE else "true"
        ovl = "false" if flags & gemm.GEMM_FLAG_DEOPT_NO_OVERLAP else "true"
        if "(persistent,B-row-major)" in path:
            pats.append(r"k4_mfma_ring<gl::RingCfg<%s, \d+, true>" % dt)
        elif "(persistent)" in path:
            pats.append(r"k4_mfma_ring<gl::RingCfg<%s, \d+, false>" % dt)
        elif bm == 128 and stages == 4:
            pats.append(r"k4_mfma_fast<gl::FastCfgDeep<%s> >" % dt)     # 128-tiles, at most one per CU, long K: nine-region ring
        else:
            # (two-byte types on 256-tiles with none of the switches multiply with the 16x16x32 instruction)
            mi16 = ("true" if in_dtype in (gen.BF16, gen.F16) and bm == 256 and not (flags & (gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE |
                    gemm.GEMM_FLAG_DEOPT_NO_OVERLAP | gemm.GEMM_FLAG_MFMA_32X32)) else "false")
            pats.append(r"k4_mfma_fast<gl::FastCfg<%s, %d, \d+, %s, %s, \d+, false, %s>" % (dt, bm, swz, ovl, mi16))
        if "packed" in path:
            pats.append(r"k4_pack_(rows|transpose)<%s>" % dt)
        if "splitK" in path:
            pats.append(r"k4_splitk_reduce<%s>" % dt)
        if "stream(M-tail)" in path:
            pats.append(r"k4_stream<gl::StreamCfg<%s, " % dt)
        if "+masked(" in path or "+split(" in path:
            pats.append(r"k4_mfma_masked<%s, " % dt)
        if "+thin(" in path or "+split(" in path:
            pats.append(r"k4_thin_brow<gl::ThinCfg<%s, " % dt)
        return pats
    return [r"k4_mfma_masked<%s, %d, %d, " % (dt, bm, bn)]


def compile_leg(rebuild: bool = False) -> dict:
    """Brings the library up to date (mtimes of sources and headers against objects; `rebuild` forces a
    full compile) and returns the compile record; a failed build is a verdict, not an exception."""
    from . import build as gl_build
    try:
        # stale = no library, or one linked from other sources than those on disk (by digest, so that a
        # copied tree with reshuffled file times neither hides an edit nor triggers a needless compile)
        was_stale = gl_build.is_stale()
        built = []
        lib_path = gemm.LIB_PATH
        if was_stale or rebuild:
            loaded = gemm._lib is not None
            lib_path = gl_build.build(force=rebuild)
            built = gl_build.last_built()
            if built and loaded:
                return {"ok": False, "compiled_units": built, "was_stale": was_stale,
                        "error": "the library was rebuilt after this process had loaded the old one: run the gate in a fresh process"}
        res = gl_build.resources()
        ok = res.get("sources_sha256") == gl_build.sources_digest()
        rec = {"ok": ok, "library": os.path.basename(lib_path), "abi": gemm.gemm_abi_version(), "built_now": bool(built),
               "compiled_units": built, "was_stale": was_stale, "sources_sha256": res.get("sources_sha256")}
        if not ok:
            rec["error"] = "the library's recorded source digest differs from the sources on disk"
        return rec
    except Exception as e:
        return {"ok": False, "error": str(e)[-2000:]}


def kernel_resources(patterns: Sequence[str]) -> Dict[str, dict]:
    """Registers, spills, scratch, LDS and occupancy of the kernels matching `patterns`, from the record the
    build wrote at link time."""
    from . import build as gl_build
    table = gl_build.resources()["kernels"]
    out = {}
    for name, fig in table.items():
        if any(re.search(p, name) for p in patterns):
            out[name] = {k: v for k, v in fig.items() if k != "mangled"}
    return out


# ---- counters ----------------------------------------------------------------------------------------
def read_counters(directory: str, patterns: Sequence[str], calibrate: bool = True) -> dict:
    """Per-launch hardware counters of the kernels matching `patterns` from the CSV files rocprofv3 wrote
    under `directory` (`--pmc ... --output-format csv`; several runs with different counters may share the
    directory).  Values are averaged over the dispatches of a kernel and summed over the matching kernels
    (a state's launch may consist of several).  FETCH_SIZE and WRITE_SIZE (KiB per dispatch) are also
    given in bytes, scaled by the factor the copy probe of known size shows in the same files."""
    per_kernel: Dict[str, Dict[str, List[float]]] = {}
    for path in sorted(glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                name, ctr = row.get("Kernel_Name", ""), row.get("Counter_Name", "")
                try:
                    val = float(row.get("Counter_Value", "nan"))
                except ValueError:
                    continue
                per_kernel.setdefault(name, {}).setdefault(ctr, []).append(val)
    mean = lambda v: sum(v) / len(v)
    out: dict = {"kernels": [], "per_launch": {}}
    for name, ctrs in per_kernel.items():
        if any(re.search(p, name) for p in patterns):
            out["kernels"].append(name)
            for c, v in ctrs.items():
                out["per_launch"][c] = out["per_launch"].get(c, 0.0) + mean(v)
    if calibrate:
        factor = {}
        for name, ctrs in per_kernel.items():
            if "probe_copy" in name:
                for c, v in ctrs.items():
                    if c in ("FETCH_SIZE", "WRITE_SIZE") and mean(v) > 0:
                        factor[c] = (PROBE_COPY_BYTES / 1024.0) / mean(v)
        out["calibration"] = factor
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            if c in out["per_launch"] and c in factor:
                out["per_launch"][c + "_bytes"] = out["per_launch"][c] * 1024.0 * factor[c]
    pl = out["per_launch"]
    # SQ_WAVE_CYCLES counts in units of four clocks; the busy counter of the matrix pipes in clocks
    if "SQ_VALU_MFMA_BUSY_CYCLES" in pl and pl.get("SQ_WAVE_CYCLES"):
        out["mfma_busy_per_wave_cycle"] = pl["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * pl["SQ_WAVE_CYCLES"])
    if "SQ_LDS_BANK_CONFLICT" in pl and pl.get("SQ_WAVE_CYCLES"):
        out["lds_bank_conflict_per_wave_cycle_unit"] = pl["SQ_LDS_BANK_CONFLICT"] / pl["SQ_WAVE_CYCLES"]
    return out


PROBE_COPY_BYTES = 256 << 20     # what profile_run's calibration launch copies


# ---- skill-record fields derived from entries ----------------------------------------------------------
def effect_of(entry: dict, predecessor: Optional[dict]) -> Optional[dict]:
    """`effect`: what the transition into this state changed, measured against the predecessor's entry on
    the same workload: latency ratio and counter deltas; `regression` flags a forward step that is slower."""
    if not predecessor or not entry.get("profile") or not predecessor.get("profile"):
        return None
    a, b = predecessor["profile"], entry["profile"]
    eff = {"against": predecessor.get("variant_name", predecessor.get("variant")), "median_us_before": a["median_us"],
           "median_us_after": b["median_us"], "speedup": a["median_us"] / b["median_us"],
           "regression": b["median_us"] > 1.02 * a["median_us"]}
    ca, cb = (a.get("counters") or {}).get("per_launch", {}), (b.get("counters") or {}).get("per_launch", {})
    delta = {c: {"before": ca[c], "after": cb[c]} for c in sorted(set(ca) & set(cb))}
    if delta:
        eff["counters"] = delta
        # what the counters say about the step, in words (kept with the numbers: Sec. 3.3 feeds profile deltas into the record)
        ratio = lambda c: (cb[c] / ca[c]) if c in delta and ca[c] else None
        parts = []
        for c, what in (("SQ_INSTS_LDS", "LDS instructions"), ("SQ_INSTS_VMEM_RD", "vector memory reads"), ("SQ_INSTS_VALU", "VALU instructions"),
                        ("SQ_WAIT_INST_ANY", "wave cycles spent waiting"), ("FETCH_SIZE_bytes", "bytes fetched past L2")):
            r = ratio(c)
            if r is not None:
                parts.append("%s x%.2f" % (what, r))
        if parts:
            eff["reading"] = ("slower" if eff["regression"] else "faster" if eff["speedup"] > 1.02 else "level") + ": " + ", ".join(parts)
    return eff


def scope_of(variant: int) -> dict:
    """`scope`: where the record applies (platform, language) and which intents are already in place."""
    return dict(SCOPE, prior_actions=[gemm.gemm_variant_intent(v) for v in range(1, variant)])


def run_gate(variant: int, cfg: gen.Config, reference: Callable[[gen.Inputs], Reference], *,
             seeds: Iterable[int] = (0, 1, 2), warmup: int = 25, reps: int = 100, strict: bool = False,
             time_budget_s: float = 3.0, inputs_cache: Optional[Dict[int, gen.Inputs]] = None,
             rebuild: bool = False, lend_workspace: bool = True, extra_flags: int = 0,
             ledger_path: Optional[str] = None, predecessor: Optional[dict] = None,
             counters_dir: Optional[str] = None, risk: Optional[dict] = None) -> dict:
    """Run the gate for (variant, cfg) and return the ledger entry (also appended to ledger_path).

    `reference(inputs)` supplies the values C is compared against.  `reps` is cut down for states so
    slow that 100 launches would exceed `time_budget_s` (the entry records the number used).
    `extra_flags` are GEMM_FLAG_DEOPT_* bits: the gate applied to a simplification of the expert state.
    `predecessor` is the entry of the state before this one on the same workload (for `effect`);
    `counters_dir` a directory of rocprofv3 counter files for this (state, workload); `risk` the result
    of `risk_probe` for this state.
    """
    import torch

    entry: dict = {"variant": variant, "workload": cfg.name, "time": time.time(),
                   "shape": [cfg.M, cfg.N, cfg.K, cfg.batch], "in_dtype": gen.DTYPE_NAMES[cfg.in_dtype],
                   "strict": strict, "flags": extra_flags}
    # ---- compile ---------------------------------------------------------------------------------
    entry["compile"] = compile_leg(rebuild)
    if not entry["compile"]["ok"]:
        entry["verdict"] = "failed(compile)"
        return _finish(entry, ledger_path)
    entry["variant_name"] = gemm.gemm_variant_name(variant)
    entry["intent"] = gemm.gemm_variant_intent(variant)
    entry["scope"] = scope_of(variant)

    if not torch.cuda.is_available():
        raise RuntimeError("the gate's correctness and profile legs need a GPU")
    stream = torch.cuda.Stream()
    flags = (gemm.GEMM_FLAG_STRICT if strict else 0) | extra_flags
    tol = TOLERANCE[cfg.in_dtype]
    seed_results: List[dict] = []
    timing = None
    verdict = "passed"
    patterns: List[str] = []
    for seed in seeds:
        inp = inputs_cache[seed] if inputs_cache is not None and seed in inputs_cache else gen.make_inputs(cfg, seed)
        if inputs_cache is not None:
            inputs_cache[seed] = inp
        hA = torch.from_numpy(np.ascontiguousarray(inp.A).reshape(-1).view(np.uint8))
        hB = torch.from_numpy(np.ascontiguousarray(inp.B).reshape(-1).view(np.uint8))
        dA, dB = hA.cuda(), hB.cuda()
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
            patterns = kernel_patterns(variant, cfg.in_dtype, q.path, q.bm, q.bn, q.threads, extra_flags, q.stages)
            try:
                entry["compile"]["kernels"] = kernel_resources(patterns)
            except Exception as e:      # a library built by other means carries no record: say so, do not guess
                entry["compile"]["kernels"] = {}
                entry["compile"]["resources_error"] = str(e)
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
        # ---- profile (on the last seed's operands, rotated over OPERAND_SETS copies) -----------------
        last = seed == list(seeds)[-1]
        if last and verdict == "passed":
            sets = [(dA, dB, dC)]
            footprint = hA.numel() + hB.numel() + dC.numel()
            nsets = OPERAND_SETS if footprint * OPERAND_SETS <= (24 << 30) else 1
            for _ in range(nsets - 1):
                sets.append((hA.cuda(), hB.cuda(), torch.empty_like(dC)))
            torch.cuda.synchronize()

            def launch(i):
                A, B, C_ = sets[i % len(sets)]
                return gemm.gemm_run_ex(variant, d, A, B, C_)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            launch(0)
            e1.record(stream)
            stream.synchronize()
            one = e0.elapsed_time(e1) * 1e-3
            n = int(max(3, min(reps, time_budget_s / max(one, 1e-6))))
            w = int(min(warmup, max(1, n // 4)))
            for i in range(w):
                launch(i)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            rcs = []
            for i, (a, b) in enumerate(ev):
                a.record(stream)
                rcs.append(launch(i))
                b.record(stream)
            stream.synchronize()
            if any(r != gemm.GEMM_OK for r in rcs):
                entry["verdict"] = "failed(launch in the profile leg)"
                return _finish(entry, ledger_path)
            timing = _stats([a.elapsed_time(b) for a, b in ev])
            timing["warmup"] = w
            timing["cache_state"] = f"operands rotated over {len(sets)} buffer sets"
            med = timing["median_us"] * 1e-6
            timing["TFLOP/s"] = cfg.flops / med / 1e12
            timing["GB/s"] = cfg.algorithmic_bytes / med / 1e9
            if counters_dir:
                timing["counters"] = read_counters(counters_dir, patterns)
            del sets
        del dA, dB, dC, ws
    entry["correctness"] = seed_results
    entry["profile"] = timing
    entry["effect"] = effect_of(entry, predecessor)
    if risk is not None:
        entry["risk"] = risk
    entry["verdict"] = verdict
    return _finish(entry, ledger_path)


def risk_probe(variant: int, violating: gen.Config, conforming: gen.Config, reference_v: Callable, reference_c: Callable, *,
               seeds: Iterable[int] = (0,), ledger_path: Optional[str] = None, time_budget_s: float = 1.0) -> dict:
    """`risk`: what the state does where its conditions fail.  Runs the gate on a workload that violates
    them -- under GEMM_FLAG_STRICT (expected: a refusal naming the conditions) and without (the state's own
    slow path, which must still be correct) -- and on a conforming workload of the same size, and reports
    the refusal mask, the slow path and the measured slowdown."""
    refused = run_gate(variant, violating, reference_v, seeds=seeds, strict=True, ledger_path=ledger_path)
    slow = run_gate(variant, violating, reference_v, seeds=seeds, lend_workspace=False, ledger_path=ledger_path,
                    time_budget_s=time_budget_s)
    fast = run_gate(variant, conforming, reference_c, seeds=seeds, ledger_path=ledger_path, time_budget_s=time_budget_s)
    out = {"violating_workload": violating.name, "conforming_workload": conforming.name,
           "violated": (refused.get("query") or {}).get("violated", []), "strict": refused["verdict"],
           "slow_path": (slow.get("query") or {}).get("path"), "slow_path_verdict": slow["verdict"],
           "fast_path": (fast.get("query") or {}).get("path"), "fast_path_verdict": fast["verdict"]}
    if slow.get("profile") and fast.get("profile"):
        out["slow_path_us"], out["fast_path_us"] = slow["profile"]["median_us"], fast["profile"]["median_us"]
        out["slowdown"] = slow["profile"]["median_us"] / fast["profile"]["median_us"]
    return out


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
    rows = ["state          workload  verdict   path                                   max err    median us   TFLOP/s    GB/s    vs predecessor"]
    for e in entries:
        errs = [s["error"] for s in e.get("correctness", [])]
        p = e.get("profile") or {}
        eff = e.get("effect") or {}
        rows.append("%-14s %-9s %-9s %-38s %-10s %-11s %-10s %-7s %s" % (
            e.get("variant_name", e["variant"]), e["workload"], e["verdict"][:9], e.get("query", {}).get("path", "")[:38],
            ("%.2e" % max(errs)) if errs else "-", ("%.1f" % p["median_us"]) if p else "-",
            ("%.2f" % p["TFLOP/s"]) if p else "-", ("%.0f" % p["GB/s"]) if p else "-",
            ("%.2fx%s" % (eff["speedup"], " REGRESSION" if eff["regression"] else "")) if eff else "-"))
    return "\n".join(rows)


def format_resources(entries: Sequence[dict]) -> str:
    """Plain-text table of the compile leg: one line per kernel of each (state, workload)."""
    rows = ["state          workload  kernel                                                                           vgpr agpr sgpr spill(v/s) scratch  lds    waves/SIMD"]
    seen = set()
    for e in entries:
        for name, f in (e.get("compile", {}).get("kernels") or {}).items():
            key = (e.get("variant_name"), e["workload"], name)
            if key in seen:
                continue
            seen.add(key)
            short = re.sub(r"^void gl::|\(gl::Args.*$", "", name)
            rows.append("%-14s %-9s %-80s %-4d %-4d %-4d %d/%-8d %-8d %-6d %d" % (
                e.get("variant_name", e["variant"]), e["workload"], short[:80], f.get("vgpr", -1), f.get("agpr", -1), f.get("sgpr", -1),
                f.get("vgpr_spill", -1), f.get("sgpr_spill", -1), f.get("scratch_bytes_per_lane", -1), f.get("lds_bytes", -1),
                f.get("waves_per_simd", -1)))
    return "\n".join(rows)
