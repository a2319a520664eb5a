"""The validation gate over the whole lineage at the full benchmark sizes: every state K0..K4 on
every workload C1..C5, three seeds each, in the launch configuration the benchmark times.

Reference values come from the CPU oracle: at seed 0 the full product of every workload (all 67
million outputs of the headline workload), at seeds 1 and 2 the full product where it is small and
sampled outputs elsewhere (random points, first/last rows and columns, points around workgroup-tile
corners), which the oracle evaluates one by one.  The ledger (gate_ledger.jsonl), its table (gate_table.txt) and the tile
sweep (tile_sweep.txt) are written to the directory GEMM_GATE_OUT names, by default gate_out/ at the
repository root.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_28213_amd import gate, gemm
from paper_2605_28213_amd import inputs as gen

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT_DIR = os.environ.get("GEMM_GATE_OUT") or os.path.join(ROOT, "gate_out")
LEDGER = os.path.join(OUT_DIR, "gate_ledger.jsonl")
TABLE = os.path.join(OUT_DIR, "gate_table.txt")
# optional: a directory of rocprofv3 counter files, one sub-directory "<variant>_<workload>" per pair, written by
# running `python3 -m paper_2605_28213_amd.profile_run` under rocprofv3 (the commands are in that module)
COUNTERS = os.environ.get("GEMM_GATE_COUNTERS")


def counters_dir(variant, name):
    d = os.path.join(COUNTERS, f"{variant}_{name}") if COUNTERS else None
    return d if d and os.path.isdir(d) else None
_entries = []
# the oracle's whole product at seed 0 up to the headline workload's size (about 20 s of host time there)
FULL_PRODUCT_FLOPS = 1.2e12


def sample_points(cfg, rng, n_random=3000):
    M, N, nb = cfg.M, cfg.N, cfg.batch
    pb = [rng.integers(0, nb, n_random)]
    pi = [rng.integers(0, M, n_random)]
    pj = [rng.integers(0, N, n_random)]
    # last row / last column / first row of a random batch item: where tails and masks live
    b = int(rng.integers(0, nb))
    cols = rng.choice(N, size=min(N, 1024), replace=False)
    rows = rng.choice(M, size=min(M, 1024), replace=False)
    for i in (0, M - 1):
        pb.append(np.full(cols.size, b)); pi.append(np.full(cols.size, i)); pj.append(cols)
    for j in (0, N - 1):
        pb.append(np.full(rows.size, b)); pi.append(rows); pj.append(np.full(rows.size, j))
    # corners of 256 x 256 tiles
    ti = np.array([t for t in (255, 256, 257, 2047, 2048, 4095, 4096) if t < M])
    tj = np.array([t for t in (255, 256, 257, 2047, 2048, 4095, 4096) if t < N])
    if ti.size and tj.size:
        gi, gj = np.meshgrid(ti, tj, indexing="ij")
        pb.append(np.full(gi.size, b)); pi.append(gi.ravel()); pj.append(gj.ravel())
    return np.concatenate(pb), np.concatenate(pi), np.concatenate(pj)


class OracleReference:
    """Callable handed to the gate; caches the oracle's values per seed so that the five states of
    one workload are compared against the same numbers."""

    def __init__(self, cfg):
        self.cfg, self.cache = cfg, {}

    def __call__(self, inp):
        if inp.seed in self.cache:
            return self.cache[inp.seed]
        c = self.cfg
        if c.flops <= 1e9 or (inp.seed == 0 and c.flops <= FULL_PRODUCT_FLOPS):
            C_ref, D = oracle.gemm(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, inp.A, inp.lda, inp.B, inp.ldb,
                                   batch=c.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
                                   scale_a=inp.scale_a, scale_b=inp.scale_b, bias=inp.bias)
            ref = gate.Reference(C_ref, D)
        else:
            pts = sample_points(c, np.random.default_rng(100 + inp.seed))
            C_ref, D = oracle.gemm_points(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, inp.A, inp.lda, inp.B,
                                          inp.ldb, *pts, batch=c.batch, stride_a=inp.stride_a, stride_b=inp.stride_b,
                                          scale_a=inp.scale_a, scale_b=inp.scale_b, bias=inp.bias)
            ref = gate.Reference(C_ref, D, pts)
        self.cache[inp.seed] = ref
        return ref


_shared = {}


def reference_for(cfg):
    """One OracleReference per workload for the whole module: the headline workload is gated by four tests
    and its full product is evaluated once."""
    if cfg.name not in _shared:
        _shared[cfg.name] = OracleReference(cfg)
    return _shared[cfg.name]


@pytest.fixture(scope="module", autouse=True)
def ledger_file():
    os.makedirs(os.path.dirname(LEDGER), exist_ok=True)
    if os.path.exists(LEDGER):
        os.remove(LEDGER)
    yield
    with open(TABLE, "w") as f:
        f.write(gate.format_table(_entries) + "\n\n" + json.dumps(gate.pass_rate(_entries)) + "\n")
    with open(os.path.join(OUT_DIR, "gate_resources.txt"), "w") as f:
        f.write(gate.format_resources(_entries) + "\n")


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_every_state_passes_the_gate(name):
    cfg = gen.CONFIGS[name]
    reference, cache = reference_for(cfg), {}
    prev = None
    for v in range(gemm.GEMM_VARIANT_COUNT):
        print(f"[gate] {name} {gemm.gemm_variant_name(v)}", flush=True)
        e = gate.run_gate(v, cfg, reference, inputs_cache=cache, ledger_path=LEDGER, time_budget_s=1.0, predecessor=prev,
                          counters_dir=counters_dir(v, name))
        _entries.append(e)
        assert e["compile"]["ok"] and not e["compile"]["was_stale"] and len(e["compile"]["sources_sha256"]) == 64
        assert e["verdict"] == "passed", (name, e["variant_name"], e["verdict"], e.get("correctness"))
        assert len(e["correctness"]) == 3 and all(s["all_outputs_finite"] for s in e["correctness"])
        assert e["profile"]["launches"] >= 3 and "rotated over 3" in e["profile"]["cache_state"]
        # compile leg: the compiler's figures for the kernels this state launches; none may spill to scratch
        assert e["compile"]["kernels"], (name, e["variant_name"], e["query"]["path"])
        assert all(k["scratch_bytes_per_lane"] == 0 and k["vgpr_spill"] == 0 for k in e["compile"]["kernels"].values())
        # skill-record fields: what the transition changed against the state before it, and where it applies
        assert (e["effect"] is None) == (v == 0) and e["scope"]["prior_actions"] == [gemm.gemm_variant_intent(u) for u in range(1, v)]
        if prev is not None:
            assert e["effect"]["against"] == prev["variant_name"] and e["effect"]["speedup"] > 0
        prev = e
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["P4096", "P2048", "PBMM16", "PBMM32", "PADDMM"])
def test_paper_shapes_pass_the_gate(name):
    """The paper's own GEMM shape and its held-out plain, batched and bias-added GEMM shapes (bf16):
    the expert state at three seeds, the earlier states at one."""
    cfg = gen.CONFIGS[name]
    reference, cache = OracleReference(cfg), {}
    for v in reversed(range(gemm.GEMM_VARIANT_COUNT)):
        print(f"[gate] {name} {gemm.gemm_variant_name(v)}", flush=True)
        seeds = (0, 1, 2) if v == gemm.GEMM_K4_MFMA else (0,)
        e = gate.run_gate(v, cfg, reference, seeds=seeds, inputs_cache=cache, ledger_path=LEDGER, time_budget_s=0.5)
        _entries.append(e)
        assert e["verdict"] == "passed", (name, e["variant_name"], e["verdict"], e.get("correctness"))
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["D32", "D64", "D16_e4m3"])
def test_decode_shapes_with_32_and_64_rows_stream(name):
    """bf16 32 and 64 x 16384 x 16384, e4m3 16 x 16384 x 16384: the expert state reads B once, at more than
    half of the HBM roofline."""
    cfg = gen.CONFIGS[name]
    reference, cache = OracleReference(cfg), {}
    e = gate.run_gate(gemm.GEMM_K4_MFMA, cfg, reference, inputs_cache=cache, ledger_path=LEDGER)
    _entries.append(e)
    assert e["verdict"] == "passed" and e["query"]["path"] == "mfma16-stream(small-M)", e
    bytes_moved = cfg.algorithmic_bytes
    assert bytes_moved / (e["profile"]["median_us"] * 1e-6) > 0.5 * 8e12, e["profile"]
    torch.cuda.empty_cache()


def test_split_k_on_a_decode_shape_passes_the_gate_and_is_faster():
    """bf16 128 x 16384 x 16384 (more rows than the streaming kernel takes, 128 tiles): the expert state at
    three seeds with the scratch its split-K form asks for, and once without; the split form must win."""
    cfg = gen.CONFIGS["D128"]
    reference, cache = OracleReference(cfg), {}
    split = gate.run_gate(gemm.GEMM_K4_MFMA, cfg, reference, inputs_cache=cache, ledger_path=LEDGER, lend_workspace=True)
    plain = gate.run_gate(gemm.GEMM_K4_MFMA, cfg, reference, seeds=(0,), inputs_cache=cache, ledger_path=LEDGER, lend_workspace=False)
    split["variant_name"] += " [splitK]"
    _entries.extend([split, plain])
    assert split["verdict"] == plain["verdict"] == "passed", (split.get("correctness"), plain.get("correctness"))
    assert "splitK(4)" in split["query"]["path"] and "splitK" not in plain["query"]["path"]
    # (the unsplit form runs the nine-region ring of the 128-tile kernel: 128 tiles, 256 slabs; 178 us against 152)
    assert split["profile"]["median_us"] < 0.92 * plain["profile"]["median_us"], (split["profile"], plain["profile"])
    torch.cuda.empty_cache()


def test_simplifications_of_the_expert_state_pass_and_cost_time():
    """Guided deoptimisation on the expert kernel: with the LDS swizzle removed, or with loads no longer
    overlapping the MFMAs, the kernel still passes the gate on the headline workload and is slower;
    the ledger keeps the latency each optimisation buys."""
    cfg = gen.CONFIGS["C2"]
    reference, cache = reference_for(cfg), {}
    base = gate.run_gate(gemm.GEMM_K4_MFMA, cfg, reference, seeds=(0,), inputs_cache=cache, ledger_path=LEDGER)
    assert base["verdict"] == "passed"
    for flags, tag in ((gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE, "-noswz"), (gemm.GEMM_FLAG_DEOPT_NO_OVERLAP, "-noovl"),
                       (gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE | gemm.GEMM_FLAG_DEOPT_NO_OVERLAP, "-noswz-noovl")):
        e = gate.run_gate(gemm.GEMM_K4_MFMA, cfg, reference, seeds=(0,), inputs_cache=cache, extra_flags=flags,
                          ledger_path=LEDGER, time_budget_s=1.0)
        e["variant_name"] = "K4_mfma" + tag
        _entries.append(e)
        assert e["verdict"] == "passed" and e["query"]["path"].endswith(tag), e
        assert e["profile"]["median_us"] > 1.05 * base["profile"]["median_us"], (tag, e["profile"], base["profile"])
    # the switches belong to K4's fast kernel: any other state refuses them
    d = gemm.make_desc(512, 512, 512, gen.BF16, gen.BF16, gen.ROW_MAJOR, gen.COL_MAJOR, flags=gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE)
    assert gemm.gemm_query(gemm.GEMM_K3_PIPELINED, d).status == gemm.GEMM_ERR_BAD_ARG
    torch.cuda.empty_cache()


def test_deoptimisation_trace_of_the_headline_workload():
    """The backward walk from the expert state, one optimisation removed per edge, every state through
    the gate (Sec. 3.2): all must pass, and the table is kept with the gate's output."""
    from paper_2605_28213_amd import deopt
    cfg = gen.CONFIGS["C2"]
    entries = deopt.trace(cfg, reference_for(cfg), seeds=(0,), ledger_path=LEDGER)
    for e in entries:
        e["variant_name"] = e["variant_name"] + " [" + e["deopt_label"] + "]"
        _entries.append(e)
        assert e["verdict"] == "passed", (e["deopt_label"], e["verdict"], e.get("correctness"))
    with open(os.path.join(OUT_DIR, "deopt_trace.txt"), "w") as f:
        f.write(deopt.format_trace(entries) + "\n")
    med = {e["deopt_label"]: e["profile"]["median_us"] for e in entries}
    assert med["- LDS staging (K0)"] > med["- MFMA (K3)"] > med["- load/MFMA overlap"] > med["expert (K4)"]
    torch.cuda.empty_cache()


def test_frozen_configuration_rules_agree_with_the_sweep():
    """The library's default configuration must be the fastest point of the sweep, within noise, on workloads of
    every kind the rules decide: tile side, tile walk and persistent form of the tiled kernel (headline, short-K
    batched e4m3 and bf16, a product with too few 256-tiles), and the streaming kernel's six forms (16, 32 and 64
    rows).  Operands are rotated over three sets.  The sweep table is kept with the gate's output."""
    from paper_2605_28213_amd import tune
    lines, checks = [], []
    for name in ("C2", "C5", "P2048", "PBMM32", "C4", "D32", "D64"):
        r = tune.sweep(gen.CONFIGS[name], reps=30)
        best = tune.best_point(r)
        timed = {k: round(v["median_us"], 1) for k, v in r.items() if "median_us" in v}
        lines.append(f"{name}: default [{r['default']['path']}, tile {r['default']['tile']}, grid {r['default']['grid']}] " + json.dumps(timed))
        checks.append((name, best, timed, r["default"]["median_us"], r[best]["median_us"]))
    with open(os.path.join(OUT_DIR, "tile_sweep.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    for name, best, timed, t_default, t_best in checks:
        assert len(timed) >= 3, (name, timed)                               # the default and at least two other points (64 rows: two forms hold them)
        assert t_default <= 1.12 * t_best, (name, best, timed)
    torch.cuda.empty_cache()


def test_strict_mode_refuses_and_names_the_violated_conditions():
    """The ragged fp16 workload violates the alignment conditions of K2..K4; under STRICT the gate
    records a refusal with the condition names instead of running the masked path."""
    cfg = gen.CONFIGS["C3_small"]
    for v in (gemm.GEMM_K2_VECTORIZED, gemm.GEMM_K3_PIPELINED, gemm.GEMM_K4_MFMA):
        e = gate.run_gate(v, cfg, OracleReference(cfg), seeds=(0,), strict=True, ledger_path=LEDGER)
        _entries.append(e)
        assert e["verdict"].startswith("refused(precondition")
        assert "LD16_A" in e["query"]["violated"] and "correctness" not in e


def test_risk_field_of_the_conditioned_states():
    """What K2, K3 and K4 do where their conditions fail (the ragged fp16 workload, full size and reduced):
    refusal with the violated conditions under STRICT, their own slow path (still correct) otherwise, and
    the measured slowdown against a conforming workload of the same size; the complete record (intent,
    pre, effect, evidence, risk, scope, ver) goes to the ledger."""
    for vname, cname in (("C3", "C3_aligned"), ("C3_small", "C3_small_aligned")):
        viol = gen.CONFIGS[vname]
        up = lambda n, m: (n + m - 1) // m * m
        conf = gen.Config(cname, up(viol.M, 8), up(viol.N, 8), up(viol.K, 64), viol.in_dtype, viol.out_dtype, gen.ROW_MAJOR,
                          gen.COL_MAJOR, viol.dist)
        ref_v, ref_c = reference_for(viol), reference_for(conf)
        prev = None
        for v in (gemm.GEMM_K2_VECTORIZED, gemm.GEMM_K3_PIPELINED, gemm.GEMM_K4_MFMA):
            print(f"[risk] {vname} {gemm.gemm_variant_name(v)}", flush=True)
            risk = gate.risk_probe(v, viol, conf, ref_v, ref_c, ledger_path=LEDGER, time_budget_s=0.5)
            # (K4 on the full-size ragged workload: the persistent kernel reads B row-major in place with under-aligned
            # loads, the thin kernel takes the three rows past the last whole tile; that path relies on none of the
            # violated conditions, so the strict call is not refused.  Everywhere else: a refusal and the masked paths.)
            in_place = v == gemm.GEMM_K4_MFMA and vname == "C3"
            if in_place:
                assert risk["strict"] == "passed" and risk["violated"] == [], risk
            else:
                assert risk["strict"].startswith("refused(precondition") and "LD16_A" in risk["violated"], risk
            assert risk["slow_path_verdict"] == "passed" and risk["fast_path_verdict"] == "passed", risk
            assert ("B-row-major" if in_place else "masked") in risk["slow_path"] and "masked" not in risk["fast_path"], risk
            assert risk["slowdown"] > 1.0, risk
            e = gate.run_gate(v, conf, ref_c, seeds=(0,), ledger_path=LEDGER, time_budget_s=0.5, predecessor=prev, risk=risk)
            e["workload"] = conf.name
            _entries.append(e)
            for field in ("intent", "query", "effect", "profile", "risk", "scope", "correctness"):
                assert field in e, field
            prev = e
    torch.cuda.empty_cache()


def test_pass_rate_of_the_ledger():
    pr = gate.pass_rate(_entries)
    assert pr["attempted"] >= 5 * 3 * 4 and pr["passed"] == pr["attempted"]
    assert len(pr["refused"]) >= 3
