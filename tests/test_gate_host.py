"""Host-side pieces of the gate: the acceptance metric, the pass-rate bookkeeping, the ledger table."""
import numpy as np

from paper_2605_28213_amd import gate


def test_normalised_error_definition():
    C_ref = np.array([[1.0, -2.0], [0.0, 4.0]])
    D = np.array([[2.0, 4.0], [0.0, 8.0]])
    C = C_ref + np.array([[0.02, -0.04], [0.0, 0.04]])
    assert abs(gate.normalised_error(C, C_ref, D) - 0.01) < 1e-12
    assert gate.normalised_error(C_ref, C_ref, D) == 0.0
    bad = C_ref.copy(); bad[1, 0] = 1e-30                       # D == 0 admits no error at all
    assert gate.normalised_error(bad, C_ref, D) == float("inf")
    nan = C_ref.copy(); nan[0, 0] = np.nan
    assert gate.normalised_error(nan, C_ref, D) == float("inf")
    assert gate.normalised_error(np.zeros((2, 2)), np.zeros((2, 2)), np.zeros((2, 2))) == 0.0


def test_pass_rate_and_table():
    ok = {"variant": 4, "variant_name": "K4_mfma", "workload": "C2", "verdict": "passed", "query": {"path": "p"},
          "correctness": [{"seed": s, "error": 1e-3, "pass": True} for s in range(3)],
          "profile": {"median_us": 800.0, "TFLOP/s": 1374.0, "GB/s": 503.0}}
    bad = dict(ok, workload="C5", verdict="failed(correctness)",
               correctness=[{"seed": 0, "error": 0.5, "pass": False}, {"seed": 1, "error": 1e-3, "pass": True}])
    ref = {"variant": 4, "variant_name": "K4_mfma", "workload": "C1", "verdict": "refused(precondition: DTYPE_HAS_MFMA)"}
    pr = gate.pass_rate([ok, bad, ref])
    assert pr["attempted"] == 5 and pr["passed"] == 4 and pr["rate"] == 0.8 and len(pr["refused"]) == 1
    table = gate.format_table([ok, bad, ref])
    assert "K4_mfma" in table and "refused" in table and "800.0" in table


def test_compile_leg_rebuilds_a_stale_unit_and_records_kernel_resources():
    """An edited source makes the library stale (by digest): the compile leg recompiles exactly that unit,
    relinks, and the record of the new library carries the digest of the sources on disk and the
    compiler's figures for every kernel."""
    import os
    import subprocess
    import sys
    import textwrap
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = os.path.join(root, "paper_2605_28213_amd", "csrc", "k0_naive.hip")
    original = open(src).read()
    prog = textwrap.dedent("""
        import json, sys
        sys.path.insert(0, %r)
        from paper_2605_28213_amd import gate, build
        print(json.dumps([gate.compile_leg(), build.is_stale()]))
    """ % root)
    try:
        with open(src, "a") as f:
            f.write("\n// (edited by the compile-leg test)\n")
        rec, stale = __import__("json").loads(subprocess.run([sys.executable, "-c", prog], check=True, capture_output=True,
                                                              text=True).stdout.strip().splitlines()[-1])
        assert rec["ok"] and rec["was_stale"] and rec["built_now"] and rec["compiled_units"] == ["k0_naive.hip"] and not stale
    finally:
        with open(src, "w") as f:
            f.write(original)
    rec, stale = __import__("json").loads(subprocess.run([sys.executable, "-c", prog], check=True, capture_output=True,
                                                          text=True).stdout.strip().splitlines()[-1])
    assert rec["ok"] and rec["compiled_units"] == ["k0_naive.hip"] and not stale       # back to the committed source
    from paper_2605_28213_amd import build
    kernels = build.resources()["kernels"]
    fast = [v for k, v in kernels.items() if "k4_mfma_fast<gl::FastCfg<gl::BF16, 256, 8, true, true, 0, false, false>" in k]
    assert len(fast) == 1 and fast[0]["agpr"] == 256 and fast[0]["vgpr_spill"] == 0 and fast[0]["scratch_bytes_per_lane"] == 0
    assert fast[0]["lds_bytes"] == 5 * 32768 and fast[0]["waves_per_simd"] == 1
    # the pipelined state's asynchronous form: three workgroups per CU by LDS (3 stages x 16 KB) and by registers, no spill
    pipe = {k: v for k, v in kernels.items() if "valu_async<" in k}
    assert len(pipe) == 8 and all(v["vgpr_spill"] == 0 and v["scratch_bytes_per_lane"] == 0 for v in pipe.values())
    assert all(v["waves_per_simd"] >= 3 and v["lds_bytes"] == 3 * 16384 for k, v in pipe.items() if ", 8>" in k)
    # the thin kernel for a row-major B: at most 256 registers (two waves per SIMD in a workgroup of eight), no spill
    thin = {k: v for k, v in kernels.items() if "k4_thin_brow<" in k}
    assert len(thin) == 12 and all(v["vgpr_spill"] == 0 and v["scratch_bytes_per_lane"] == 0 and v["waves_per_simd"] >= 2 for v in thin.values())


def test_every_state_and_path_maps_to_kernels_of_the_library():
    from paper_2605_28213_amd import gemm
    from paper_2605_28213_amd import inputs as gen
    cases = [(0, gen.F32, "naive", 16, 16, 256, 0), (1, gen.BF16, "lds-tiled", 64, 64, 256, 0), (2, gen.F16, "vec16", 128, 128, 256, 0),
             (3, gen.E4M3, "vec16", 64, 64, 256, 0),
             (3, gen.BF16, "vec16-direct-to-lds(3 stages)", 128, 128, 256, 0), (3, gen.F32, "vec16-direct-to-lds(3 stages)", 64, 64, 256, 0), (2, gen.BF16, "elementwise-masked(-novec)", 128, 128, 256, gemm.GEMM_FLAG_DEOPT_NO_VECTOR),
             (4, gen.BF16, "mfma32-direct-to-lds", 256, 256, 256, 0), (4, gen.E4M3, "mfma32-direct-to-lds", 128, 128, 256, 0),
             (4, gen.F16, "mfma32-direct-to-lds-mfma32x32", 256, 256, 256, gemm.GEMM_FLAG_MFMA_32X32),
             (4, gen.E4M3, "mfma32-direct-to-lds(persistent)", 256, 256, 256, 0),
             (4, gen.BF16, "mfma32-direct-to-lds-noswz", 256, 256, 256, gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE),
             (4, gen.F16, "mfma32-packed+direct-to-lds+stream(M-tail)", 256, 256, 256, 0),
             (4, gen.F16, "mfma32-direct-to-lds(persistent,B-row-major)+thin(M-tail)", 256, 256, 256, 0),
             (4, gen.BF16, "mfma16-thin(B-row-major)", 32, 64, 512, 0),
             (4, gen.BF16, "mfma32-direct-to-lds+splitK(4)", 128, 128, 256, 0), (4, gen.BF16, "mfma16-stream(small-M)", 16, 16, 64, 0),
             (4, gen.F32, "mfma32-elementwise-masked", 64, 64, 256, 0), (4, gen.F16, "mfma32-vec16-masked", 128, 128, 256, 0)]
    deep = gate.kernel_patterns(4, gen.BF16, "mfma32-direct-to-lds", 128, 128, 256, 0, stages=4)    # nine-region ring of the 128-tile kernel
    assert deep == [r"k4_mfma_fast<gl::FastCfgDeep<gl::BF16> >"] and gate.kernel_resources(deep)
    for (v, dt, path, bm, bn, threads, flags) in cases:
        pats = gate.kernel_patterns(v, dt, path, bm, bn, threads, flags)
        found = gate.kernel_resources(pats)
        assert found, (v, path, pats)
        for p in pats:
            assert any(__import__("re").search(p, k) for k in found), (p, path)


def test_counter_files_are_read_per_launch_and_calibrated(tmp_path):
    head = '"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id","Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count","Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"'
    k = "void gl::k4_mfma_fast<gl::FastCfg<gl::BF16, 256, 8, true, true, 0, false, true> >(gl::Args, int, int, int)"
    row = lambda i, name, c, v: '%d,%d,"Agent 1",2,1,1,1,1,"%s",256,0,0,0,0,0,"%s",%f,0,1' % (i, i, name, c, v)
    (tmp_path / "f_counter_collection.csv").write_text("\n".join([head, row(1, k, "FETCH_SIZE", 800000.0), row(2, k, "FETCH_SIZE", 780000.0),
        row(3, "gl::probe_copy(unsigned int __vector(4)*, unsigned int __vector(4) const*, unsigned long)", "FETCH_SIZE", 131072.0)]) + "\n")
    (tmp_path / "s_counter_collection.csv").write_text("\n".join([head, row(1, k, "SQ_VALU_MFMA_BUSY_CYCLES", 3600.0), row(1, k, "SQ_WAVE_CYCLES", 1000.0),
        row(1, "some other kernel", "SQ_WAVE_CYCLES", 5.0)]) + "\n")
    c = gate.read_counters(str(tmp_path), [r"k4_mfma_fast<gl::FastCfg<gl::BF16, 256"])
    assert c["kernels"] == [k] and c["per_launch"]["FETCH_SIZE"] == 790000.0
    assert abs(c["calibration"]["FETCH_SIZE"] - 2.0) < 1e-12
    assert c["per_launch"]["FETCH_SIZE_bytes"] == 790000.0 * 1024 * 2
    assert abs(c["mfma_busy_per_wave_cycle"] - 0.9) < 1e-12


def test_effect_flags_a_forward_step_that_is_slower():
    prev = {"variant_name": "K2_vectorized", "profile": {"median_us": 100.0, "counters": {"per_launch": {"SQ_INSTS_LDS": 10.0}}}}
    cur = {"variant_name": "K3_pipelined", "profile": {"median_us": 110.0, "counters": {"per_launch": {"SQ_INSTS_LDS": 12.0}}}}
    e = gate.effect_of(cur, prev)
    assert e["regression"] and abs(e["speedup"] - 100.0 / 110.0) < 1e-12 and e["counters"]["SQ_INSTS_LDS"] == {"before": 10.0, "after": 12.0}
    assert not gate.effect_of(prev, dict(cur, profile={"median_us": 400.0}))["regression"]
    assert gate.effect_of(cur, None) is None
    assert gate.scope_of(3)["prior_actions"] == ["tile / sm_stage", "vectorize_global"] and "gfx950" in gate.scope_of(0)["platform"]
