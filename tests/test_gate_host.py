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
