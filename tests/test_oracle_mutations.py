"""Mutation check of the oracle's pins (CPU only).

Each case plants one plausible mistake in a copy of ``gemm_oracle.c`` (a dropped term, a
wrong sign, a transposed operand, an off-by-one, a wrong bias), builds it, swaps it in for
the real library and requires that at least one pin in ``test_oracle_pins`` fails.
"""
import os
import subprocess

import pytest

import oracle as oracle_mod
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "gemm_oracle.c")

MUTATIONS = {
    "transposed_B_index": ("return layout == ORACLE_ROW_MAJOR ? r * ld + c : c * ld + r;",
                           "return layout == ORACLE_ROW_MAJOR ? c * ld + r : r * ld + c;"),
    "dropped_last_k_full": ("for (int64_t k = 0; k < K; ++k) {\n                    double p = Ad",
                            "for (int64_t k = 0; k + 1 < K; ++k) {\n                    double p = Ad"),
    "sign_slip": ("acc += p;", "acc -= p;"),
    "mag_without_abs": ("mag += fabs(p);", "mag += p;"),
    "scale_a_ignored": ("if (scale_a) s *= (double)scale_a[b];", ""),
    "scale_sign_kept_in_D": ("D[b * stride_c + i * ldc + j] = fabs(s) * mag;", "D[b * stride_c + i * ldc + j] = s * mag;"),
    "bf16_wrong_mantissa_width": ("return decode_fields(s, e, m, 127, 7);", "return decode_fields(s, e, m, 127, 8);"),
    "e4m3_fnuz_bias": ("return decode_fields(s, e, m, 7, 3);", "return decode_fields(s, e, m, 8, 3);"),
    "e4m3_ieee_like_specials": ("if (e == 0xFu && m == 0x7u) return NAN;", "if (e == 0xFu) return NAN;"),
    "f16_subnormal_off": ("mag = ldexp((double)m, 1 - bias - mbits);", "mag = ldexp((double)m, -bias - mbits);"),
    "A_indexed_as_B": ("Ad[i * K + k] = load_elem(dtype, Ab, mat_index(layout_a, i, k, lda));",
                       "Ad[i * K + k] = load_elem(dtype, Ab, mat_index(layout_a, k, i, lda));"),
    "batch_stride_dropped": ("(size_t)(b * stride_b);\n        const double s = batch_scale(scale_a, scale_b, b);\n\n#pragma",
                             "(size_t)(0 * stride_b);\n        const double s = batch_scale(scale_a, scale_b, b);\n\n#pragma"),
    "points_k_off_by_one": ("for (int64_t k = 0; k < K; ++k) {\n            double a = load_elem",
                            "for (int64_t k = 1; k < K; ++k) {\n            double a = load_elem"),
}


def _pins_that_apply():
    """(callable, kwargs) pairs: a cross-section of the pin file, cheap enough to run per mutant."""
    R, C = pins.ROW, pins.COL
    calls = [
        (pins.test_decode_bf16_every_code, {}),
        (pins.test_decode_f16_every_code, {}),
        (pins.test_decode_e4m3_every_code_vs_torch_and_spec, {}),
        (pins.test_sign_and_operand_order_matter, {}),
        (pins.test_batch_scales_and_points, {}),
        (pins.test_padding_is_never_read_and_empty_K, {}),
        (pins.test_transpose_identity, {"dt": pins.F32}),
    ]
    for dt in pins.ALL_DTYPES:
        calls.append((pins.test_all_ones_gives_K, {"dt": dt, "K": 7}))
        calls.append((pins.test_integer_valued_exact_vs_int64_matmul, {"dt": dt, "la": R, "lb": C}))
        calls.append((pins.test_exact_rational_brute_force, {"dt": dt, "M": 2, "N": 3, "K": 5, "la": C, "lb": R}))
    return calls


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the table"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(text.replace(old, new, 1))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so), str(mutated), "-lm"],
                   check=True)
    oracle_mod._load()                                  # make sure the real one is built and bound first
    monkeypatch.setattr(oracle_mod, "_lib", oracle_mod._bind(str(so)))
    caught = []
    for fn, kw in _pins_that_apply():
        try:
            fn(oracle_mod, **kw)
        except (AssertionError, ValueError):
            caught.append(fn.__name__)
    assert caught, f"mutation {name!r} survived every pin"


def test_unmutated_oracle_passes_the_same_selection():
    for fn, kw in _pins_that_apply():
        fn(oracle_mod, **kw)
