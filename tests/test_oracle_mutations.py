"""Mutation check of the oracle's pins (CPU only).

Each case plants one plausible mistake in a copy of ``gemm_oracle.c``, ``conv_oracle.c`` or ``topk_oracle.c`` (a
dropped term, a wrong sign, a transposed operand, an off-by-one, a wrong bias, a flipped filter),
builds it, swaps it in for the real library and requires that at least one pin in
``test_oracle_pins`` / ``test_conv_oracle_pins`` / ``test_topk_oracle_pins`` fails.
"""
import os
import subprocess

import pytest

import oracle as oracle_mod
from tests import test_conv_oracle_pins as conv_pins
from tests import test_oracle_pins as pins
from tests import test_topk_oracle_pins as topk_pins

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


# ---------------------------------------------------------------- convolution oracle
CONV_SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "conv_oracle.c")

CONV_MUTATIONS = {
    "filter_flipped": ("wd[((f * R + r) * S + s) * C + c]", "wd[((f * R + (R - 1 - r)) * S + (S - 1 - s)) * C + c]"),
    "padding_sign": ("const int64_t h = p * sh - ph + r;", "const int64_t h = p * sh + ph - r;"),
    "padding_off_by_one": ("const int64_t ww = q * sw - pw + s;", "const int64_t ww = q * sw - pw + s + 1;"),
    "taps_swapped": ("const int64_t h = p * sh - ph + r;", "const int64_t h = p * sh - ph + (r * S) / R;"),
    "stride_dropped": ("const int64_t ww = q * sw - pw + s;", "const int64_t ww = q - pw + s;"),
    "image_transposed": ("xd[((n * H + h) * W + ww) * C + c]", "xd[((n * W + ww) * H + h) * C + c]"),
    "border_replicated": ("if (h < 0 || h >= H || ww < 0 || ww >= W) continue;",
                          "if (h < 0 || h >= H || ww < 0 || ww >= W) { for (int64_t c = 0; c < C; ++c) { acc += wd[((f * R + r) * S + s) * C + c]; } continue; }"),
    "mag_without_abs": ("mag += fabs(pr);", "mag += pr;"),
    "last_channel_dropped": ("for (int64_t c = 0; c < C; ++c) {\n                const double pr", "for (int64_t c = 0; c + 1 < C; ++c) {\n                const double pr"),
    "width_from_height_stride": ("*Q = conv_out(W, pad_w, S, stride_w);", "*Q = conv_out(W, pad_w, S, stride_h);"),
    "output_size_rounds_up": ("return (extent + 2 * pad - filt) / stride + 1;", "return (extent + 2 * pad - filt + stride - 1) / stride + 1;"),
    "batch_index_dropped": ("xd[((n * H + h) * W + ww) * C + c]", "xd[((0 * H + h) * W + ww) * C + c]"),
}


def _conv_pins_that_apply():
    calls = [
        (conv_pins.test_centre_tap_identity_filter_returns_the_input, {"dt": pins.F32}),
        (conv_pins.test_all_ones_counts_the_taps_inside_the_image, {"dt": pins.F16}),
        (conv_pins.test_output_size_strides_and_paddings, {}),
        (conv_pins.test_one_by_one_filter_is_a_matrix_product, {"dt": pins.BF16}),
        (conv_pins.test_integer_valued_against_scipy_correlate2d, {}),
        (conv_pins.test_exact_rational_brute_force, {"dt": pins.F16}),
        (conv_pins.test_linearity_and_channel_order, {}),
    ]
    for r, s_ in [(0, 0), (2, 1)]:
        calls.append((conv_pins.test_single_tap_shifts_the_image_without_flipping_the_filter, {"r": r, "s": s_}))
    for geom in [((2, 2), (1, 1), 3, 3), ((1, 2), (0, 2), 3, 2)]:
        calls.append((conv_pins.test_integer_valued_against_torch_fp64_conv2d, {"dt": pins.F32, "geom": geom}))
    return calls


@pytest.mark.parametrize("name", sorted(CONV_MUTATIONS))
def test_planted_conv_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = CONV_MUTATIONS[name]
    text = open(CONV_SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the table"
    mutated = tmp_path / "mutant_conv.c"
    mutated.write_text(text.replace(old, new, 1))
    so = tmp_path / "libmutant_conv.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so), SRC, str(mutated), "-lm"],
                   check=True)
    oracle_mod._load()
    monkeypatch.setattr(oracle_mod, "_lib", oracle_mod._bind(str(so)))
    caught = []
    for fn, kw in _conv_pins_that_apply():
        try:
            fn(oracle_mod, **kw)
        except (AssertionError, ValueError):
            caught.append(fn.__name__)
    assert caught, f"mutation {name!r} survived every pin"


def test_unmutated_conv_oracle_passes_the_same_selection():
    for fn, kw in _conv_pins_that_apply():
        fn(oracle_mod, **kw)


# ---------------------------------------------------------------- top-k oracle
TOPK_SRC = os.path.join(os.path.dirname(oracle_mod.__file__), "topk_oracle.c")

TOPK_MUTATIONS = {
    "smallest_instead_of_largest": ("if (row[j] > row[i] || (row[j] == row[i] && j < i)) ++rank;",
                                    "if (row[j] < row[i] || (row[j] == row[i] && j < i)) ++rank;"),
    "ties_to_higher_index": ("(row[j] == row[i] && j < i)", "(row[j] == row[i] && j > i)"),
    "ties_all_selected": ("if (row[j] > row[i] || (row[j] == row[i] && j < i)) ++rank;", "if (row[j] > row[i]) ++rank;"),
    "ties_count_twice": ("(row[j] == row[i] && j < i)", "(row[j] == row[i] && j != i)"),
    "one_too_few": ("if (rank < k && out < k) {", "if (rank + 1 < k && out < k) {"),
    "row_stride_dropped": ("const float *row = x + b * ld;", "const float *row = x + b * n;"),
    "values_from_first_row": ("val[b * k + out] = row[i];", "val[b * k + out] = x[i];"),
}


def _topk_pins_that_apply():
    return [(topk_pins.test_ramps_and_constant_rows, {}),
            (topk_pins.test_edge_values_of_k_and_signed_zeros, {}),
            (topk_pins.test_against_stable_argsort_and_torch_topk, {"n": 257, "k": 100}),
            (topk_pins.test_exhaustive_short_rows_over_a_small_alphabet, {}),
            (topk_pins.test_rows_are_independent_and_strided_rows_work, {})]


@pytest.mark.parametrize("name", sorted(TOPK_MUTATIONS))
def test_planted_topk_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = TOPK_MUTATIONS[name]
    text = open(TOPK_SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the table"
    mutated = tmp_path / "mutant_topk.c"
    mutated.write_text(text.replace(old, new, 1))
    so = tmp_path / "libmutant_topk.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so), SRC, str(mutated), "-lm"], check=True)
    oracle_mod._load()
    monkeypatch.setattr(oracle_mod, "_lib", oracle_mod._bind(str(so)))
    caught = []
    for fn, kw in _topk_pins_that_apply():
        try:
            fn(oracle_mod, **kw)
        except (AssertionError, ValueError):
            caught.append(fn.__name__)
    assert caught, f"mutation {name!r} survived every pin"
