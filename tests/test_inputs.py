"""Seeded input generator: statistics, determinism, frozen first draws, workload table (CPU only)."""
import os

import numpy as np

from paper_2605_28213_amd import inputs as gen

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "generator_first8.txt")


def test_frozen_first_draws():
    for line in open(GOLDEN):
        if line.startswith("#"):
            continue
        head, vals = line.split(":")
        kind, seed, tensor = head.split()
        want = np.array([float.fromhex(v) for v in vals.split()], np.float32)
        got = (gen.uniform_pm1 if kind == "uniform" else gen.normal)(int(seed), int(tensor), 8)
        np.testing.assert_array_equal(got, want)


def test_chunking_and_offsets_do_not_change_values():
    n = (1 << 22) + 1234                   # crosses the chunk boundary used for threading
    full = gen.normal(3, 1, n, 0.5)
    part = gen.unit_uniform(3, 1, n - 10, 10, 0)
    u1 = gen.unit_uniform(3, 1, 0, n, 0)
    np.testing.assert_array_equal(u1[-10:], part)
    np.testing.assert_array_equal(full[:100], gen.normal(3, 1, 100, 0.5))
    assert not np.array_equal(gen.normal(3, 1, 100), gen.normal(4, 1, 100))
    assert not np.array_equal(gen.normal(3, 1, 100), gen.normal(3, 2, 100))


def test_moments():
    n = 1_000_000
    u = gen.uniform_pm1(0, 1, n).astype(np.float64)
    assert u.min() > -1 and u.max() < 1
    assert abs(u.mean()) < 4 * (1 / np.sqrt(3)) / np.sqrt(n)
    assert abs(u.var() - 1 / 3) < 4 * np.sqrt(4 / 45) / np.sqrt(n)
    z = gen.normal(0, 2, n, 0.02).astype(np.float64) / 0.02
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs((z ** 4).mean() - 3) < 0.1
    # the two words of one element are uncorrelated
    a, b = gen.unit_uniform(0, 1, 0, n, 0), gen.unit_uniform(0, 1, 0, n, 1)
    assert abs(np.corrcoef(a, b)[0, 1]) < 4 / np.sqrt(n)
    s = gen.uniform_range(0, 3, 10000, 0.5, 2.0)
    assert s.min() >= 0.5 and s.max() <= 2.0


def test_workload_table_matches_the_five_configs():
    c = gen.CONFIGS
    assert (c["C1"].M, c["C1"].N, c["C1"].K, c["C1"].in_dtype) == (256, 256, 256, gen.F32)
    assert (c["C2"].M, c["C2"].layout_a, c["C2"].layout_b) == (8192, gen.ROW_MAJOR, gen.COL_MAJOR)
    assert (c["C3"].M, c["C3"].N, c["C3"].K) == (4099, 4093, 4097) and c["C3"].ld == (4097, 4093, 4093)
    assert (c["C4"].M, c["C4"].N, c["C4"].K) == (16, 16384, 16384)
    assert (c["C5"].batch, c["C5"].in_dtype, c["C5"].out_dtype, c["C5"].scaled) == (64, gen.E4M3, gen.BF16, True)
    assert c["C2"].flops == 2 * 8192 ** 3 and c["C2"].algorithmic_bytes == 402653184
    assert c["C4"].algorithmic_bytes == 537919488 and c["C5"].algorithmic_bytes == 268435456
    assert c["C3"].algorithmic_bytes == 100679662


def test_make_inputs_shapes_and_scales():
    inp = gen.make_inputs(gen.CONFIGS["C5_small"], 1)
    cfg = inp.cfg
    assert inp.A.dtype == np.uint8 and inp.A.size == cfg.batch * cfg.M * cfg.K
    assert inp.scale_a.shape == (cfg.batch,) and inp.scale_a.dtype == np.float32
    assert np.all((inp.A & 0x7F) != 0x7F)          # no NaN codes
    inp3 = gen.make_inputs(gen.CONFIGS["C3_small"], 2)
    assert inp3.lda == 259 and inp3.ldb == 301 and inp3.ldc == 301 and inp3.scale_a is None
    again = gen.make_inputs(gen.CONFIGS["C3_small"], 2)
    np.testing.assert_array_equal(inp3.A, again.A)


def test_conv_and_topk_workload_tables_and_generators():
    c = gen.CONV_CONFIGS["CONV"]
    assert (c.N, c.H, c.W, c.C, c.F, c.R, c.S, c.stride, c.pad, c.in_dtype) == (8, 56, 56, 64, 128, 3, 3, (1, 1), (1, 1), gen.F16)
    assert (c.P, c.Q) == (56, 56) and c.flops == 2 * 8 * 56 * 56 * 128 * 576
    assert c.algorithmic_bytes == (8 * 56 * 56 * 64 + 128 * 576 + 8 * 56 * 56 * 128) * 2
    s2 = gen.CONV_CONFIGS["CONV_stride2"]
    assert (s2.P, s2.Q) == (9, 8) and s2.biased
    ci = gen.make_conv_inputs(gen.CONV_CONFIGS["CONV_small"], 3)
    assert ci.x.shape == (2, 13, 11, 64) and ci.w.shape == (40, 3, 3, 64) and ci.x.dtype == np.uint16 and ci.bias is None
    np.testing.assert_array_equal(ci.x, gen.make_conv_inputs(gen.CONV_CONFIGS["CONV_small"], 3).x)
    assert not np.array_equal(ci.x, gen.make_conv_inputs(gen.CONV_CONFIGS["CONV_small"], 4).x)
    f8 = gen.make_conv_inputs(gen.CONV_CONFIGS["CONV_fp8"], 0)
    assert f8.x.dtype == np.uint8 and np.all((f8.w & 0x7F) != 0x7F)

    t = gen.TOPK_CONFIGS["TOPK"]
    assert (t.batch, t.n, t.k) == (64, 4096, 512) and t.algorithmic_bytes == 64 * (4096 * 4 + 512 * 8)
    r = gen.TOPK_CONFIGS["TOPK_ragged"]
    x = gen.make_topk_inputs(r, 1)
    assert x.shape == (3, 4100) and x.dtype == np.float32 and np.all(x[:, r.n:] == np.float32(1e30))
    assert np.all(x[:, : r.n] * 4 == np.round(x[:, : r.n] * 4))        # the tie-heavy variant: multiples of 1/4
    counts = np.unique(x[0, : r.n], return_counts=True)[1]
    assert counts.max() > 100                                           # many equal values
    np.testing.assert_array_equal(x, gen.make_topk_inputs(r, 1))
