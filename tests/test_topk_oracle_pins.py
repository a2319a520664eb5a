"""Pins for the CPU oracle of row-wise top-k (no GPU, no HIP library).

The paper names the workload's shape only (Sec. 4.1 workload table: batch 64, sequence 4096,
k = 512, FP32); the selection itself has a plain definition, and the pins are closed forms, two
library routines and an exhaustive brute force.
"""
import itertools

import numpy as np
import pytest
import torch


def test_ramps_and_constant_rows(oracle):
    n, k = 37, 9
    up = np.arange(n, dtype=np.float32)[None, :]
    idx, val = oracle.topk(up, k)
    assert idx[0].tolist() == list(range(n - k, n)) and val[0].tolist() == list(range(n - k, n))
    down = up[:, ::-1].copy()
    idx, val = oracle.topk(down, k)
    assert idx[0].tolist() == list(range(k)) and val[0].tolist() == [float(n - 1 - i) for i in range(k)]
    const = np.full((1, n), 2.5, np.float32)
    idx, val = oracle.topk(const, k)
    assert idx[0].tolist() == list(range(k)) and set(val[0].tolist()) == {2.5}        # ties go to the lowest indices


def test_edge_values_of_k_and_signed_zeros(oracle):
    x = np.array([[3.0, -1.0, 7.0, 7.0, 0.0, -0.0, 2.0]], np.float32)
    idx, val = oracle.topk(x, 0)
    assert idx.shape == (1, 0)
    idx, val = oracle.topk(x, 1)
    assert idx[0].tolist() == [2] and val[0].tolist() == [7.0]                        # first of the equal maxima
    idx, val = oracle.topk(x, 7)
    assert idx[0].tolist() == list(range(7))
    np.testing.assert_array_equal(val.view(np.uint32), x.view(np.uint32))              # values are copied bit for bit
    idx, val = oracle.topk(x, 5)                                                       # 7 7 3 2 and one of the zeros: +0.0 at index 4
    assert idx[0].tolist() == [0, 2, 3, 4, 6]
    y = np.array([[-0.0, 0.0, -5.0]], np.float32)
    idx, val = oracle.topk(y, 1)
    assert idx[0].tolist() == [0] and np.signbit(val[0, 0])                            # -0.0 ties with +0.0; lower index wins
    with pytest.raises(ValueError):
        oracle.topk(x, 8)
    with pytest.raises(ValueError):
        oracle.topk(np.array([[1.0, np.nan]], np.float32), 1)


@pytest.mark.parametrize("n,k", [(1, 1), (64, 5), (257, 100), (1000, 999), (4096, 512)])
def test_against_stable_argsort_and_torch_topk(oracle, n, k):
    rng = np.random.default_rng(n + k)
    x = rng.standard_normal((5, n)).astype(np.float32)
    x[1] = np.round(x[1] * 2) / 2            # many ties, also at the threshold
    x[2] = np.abs(x[2])
    x[3, ::3] = x[3, 0]
    idx, val = oracle.topk(x, k)
    for b in range(5):
        order = np.argsort(-x[b].astype(np.float64), kind="stable")[:k]                # descending value, then index
        np.testing.assert_array_equal(idx[b], np.sort(order))
        np.testing.assert_array_equal(val[b], x[b][np.sort(order)])
        tv = torch.topk(torch.from_numpy(x[b]), k).values.numpy()
        np.testing.assert_array_equal(np.sort(val[b])[::-1], tv)                        # the multiset of values is unique


def test_exhaustive_short_rows_over_a_small_alphabet(oracle):
    alphabet = np.array([-1.0, 0.0, 0.5], np.float32)
    for n in range(1, 6):
        rows = np.array(list(itertools.product(alphabet, repeat=n)), np.float32)
        for k in range(0, n + 1):
            idx, val = oracle.topk(rows, k)
            for r in range(rows.shape[0]):
                want = sorted(sorted(range(n), key=lambda i: (-rows[r, i], i))[:k])
                assert idx[r].tolist() == want
                assert val[r].tolist() == [rows[r, i] for i in want]


def test_rows_are_independent_and_strided_rows_work(oracle):
    rng = np.random.default_rng(9)
    wide = rng.standard_normal((4, 80)).astype(np.float32)
    view = wide[:, :50]                      # leading dimension 80, row length 50
    idx, val = oracle.topk(view, 7)
    for b in range(4):
        i1, v1 = oracle.topk(np.ascontiguousarray(view[b:b + 1]), 7)
        np.testing.assert_array_equal(idx[b], i1[0])
        np.testing.assert_array_equal(val[b], v1[0])
        assert idx[b].max() < 50
