"""The seeded input generators: key stream, value maps, host/device agreement."""
import os

import numpy as np
import pytest
import torch

from paper_2507_05753_amd import inputs

GOLDEN_DIR = os.path.join(os.path.dirname(__file__), "golden")


def test_key_stream_is_splitmix64():
    want = [int(l) for l in open(os.path.join(GOLDEN_DIR, "splitmix64_seed1234567.txt"))
            if l.strip() and not l.startswith("#")]
    got = inputs.keys(1234567, np.arange(len(want), dtype=np.uint64))
    assert [int(v) for v in got] == want


def test_keys_are_distinct_and_counter_based():
    k = inputs.keys(3, np.arange(200000, dtype=np.uint64))
    assert np.unique(k).size == k.size
    sub = inputs.keys(3, np.arange(777, 999, dtype=np.uint64))
    assert np.array_equal(sub, k[777:999])


@pytest.mark.parametrize("mode,scale", [("R", 0), ("R", -6), ("L", 0), ("L", -6)])
def test_value_maps(mode, scale):
    v = inputs.matrix(5, 300, 70, mode, scale)
    assert v.dtype == np.float32 and v.shape == (300, 70)
    s = 2.0 ** scale
    assert v.min() >= -1.0 * s and v.max() < 1.0 * s
    grid = 2.0 ** (-23 if mode == "R" else -3) * s
    q = v.astype(np.float64) / grid
    assert np.array_equal(q, np.round(q))
    assert abs(v.mean() + grid / 2) < 0.02 * s   # the grid is [-1, 1) so the mean sits half a step below 0
    if mode == "L":
        assert set(np.unique(q).tolist()) == set(range(-8, 8))


def test_row_subsets_match_the_full_matrix():
    A = inputs.matrix(9, 50, 33, "R", -6)
    assert np.array_equal(inputs.matrix(9, 50, 33, "R", -6, row_begin=7, row_end=21), A[7:21])
    assert np.array_equal(inputs.matrix(9, 50, 33, "R", -6, chunk_rows=3), A)
    rows = [49, 0, 7, 7]
    assert np.array_equal(inputs.matrix_rows(9, 33, rows, "R", -6), A[rows])


@pytest.mark.parametrize("mode,scale", [("R", 0), ("R", -6), ("L", -6)])
def test_torch_generator_matches_numpy_bit_for_bit(mode, scale):
    a = inputs.matrix(123456789, 257, 63, mode, scale)
    b = inputs.matrix_torch(123456789, 257, 63, mode, scale, chunk_elems=1000).numpy()
    assert np.array_equal(a, b)


def test_zipf_mode_keeps_duplicates():
    X = inputs.matrix(4, 2000, 100, "Z")
    vals, counts = np.unique(X, return_counts=True)
    top = counts.max() / X.size
    assert 0.06 < top < 0.09           # rank 1 carries about 7.5 % of the mass
    assert vals.size < 0.9 * X.size    # many repeated values
    assert X.min() >= -1.0 and X.max() < 1.0


def test_layer_inputs_streams_and_configs():
    X, W, b = inputs.layer_inputs(1, 10, 12, 14, "R", bias=True)
    assert X.shape == (10, 12) and W.shape == (14, 12) and b.shape == (14,)
    assert np.array_equal(X, inputs.matrix(1, 10, 12, "R"))
    assert np.array_equal(W, inputs.matrix(1 + inputs.W_STREAM, 14, 12, "R", inputs.W_SCALE_EXP))
    assert np.abs(W).max() < 2.0 ** -6
    for c, cfg in inputs.CONFIGS.items():
        n = cfg["M"] * cfg["K"]
        assert n == {1: 10 ** 4, 2: 10 ** 6, 3: 10 ** 8, 4: 10 ** 8, 5: 2 * 10 ** 9}[c]
        assert cfg["seed"] == c
