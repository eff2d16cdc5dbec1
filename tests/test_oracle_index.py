"""Pins for the oracle's index construction (Section III, definition of ind_i; Section III-B)."""
import itertools

import numpy as np
import pytest

import oracle
import samo_inputs as si
from conftest import read_golden


def test_paper_worked_example(golden_dir):
    gold = read_golden(golden_dir + "/index_example.txt")
    rows, cols = map(int, gold["shape"].split())
    coords = list(map(int, gold["nonzero_coords"].split()))
    want = np.array(list(map(int, gold["flat_indices"].split())), np.int32)
    dense = np.zeros((rows, cols), np.uint8)
    for r, c in zip(coords[0::2], coords[1::2]):
        dense[r, c] = 1
    got = oracle.build_index(np.ascontiguousarray(dense).reshape(-1))
    assert got.dtype == np.int32
    assert np.array_equal(got, want)


@pytest.mark.parametrize("n", [0, 1, 2, 5, 12])
def test_brute_force_every_mask(n):
    for bits in itertools.product((0, 1), repeat=n):
        mask = np.array(bits, np.uint8)
        want = [j for j in range(n) if bits[j]]
        got = oracle.build_index(mask)
        assert got.tolist() == want


@pytest.mark.parametrize("n", [1, 63, 64, 65, 1023, 1024, 1025, 4097])
def test_edge_masks_invariants(n):
    for name, mask in si.edge_masks(n).items():
        idx = oracle.build_index(mask)
        assert idx.shape[0] == np.count_nonzero(mask), name
        assert np.all(np.diff(idx.astype(np.int64)) > 0), name
        assert np.all(mask[idx] != 0), name
        comp = mask.copy()
        comp[idx] = 0
        assert not comp.any(), name


def test_matches_library_flatnonzero_on_config1():
    mask = si.bernoulli_mask(1024 * 1024, 0.1, 0)
    idx = oracle.build_index(mask)
    assert np.array_equal(idx, np.flatnonzero(mask).astype(np.int32))
    # Bernoulli(0.1) over 2^20 draws: mean 104857.6, sd 307
    assert abs(idx.shape[0] - 104857.6) < 6 * 307


def test_mask_not_weight_defines_the_index():
    # a kept weight that is exactly zero stays in the index (the mask is the pruner's output)
    mask = np.array([1, 0, 1, 1], np.uint8)
    p = np.array([0.0, -0.0, 3.0], np.float32)
    idx = oracle.build_index(mask)
    w = oracle.decompress(p, idx, 4)
    assert idx.tolist() == [0, 2, 3]
    assert w.tolist() == [0x0000, 0x0000, 0x8000, 0x4200]


def test_rejects_layers_beyond_int32():
    with pytest.raises((ValueError, TypeError)):
        oracle.build_index(np.lib.stride_tricks.as_strided(np.zeros(1, np.uint8), (2**31,), (0,)))
