"""Pins for the analytic memory model (Section III-D, Eq. (1)-(5), Fig. 2 caption)."""
import pytest

import oracle
from conftest import read_golden


@pytest.fixture(scope="module")
def gold(golden_dir):
    return read_golden(golden_dir + "/memory_model.txt")


def test_default_and_samo_bytes(gold):
    phi = 2_516_582_400
    for p_num, p_den in ((0, 1), (1, 4), (4, 5), (9, 10), (19, 20), (1, 1)):
        nnz = phi * (p_den - p_num) // p_den
        mm = oracle.memory_model(phi, nnz)
        assert mm.default_bytes == int(gold["default_bytes_per_param"]) * phi
        assert mm.samo_bytes == int(gold["samo_bytes_per_kept_param"]) * nnz + int(gold["samo_bytes_per_param"]) * phi
        # Eq. (5): saving = (24 p - 6) phi
        assert mm.saved_bytes * p_den == (int(gold["saving_slope"]) * p_num + int(gold["saving_offset"]) * p_den) * phi


def test_break_even_and_printed_percentages(gold):
    phi = 1_000_000
    be = float(gold["break_even_sparsity"])
    assert oracle.memory_model(phi, int(phi * (1 - be))).saved_bytes == 0
    assert oracle.memory_model(phi, int(phi * (1 - be)) + 1).saved_bytes < 0
    assert round(100 * oracle.memory_model(phi, 200_000).saved_fraction) == int(gold["saved_percent_at_0.8"])
    assert round(100 * oracle.memory_model(phi, 100_000).saved_fraction) == int(gold["saved_percent_at_0.9"])


def test_resident_bytes_of_the_fused_pipeline():
    # idx + p + m + v at 4 bytes per kept parameter, dense fp16 weights at 2 per parameter
    assert oracle.resident_bytes(1000, 100) == 16 * 100 + 2 * 1000
    assert oracle.resident_bytes(1000, 100) < oracle.memory_model(1000, 100).samo_bytes
