"""Pins for the oracle's data movement: expansion is the inverse of compression (Section
III-C), pruned positions are explicit zeros (Section III-C, forward pass), gather reduces to
a library cast-and-multiply, brute force on tiny layers."""
import itertools

import numpy as np
import pytest

import oracle
import samo_inputs as si


def _masked_fp16(n, seed, keep=0.1):
    mask = si.bernoulli_mask(n, keep, seed)
    w16 = si.weights(n, seed).astype(np.float16).view(np.uint16)
    wm = np.where(mask != 0, w16, np.uint16(0))
    return mask, wm


@pytest.mark.parametrize("n,keep", [(1, 1.0), (7, 0.5), (1000, 0.1), (1 << 20, 0.1), (65537, 0.9)])
def test_expand_inverts_compress_bit_for_bit(n, keep):
    mask, wm = _masked_fp16(n, 11, keep)
    idx = oracle.build_index(mask)
    c16 = oracle.compress_f16(wm, idx)
    assert np.array_equal(c16, wm[idx])                       # library fancy-indexing
    back = oracle.decompress(oracle.f16_bits_to_f32(c16), idx, n)
    assert np.array_equal(back, wm)


def test_compress_of_expand_is_fp16_rounding():
    n = 50000
    mask = si.bernoulli_mask(n, 0.2, 3)
    idx = oracle.build_index(mask)
    p = si.weights(idx.shape[0], 4)
    w = oracle.decompress(p, idx, n)
    assert np.array_equal(oracle.compress_f16(w, idx), p.astype(np.float16).view(np.uint16))


def test_decompress_defines_every_element_over_garbage():
    n = 4099
    mask = si.bernoulli_mask(n, 0.1, 5)
    idx = oracle.build_index(mask)
    p = si.weights(idx.shape[0], 6)
    w = np.full(n, 0x7E00, np.uint16)                         # NaN garbage in the old theta16
    oracle.decompress(p, idx, n, w)
    assert np.all(w[mask == 0] == 0x0000)
    assert np.array_equal(w[idx], p.astype(np.float16).view(np.uint16))


def test_decompress_empty_index_is_zero_fill():
    w = oracle.decompress(np.empty(0, np.float32), np.empty(0, np.int32), 33)
    assert w.shape == (33,) and not w.any()


def test_config1_has_fp16_subnormal_weights():
    # Bernoulli masks keep small weights, so the subnormal branch of the converter is exercised
    mask = si.bernoulli_mask(1 << 20, 0.1, 0)
    w = si.weights(1 << 20, 0)[mask != 0]
    assert np.count_nonzero(np.abs(w) < 2.0 ** -14) > 50


@pytest.mark.parametrize("n", [1, 2, 3, 6])
def test_brute_force_tiny_layers(n):
    rng = np.random.default_rng(n)
    for bits in itertools.product((0, 1), repeat=n):
        mask = np.array(bits, np.uint8)
        idx = oracle.build_index(mask)
        p = rng.standard_normal(idx.shape[0]).astype(np.float32)
        g = rng.standard_normal(n).astype(np.float16)
        w = oracle.decompress(p, idx, n)
        gc = oracle.gather(g.view(np.uint16), idx, 0.25)
        k = 0
        for j in range(n):
            if bits[j]:
                assert w[j] == np.float16(p[k]).view(np.uint16)
                assert gc[k] == np.float32(g[j]) * np.float32(0.25)
                k += 1
            else:
                assert w[j] == 0
        assert k == idx.shape[0]


def test_gather_is_cast_and_one_fp32_multiply():
    n = 1 << 18
    mask = si.bernoulli_mask(n, 0.1, 7)
    idx = oracle.build_index(mask)
    g = si.grads_fp16(n, 7)
    for inv in (1.0 / 1024.0, 1.0, np.float32(1.0) / np.float32(3.0), 1e-3):
        got = oracle.gather(g, idx, inv)
        want = g.view(np.float16)[idx].astype(np.float32) * np.float32(inv)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # a power-of-two loss scale is undone exactly
    assert np.array_equal(oracle.gather(g, idx, 1 / 1024.0) * np.float32(1024),
                          g.view(np.float16)[idx].astype(np.float32))


def test_gather_never_reads_pruned_positions():
    n = 5000
    mask = si.bernoulli_mask(n, 0.3, 8)
    idx = oracle.build_index(mask)
    g = si.grads_fp16(n, 8)
    g2 = g.copy()
    g2[mask == 0] = 0x7C00                                     # +inf garbage where pruned
    assert np.array_equal(oracle.gather(g, idx, 0.5), oracle.gather(g2, idx, 0.5))


def test_gather_honours_fp16_subnormals_and_signed_zero():
    g = np.array([0x0001, 0x8001, 0x03FF, 0x8000, 0x0000, 0x7BFF], np.uint16)
    idx = np.arange(6, dtype=np.int32)
    got = oracle.gather(g, idx, 1.0)
    want = np.array([2.0 ** -24, -2.0 ** -24, 1023 * 2.0 ** -24, -0.0, 0.0, 65504.0], np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_index_preconditions_are_checked():
    p = np.zeros(2, np.float32)
    with pytest.raises(ValueError):
        oracle.decompress(p, np.array([1, 1], np.int32), 4)    # duplicate
    with pytest.raises(ValueError):
        oracle.decompress(p, np.array([2, 1], np.int32), 4)    # descending
    with pytest.raises(ValueError):
        oracle.decompress(p, np.array([0, 4], np.int32), 4)    # out of range


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle's C functions, built with -fsanitize=address,undefined and driven on exact-size
    heap buffers (tests/oracle_sanitizer_driver.c): no out-of-bounds access, no undefined arithmetic."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", os.path.join(root, "oracle", "samo_oracle.c"),
                           os.path.join(root, "tests", "oracle_sanitizer_driver.c"), "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    out = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert out.returncode == 0, out.stderr[-2000:]
    assert out.stdout.startswith("checksum ")
