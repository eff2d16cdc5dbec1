"""Pins of the oracle's weight-gradient + compression functions: the backward pass of a fully
connected layer (Section I: a linear transform of its input) followed by the compression of
Section III-C, which Section VI-C names as the candidate for fusion into the backward kernels."""
import numpy as np
import pytest
import torch

import oracle
import samo_inputs as si


def _halves(a):
    return np.asarray(a, np.float16).reshape(-1).view(np.uint16)


def _problem(tokens, out_f, in_f, seed, keep=0.2):
    dy = si.output_grads_fp16(tokens, out_f, seed)
    x = si.activations_fp16(tokens, in_f, seed)
    idx = oracle.build_index(si.bernoulli_mask(out_f * in_f, keep, seed))
    return dy, x, idx


def test_weight_gradient_equals_autograd_of_a_linear_layer():
    """torch's autograd through F.linear in fp64 — a separate derivation of the same gradient."""
    tokens, out_f, in_f = 37, 11, 19
    dy, x, _ = _problem(tokens, out_f, in_f, 3)
    xt = torch.from_numpy(x.view(np.float16).astype(np.float64).reshape(tokens, in_f))
    dyt = torch.from_numpy(dy.view(np.float16).astype(np.float64).reshape(tokens, out_f))
    w = torch.zeros(out_f, in_f, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.linear(xt, w).backward(dyt)
    got = oracle.linear_weight_grad(dy, x, tokens, out_f, in_f).reshape(out_f, in_f)
    assert np.allclose(got, w.grad.numpy(), rtol=1e-13, atol=1e-15)


def test_weight_gradient_by_explicit_loops_and_operand_order():
    """Brute force on a tiny case with distinct out and in sizes: a transposed operand or swapped
    roles of dY and X would give another shape or other values."""
    tokens, out_f, in_f = 5, 3, 4
    rng = np.random.default_rng(9)
    dy = rng.integers(-4, 5, (tokens, out_f)).astype(np.float16)
    x = rng.integers(-4, 5, (tokens, in_f)).astype(np.float16)
    want = np.zeros((out_f, in_f))
    for o in range(out_f):
        for i in range(in_f):
            for t in range(tokens):
                want[o, i] += float(dy[t, o]) * float(x[t, i])
    got = oracle.linear_weight_grad(_halves(dy), _halves(x), tokens, out_f, in_f)
    assert got.shape == (out_f * in_f,)
    assert np.array_equal(got.reshape(out_f, in_f), want)           # small integers: exact
    mag = oracle.linear_weight_grad_magnitude(_halves(dy), _halves(x), tokens, out_f, in_f)
    assert np.array_equal(mag.reshape(out_f, in_f), np.abs(dy.astype(np.float64)).T @ np.abs(x.astype(np.float64)))
    assert np.all(mag >= np.abs(got))


def test_weight_gradient_is_the_slope_of_the_loss():
    """Finite differences of L = sum(dY * (X W^T)) with respect to single entries of W."""
    tokens, out_f, in_f = 13, 4, 6
    dy, x, _ = _problem(tokens, out_f, in_f, 5)
    a = dy.view(np.float16).astype(np.float64).reshape(tokens, out_f)
    b = x.view(np.float16).astype(np.float64).reshape(tokens, in_f)
    w = np.random.default_rng(1).standard_normal((out_f, in_f))
    loss = lambda w_: float(np.sum(a * (b @ w_.T)))
    got = oracle.linear_weight_grad(dy, x, tokens, out_f, in_f).reshape(out_f, in_f)
    for (o, i) in [(0, 0), (3, 5), (2, 1), (1, 4)]:
        e = np.zeros_like(w)
        e[o, i] = 0.5
        slope = loss(w + e) - loss(w - e)                            # the loss is linear in W
        assert abs(slope - got[o, i]) <= 1e-12 * max(1.0, abs(slope))


def test_compressed_weight_gradient_is_fp16_rounding_then_gather():
    tokens, out_f, in_f = 64, 24, 40
    dy, x, idx = _problem(tokens, out_f, in_f, 7)
    dense = oracle.linear_weight_grad(dy, x, tokens, out_f, in_f)
    rounded = np.array([oracle.f64_to_f16_bits_scalar(float(v)) for v in dense], np.uint16)   # the C oracle's own rounding
    got = oracle.wgrad_compress(dy, x, tokens, out_f, in_f, idx)
    assert got.dtype == np.uint16 and got.shape == idx.shape
    assert np.array_equal(got, rounded[idx])
    assert np.array_equal(got, oracle.compress_f16(rounded, idx))   # Section III-B compression of the dense fp16 tensor
    # one operand all ones: every row of dW is the column sum of X times that row's constant
    ones = _halves(np.ones((tokens, out_f)))
    cols = x.view(np.float16).astype(np.float64).reshape(tokens, in_f).sum(axis=0)
    d1 = oracle.linear_weight_grad(ones, x, tokens, out_f, in_f).reshape(out_f, in_f)
    assert np.allclose(d1, np.broadcast_to(cols, (out_f, in_f)), rtol=1e-14, atol=1e-14)


def test_overflowing_sums_round_to_infinity_and_empty_index():
    tokens, out_f, in_f = 8, 2, 2
    big = _halves(np.full((tokens, out_f), 256.0))
    x = _halves(np.full((tokens, in_f), 256.0))
    idx = np.array([0, 3], np.int32)
    assert oracle.wgrad_compress(big, x, tokens, out_f, in_f, idx).tolist() == [0x7C00, 0x7C00]   # 8 * 65536 > 65504
    assert oracle.wgrad_compress(big, x, tokens, out_f, in_f, np.empty(0, np.int32)).shape == (0,)
    with pytest.raises(ValueError):
        oracle.wgrad_compress(big, x, tokens, out_f, in_f, np.array([4], np.int32))
    with pytest.raises(ValueError):
        oracle.linear_weight_grad(big, x, tokens, out_f, in_f + 1)


def test_sampled_positions_agree_with_the_dense_product():
    tokens, out_f, in_f = 50, 17, 23
    dy, x, idx = _problem(tokens, out_f, in_f, 11)
    dense = oracle.linear_weight_grad(dy, x, tokens, out_f, in_f)
    mag = oracle.linear_weight_grad_magnitude(dy, x, tokens, out_f, in_f)
    val, m = oracle.wgrad_at(dy, x, tokens, out_f, in_f, idx[::3])
    assert np.allclose(val, dense[idx[::3]], rtol=1e-13, atol=1e-15)
    assert np.allclose(m, mag[idx[::3]], rtol=1e-13)
    with pytest.raises(ValueError):
        oracle.wgrad_at(dy, x, tokens, out_f, in_f, [out_f * in_f])


def test_whole_rows_agree_with_triple_loops_and_the_per_position_routine():
    """wgrad_rows against explicit loops on small integers with out != in (every sum exact, so a
    transposed operand or a wrong row shows as a different integer), against the per-position
    routine on random halves, and the magnitude sum against its definition."""
    tokens, out_f, in_f = 5, 4, 3
    rng = np.random.default_rng(5)
    a = rng.integers(-6, 7, (tokens, out_f))
    b = rng.integers(-6, 7, (tokens, in_f))
    rows = np.array([3, 0, 2])
    val, mag = oracle.wgrad_rows(_halves(a), _halves(b), tokens, out_f, in_f, rows)
    assert val.shape == mag.shape == (3, in_f)
    for r, o in enumerate(rows):
        for i in range(in_f):
            assert val[r, i] == sum(int(a[t, o]) * int(b[t, i]) for t in range(tokens))
            assert mag[r, i] == sum(abs(int(a[t, o]) * int(b[t, i])) for t in range(tokens))
    tokens, out_f, in_f = 50, 17, 23
    dy, x, _ = _problem(tokens, out_f, in_f, 11)
    rows = np.array([16, 0, 7, 7])
    val, mag = oracle.wgrad_rows(dy, x, tokens, out_f, in_f, rows)
    pos = (rows[:, None] * in_f + np.arange(in_f)[None, :]).reshape(-1)
    v1, m1 = oracle.wgrad_at(dy, x, tokens, out_f, in_f, pos)
    assert np.allclose(val.reshape(-1), v1, rtol=1e-13, atol=1e-15) and np.allclose(mag.reshape(-1), m1, rtol=1e-13)
    assert np.allclose(val.reshape(-1), oracle.linear_weight_grad(dy, x, tokens, out_f, in_f)[pos], rtol=1e-13, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.wgrad_rows(dy, x, tokens, out_f, in_f, [out_f])


def test_input_recipe_gives_gradients_of_the_usual_spread():
    tokens, out_f, in_f = 512, 32, 48
    dy, x, _ = _problem(tokens, out_f, in_f, 2)
    dense = oracle.linear_weight_grad(dy, x, tokens, out_f, in_f)
    assert abs(dense.std() / (si.G_STD * si.LOSS_SCALE) - 1.0) < 0.1
    assert np.array_equal(dy, si.output_grads_fp16(tokens, out_f, 2)) and np.array_equal(x, si.activations_fp16(tokens, in_f, 2))
