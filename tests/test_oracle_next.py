"""Pins for the oracle functions of the widened path: compressed fp16 gradient accumulation and
up-cast (Section III-A, III-C), global gradient norm / overflow check / clipping, SGD momentum."""
import numpy as np
import pytest
import torch

import oracle
import samo_inputs as si


def test_f64_to_f16_vs_numpy_direct_cast():
    rng = np.random.default_rng(0)
    xs = np.concatenate([
        rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 6, 200000),
        np.array([0.0, -0.0, 65504.0, 65519.999999, 65520.0, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -50),
                  3 * 2.0 ** -25, 1 + 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -40, 1 + 3 * 2.0 ** -11, 5e-324, 1e-310,
                  np.inf, -np.inf, 1e300, 2.0 ** -14 - 2.0 ** -26]),
        # every exact sum of two halves near rounding boundaries: a large value plus a tiny one
        (np.arange(1024, 2048)[:, None] * 2.0 ** -10 + np.array([2.0 ** -11, 2.0 ** -11 + 2.0 ** -24, 2.0 ** -12])[None, :]).reshape(-1),
    ])
    with np.errstate(all="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f64_to_f16_bits_scalar(x) for x in xs], np.uint16)
    assert np.array_equal(got, want)
    assert (oracle.f64_to_f16_bits_scalar(float("nan")) & 0x7C00) == 0x7C00
    assert (oracle.f64_to_f16_bits_scalar(float("nan")) & 0x03FF) != 0


def test_accumulate_is_correctly_rounded_half_addition():
    n = 300000
    mask = si.bernoulli_mask(n, 0.3, 1)
    idx = oracle.build_index(mask)
    g1, g2, g3 = (si.grads_fp16(n, 1, t) for t in (1, 2, 3))
    # mix magnitudes so that exponent gaps of every size occur
    g2 = (g2.view(np.float16) * np.float16(2.0) ** np.random.default_rng(2).integers(-14, 3, n).astype(np.float16)).view(np.uint16)
    acc = oracle.compress_f16(g1, idx)
    oracle.accumulate_f16(g2, idx, acc)
    want = (g1.view(np.float16)[idx] + g2.view(np.float16)[idx]).view(np.uint16)      # numpy's half add
    assert np.array_equal(acc, want)
    # exact reference through float64 and a direct float64 -> float16 cast
    exact = g1.view(np.float16)[idx].astype(np.float64) + g2.view(np.float16)[idx].astype(np.float64)
    assert np.array_equal(acc, exact.astype(np.float16).view(np.uint16))
    oracle.accumulate_f16(g3, idx, acc)
    want = (want.view(np.float16) + g3.view(np.float16)[idx]).view(np.uint16)
    assert np.array_equal(acc, want)


def test_accumulate_overflow_and_cancellation():
    g = np.array([0x7BFF, 0x7BFF, 0x3C00, 0x0001, 0x8001], np.uint16)         # 65504, 65504, 1, tiny, -tiny
    acc = np.array([0x7BFF, 0xFBFF, 0xBC00, 0x0001, 0x0001], np.uint16)       # +65504, -65504, -1, tiny, tiny
    oracle.accumulate_f16(g, np.arange(5, dtype=np.int32), acc)
    assert acc.tolist() == [0x7C00, 0x0000, 0x0000, 0x0002, 0x0000]           # inf, +0, +0, 2 tiny, +0


def test_upcast_of_compressed_equals_gather_of_dense():
    n = 100000
    mask = si.bernoulli_mask(n, 0.1, 3)
    idx = oracle.build_index(mask)
    g = si.grads_fp16(n, 3)
    for inv in (1 / 1024.0, 1.0, 1 / 3.0):
        a = oracle.upcast(oracle.compress_f16(g, idx), inv)
        b = oracle.gather(g, idx, inv)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        want = g.view(np.float16)[idx].astype(np.float32) * np.float32(inv)   # library cast and multiply
        assert np.array_equal(a.view(np.uint32), want.view(np.uint32))


def test_sum_squares_and_clip_match_torch_clip_grad_norm():
    rng = np.random.default_rng(4)
    layers = [(rng.standard_normal(n) * s).astype(np.float32) for n, s in ((1000, 1.0), (50000, 0.01), (7, 100.0))]
    total = sum(oracle.sum_squares(x) for x in layers)
    params = [torch.nn.Parameter(torch.zeros(x.shape[0], dtype=torch.float64)) for x in layers]
    for prm, x in zip(params, layers):
        prm.grad = torch.from_numpy(x.astype(np.float64))
    for max_norm in (1.0, 50.0, 1e6):
        for prm, x in zip(params, layers):
            prm.grad = torch.from_numpy(x.astype(np.float64))
        norm = torch.nn.utils.clip_grad_norm_(params, max_norm)
        assert abs(float(norm) - np.sqrt(total)) <= 1e-12 * np.sqrt(total)
        coef = oracle.clip_coefficient(total, max_norm)
        for prm, x in zip(params, layers):
            y = x.copy()
            oracle.scale(y, coef)
            assert np.allclose(y, prm.grad.numpy(), rtol=2e-7, atol=0)
    assert oracle.clip_coefficient(total, 1e6) == np.float32(1.0)
    # exact small case: 3-4-5 triangle
    assert oracle.sum_squares(np.array([3.0, 4.0], np.float32)) == 25.0


def test_has_nonfinite():
    x = np.ones(1000, np.float32)
    assert not oracle.has_nonfinite(x)
    for bad in (np.inf, -np.inf, np.nan):
        y = x.copy()
        y[777] = bad
        assert oracle.has_nonfinite(y)
    assert not oracle.has_nonfinite(np.empty(0, np.float32))
    # an fp16 gradient that overflowed shows up after the up-cast
    assert oracle.has_nonfinite(oracle.upcast(np.array([0x3C00, 0x7C00], np.uint16), 1 / 1024.0))


@pytest.mark.parametrize("momentum,wd", [(0.9, 0.0), (0.9, 5e-4), (0.0, 0.0)])
def test_sgd_momentum_equals_dense_torch_sgd_on_masked_tensor(momentum, wd):
    n, steps = 20000, 5
    f = lambda x: float(np.float32(x))
    mask = si.bernoulli_mask(n, 0.1, 31)
    idx = oracle.build_index(mask)
    w0 = si.weights(n, 31)
    dense = torch.nn.Parameter(torch.from_numpy((w0 * mask).astype(np.float64)))
    opt = torch.optim.SGD([dense], lr=f(0.1), momentum=f(momentum), weight_decay=f(wd))
    p = w0[idx].copy()
    buf = np.zeros_like(p)
    for t in range(1, steps + 1):
        g16 = si.grads_fp16(n, 31, t)
        gc = oracle.gather(g16, idx, 1 / 1024.0)
        oracle.sgd(p, buf, gc, 0.1, momentum, wd)
        dense.grad = torch.from_numpy(g16.view(np.float16).astype(np.float64) / 1024.0 * mask)
        opt.step()
        d = dense.detach().numpy()
        assert np.allclose(p, d[idx], rtol=1e-6, atol=1e-9), t
        assert not d[mask == 0].any()
        if momentum:
            assert np.allclose(buf, opt.state[dense]["momentum_buffer"].numpy()[idx], rtol=1e-6, atol=1e-9)


def test_dp_split_equals_fused_sequence():
    # gather to compressed fp16 -> (all-reduce would go here) -> up-cast -> Adam -> expand gives
    # exactly what gather(+up-cast) -> Adam -> expand gives (Section III-C, Section IV-A)
    spec = si.config("fc1024")[0]
    data = si.make_layer(spec)
    idx = oracle.build_index(data.mask)
    cfg = oracle.AdamCfg(**si.ADAM)
    pa = data.w32[idx].copy(); ma = np.zeros_like(pa); va = np.zeros_like(pa)
    pb, mb, vb = pa.copy(), ma.copy(), va.copy()
    for t in (1, 2, 3):
        g = si.grads_fp16(spec.n, spec.seed, t)
        wa = oracle.step(g, spec.n, idx, pa, ma, va, 1 / 1024.0, cfg, t)
        gc = oracle.upcast(oracle.compress_f16(g, idx), 1 / 1024.0)
        oracle.adam(pb, mb, vb, gc, cfg, t)
        wb = oracle.decompress(pb, idx, spec.n)
        assert np.array_equal(pa, pb) and np.array_equal(ma, mb) and np.array_equal(va, vb)
        assert np.array_equal(wa, wb)
