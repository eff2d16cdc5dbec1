"""Pins of the oracle's single-precision SAMO functions (Section III: the optimizations also
apply to single-precision training): dense theta32 with explicit zeros, compressed gradient and
optimizer state, no 16-bit copies."""
import numpy as np
import pytest
import torch

import oracle
import samo_inputs as si


def _problem(n, keep, seed):
    mask = si.bernoulli_mask(n, keep, seed)
    idx = oracle.build_index(mask)
    w = np.where(mask != 0, si.weights(n, seed), np.float32(0.0)).astype(np.float32)   # theta32 with explicit +0
    return mask, idx, w


def _close(got, want):
    """fp32 state fed back each step against a double-precision run: relative 1e-6 with a floor of
    1e-6 of the tensor's rms for entries where beta * m and (1 - beta) * g cancel."""
    want = np.asarray(want, np.float64)
    floor = 1e-6 * float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    return bool(np.all(np.abs(got.astype(np.float64) - want) <= 1e-6 * np.maximum(np.abs(got), np.abs(want)) + floor))


def _grad(n, seed, t):
    return np.random.default_rng([seed, t]).standard_normal(n).astype(np.float32) * np.float32(1e-3)


def test_compress_is_a_gather_with_one_fp32_multiply():
    rng = np.random.default_rng(5)
    dense = rng.standard_normal(1000).astype(np.float32)
    idx = np.flatnonzero(rng.random(1000) < 0.3).astype(np.int32)
    assert np.array_equal(oracle.compress_f32(dense, idx, 1.0).view(np.uint32), dense[idx].view(np.uint32))
    third = np.float32(1.0 / 3.0)
    assert np.array_equal(oracle.compress_f32(dense, idx, third).view(np.uint32),
                          (dense[idx] * third).astype(np.float32).view(np.uint32))      # numpy's fp32 multiply


def test_expand_inverts_compress_and_defines_every_element():
    mask, idx, w = _problem(5003, 0.2, 11)
    c = oracle.compress_f32(w, idx)
    back = oracle.expand_f32(c, idx, w.shape[0])
    assert np.array_equal(back.view(np.uint32), w.view(np.uint32))        # W (.) M survives the round trip
    assert not back.view(np.uint32)[mask == 0].any()                     # +0 bit patterns at pruned positions
    neg = np.array([-0.0, 3.0], np.float32)
    out = oracle.expand_f32(neg, np.array([1, 3], np.int32), 5)
    assert out.view(np.uint32).tolist() == [0, 0x80000000, 0, 0x40400000, 0]   # a kept -0 keeps its sign


@pytest.mark.parametrize("wd,decoupled", [(0.0, 0), (0.05, 0), (0.05, 1)])
def test_three_steps_equal_dense_adam_on_the_masked_tensor(wd, decoupled):
    """Textbook routine: torch.optim.Adam / AdamW in fp64 on the dense tensor with the gradient
    masked.  Pruned positions see a zero gradient, so their state and update stay zero."""
    n = 4001
    mask, idx, w = _problem(n, 0.25, 21)
    cfg = oracle.AdamCfg(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wd, decoupled_wd=decoupled)
    m = np.zeros(idx.shape[0], np.float32)
    v = np.zeros_like(m)
    w_o = w.copy()
    ref = torch.tensor(w.astype(np.float64), requires_grad=True)
    opt_cls = torch.optim.AdamW if decoupled else torch.optim.Adam
    f = lambda x: float(np.float32(x))                          # the hyper-parameters are fp32 values
    opt = opt_cls([ref], lr=f(1e-3), betas=(f(0.9), f(0.999)), eps=f(1e-8), weight_decay=f(wd))
    for t in (1, 2, 3):
        g = _grad(n, 21, t)
        garbage = g.copy()
        garbage[mask == 0] = np.float32(np.nan) if t == 2 else np.float32(1e30)   # never read
        oracle.step_fp32(garbage, w_o, idx, m, v, 1.0, cfg, t)
        ref.grad = torch.tensor((g * mask).astype(np.float64))
        opt.step()
        want = ref.detach().numpy()
        assert _close(w_o[idx], want[idx])
        assert not w_o.view(np.uint32)[mask == 0].any()
        state = opt.state[ref]
        assert _close(m, state["exp_avg"].numpy()[idx])
        assert _close(v, state["exp_avg_sq"].numpy()[idx])
        assert not state["exp_avg"].numpy()[mask == 0].any()              # dense Adam keeps them at zero too


def test_first_step_closed_form_and_gradient_factor():
    """t = 1: m_hat = g, v_hat = g^2, so the step is -lr * g / (|g| + eps); the factor multiplies g."""
    n = 3000
    mask, idx, w = _problem(n, 0.5, 31)
    g = _grad(n, 31, 1)
    cfg = oracle.AdamCfg(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, decoupled_wd=0)
    for factor in (1.0, 0.25):
        w_o = w.copy()
        m = np.zeros(idx.shape[0], np.float32)
        v = np.zeros_like(m)
        oracle.step_fp32(g, w_o, idx, m, v, factor, cfg, 1)
        ge = (g[idx] * np.float32(factor)).astype(np.float64)
        want = w[idx].astype(np.float64) - float(np.float32(1e-2)) * ge / (np.abs(ge) + float(np.float32(1e-8)))
        assert np.allclose(w_o[idx], want, rtol=1e-6, atol=1e-9)
        b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
        assert np.allclose(m, (1 - b1) * ge, rtol=1e-6) and np.allclose(v, (1 - b2) * ge * ge, rtol=1e-6)


def test_garbage_at_pruned_positions_of_theta32_is_replaced_by_zero():
    n = 2000
    mask, idx, w = _problem(n, 0.1, 41)
    dirty = w.copy()
    dirty[mask == 0] = 7.0
    cfg = oracle.AdamCfg(**si.ADAM)
    m = np.zeros(idx.shape[0], np.float32)
    v = np.zeros_like(m)
    clean = w.copy()
    m2, v2 = m.copy(), v.copy()
    g = _grad(n, 41, 1)
    oracle.step_fp32(g, dirty, idx, m, v, 1.0, cfg, 1)
    oracle.step_fp32(g, clean, idx, m2, v2, 1.0, cfg, 1)
    assert np.array_equal(dirty.view(np.uint32), clean.view(np.uint32))
    assert not dirty.view(np.uint32)[mask == 0].any()
