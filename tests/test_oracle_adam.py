"""Pins for the oracle's compressed Adam (Section III-C optimizer step, Section III-D):
closed form of the first step, equality with a textbook dense Adam on the masked tensor
(torch.optim), invariants of the pruned positions."""
import numpy as np
import pytest
import torch

import oracle
import samo_inputs as si

CFG = oracle.AdamCfg(**si.ADAM)


def _f(x):
    return float(np.float32(x))


def _rel_ok(a, b, tol=1e-6):
    a = a.astype(np.float64)
    b = b.astype(np.float64)
    atol = tol * np.sqrt(np.mean(b * b)) if b.size else 0.0
    return np.all(np.abs(a - b) <= tol * np.maximum(np.abs(a), np.abs(b)) + atol)


def test_first_step_closed_form():
    # t = 1, m0 = v0 = 0: mhat = g, vhat = g^2, so p1 = p0 - lr * g / (|g| + eps),
    # m1 = (1 - b1) g, v1 = (1 - b2) g^2.
    rng = np.random.default_rng(0)
    g = np.concatenate([rng.standard_normal(1000) * 1e-3, [0.0, 1e-12, -1e-12, 1e-8, 5.0, -5.0]]).astype(np.float32)
    p0 = rng.standard_normal(g.shape[0]).astype(np.float32)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    oracle.adam(p, m, v, g, CFG, 1)
    g64, p64 = g.astype(np.float64), p0.astype(np.float64)
    lr, b1, b2, eps = _f(CFG.lr), _f(CFG.beta1), _f(CFG.beta2), _f(CFG.eps)
    want_p = p64 - lr * g64 / (np.abs(g64) + eps)
    assert np.all(np.abs(p - want_p) <= 0.5000001 * np.spacing(np.abs(want_p).astype(np.float32)))
    assert np.allclose(m, (1 - b1) * g64, rtol=1e-7, atol=0)
    assert np.allclose(v, (1 - b2) * g64 * g64, rtol=1e-7, atol=1e-45)
    # zero gradient: nothing moves; large gradient: a step of lr against the sign
    z = np.flatnonzero(g == 0)
    assert np.array_equal(p[z], p0[z]) and not m[z].any() and not v[z].any()
    big = np.abs(g) > 1
    assert np.allclose(p[big] - p0[big], -lr * np.sign(g[big]), rtol=1e-3)


@pytest.mark.parametrize("wd,decoupled", [(0.0, 0), (0.1, 0), (0.1, 1)])
def test_compressed_adam_equals_dense_adam_on_masked_tensor(wd, decoupled):
    n, steps = 20000, 5
    mask = si.bernoulli_mask(n, 0.1, 21)
    idx = oracle.build_index(mask)
    w0 = si.weights(n, 21)
    cfg = CFG._replace(weight_decay=wd, decoupled_wd=decoupled)

    # dense textbook Adam in fp64 on W (.) M with gradients masked the same way
    dense = torch.nn.Parameter(torch.from_numpy((w0 * mask).astype(np.float64)))
    kw = dict(lr=_f(cfg.lr), betas=(_f(cfg.beta1), _f(cfg.beta2)), eps=_f(cfg.eps), weight_decay=_f(wd))
    opt = (torch.optim.AdamW if decoupled else torch.optim.Adam)([dense], **kw)

    p = w0[idx].copy()
    m = np.zeros_like(p)
    v = np.zeros_like(p)
    inv = 1.0 / si.LOSS_SCALE
    for t in range(1, steps + 1):
        g16 = si.grads_fp16(n, 21, t)
        gc = oracle.gather(g16, idx, inv)
        oracle.adam(p, m, v, gc, cfg, t)
        gd = g16.view(np.float16).astype(np.float64) * inv * mask
        dense.grad = torch.from_numpy(gd)
        opt.step()
        st = opt.state[dense]
        d = dense.detach().numpy()
        assert _rel_ok(p, d[idx]), t
        assert _rel_ok(m, st["exp_avg"].numpy()[idx]), t
        assert _rel_ok(v, st["exp_avg_sq"].numpy()[idx]), t
        # pruned positions: zero grads keep m = v = 0 and the weight exactly zero
        assert not d[mask == 0].any()
        assert not st["exp_avg"].numpy()[mask == 0].any()
        assert not st["exp_avg_sq"].numpy()[mask == 0].any()


def test_small_gradients_separate_eps_placement():
    # with |g| ~ eps the position of eps (outside the square root) and the bias correction
    # both change the update by O(1); torch's Adam is the reference
    n = 512
    rng = np.random.default_rng(5)
    g = (rng.standard_normal(n) * 3e-8).astype(np.float32)
    p0 = rng.standard_normal(n).astype(np.float32)
    dense = torch.nn.Parameter(torch.from_numpy(p0.astype(np.float64)))
    opt = torch.optim.Adam([dense], lr=_f(1e-2), betas=(_f(0.9), _f(0.999)), eps=_f(1e-8))
    cfg = CFG._replace(lr=1e-2)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in (1, 2, 3):
        oracle.adam(p, m, v, g, cfg, t)
        dense.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
    assert _rel_ok(p, dense.detach().numpy())
    moved = np.abs(p.astype(np.float64) - p0)
    assert moved.max() > 1e-3                                  # the updates were not negligible


def test_three_steps_of_config1_keep_pruned_weights_zero():
    spec = si.config("fc1024")[0]
    data = si.make_layer(spec)
    idx = oracle.build_index(data.mask)
    p = data.w32[idx].copy()
    m = np.zeros_like(p)
    v = np.zeros_like(p)
    for t in (1, 2, 3):
        g = si.grads_fp16(spec.n, spec.seed, t)
        w = oracle.step(g, spec.n, idx, p, m, v, 1.0 / si.LOSS_SCALE, CFG, t)
        assert not w[data.mask == 0].any()
        assert np.array_equal(w[idx], p.astype(np.float16).view(np.uint16))
    # each step moves a weight by at most ~lr (|mhat| / sqrt(vhat) <= 1 / sqrt(1 - b2) in general,
    # about 1 for stationary gradients)
    assert np.max(np.abs(p - data.w32[idx])) < 3 * 3.5e-4


def test_step_equals_its_three_parts():
    n = 10007
    mask = si.bernoulli_mask(n, 0.15, 9)
    idx = oracle.build_index(mask)
    p = si.weights(n, 9)[idx].copy()
    m = np.abs(si.weights(idx.shape[0], 10)) * 1e-3
    v = np.abs(si.weights(idx.shape[0], 11)) * 1e-6
    g = si.grads_fp16(n, 9)
    p2, m2, v2 = p.copy(), m.copy(), v.copy()
    w = oracle.step(g, n, idx, p, m, v, 1 / 1024.0, CFG, 4)
    gc = oracle.gather(g, idx, 1 / 1024.0)
    oracle.adam(p2, m2, v2, gc, CFG, 4)
    assert np.array_equal(p, p2) and np.array_equal(m, m2) and np.array_equal(v, v2)
    assert np.array_equal(w, oracle.decompress(p2, idx, n))


def test_dense_layer_is_the_identity_index_case():
    n = 3000
    idx = oracle.build_index(np.ones(n, np.uint8))
    assert np.array_equal(idx, np.arange(n, dtype=np.int32))
    g = si.grads_fp16(n, 12)
    assert np.array_equal(oracle.gather(g, idx, 1.0), g.view(np.float16).astype(np.float32))
