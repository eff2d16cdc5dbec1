"""GPU parity of single-precision SAMO (dense theta32 with explicit zeros, dense fp32 gradient,
compressed optimizer state): the fused fp32 step against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import DEV, OCFG, assert_close, dev_f32, dev_u8

pytestmark = pytest.mark.gpu

SIZES = [1, 3, 4, 5, 1023, 1024, 1025, 4095, 4096, 4097, 8200, 100003]


def _grad32(n, seed, t):
    return np.random.default_rng([seed, t]).standard_normal(n).astype(np.float32) * np.float32(1e-3)


class Host:
    def __init__(self, n, keep, seed, dense=False):
        self.n, self.seed, self.dense = n, seed, dense
        self.mask = np.ones(n, np.uint8) if dense else si.bernoulli_mask(n, keep, seed)
        self.idx = oracle.build_index(self.mask)
        self.w = np.where(self.mask != 0, si.weights(n, seed), np.float32(0)).astype(np.float32)
        self.m = np.zeros(self.idx.shape[0], np.float32)
        self.v = np.zeros_like(self.m)


class Dev:
    def __init__(self, h):
        if h.dense:
            self.idx = self.seg_ptr = None
        else:
            ix = samo.samo_build_index(dev_u8(h.mask))
            self.idx, self.seg_ptr = ix.idx, ix.seg_ptr
        self.w, self.m, self.v = dev_f32(h.w), dev_f32(h.m), dev_f32(h.v)
        self.g = torch.empty(h.n, device=DEV)

    def layer(self, h):
        return samo.Layer(h.n, self.idx, self.seg_ptr, None, self.m, self.v, w32=self.w, g32=self.g)


def _check(d, h, what):
    got = d.w.cpu().numpy()
    assert_close(got[h.idx], h.w[h.idx], what + " w32")
    assert not got.view(np.uint32)[h.mask == 0].any(), what + ": pruned positions must be +0"
    assert_close(d.m.cpu().numpy(), h.m, what + " m")
    assert_close(d.v.cpu().numpy(), h.v, what + " v")


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("keep", [0.0, 0.05, 0.5, 1.0])
def test_fused_step_fp32_ragged_sizes(n, keep):
    h = Host(n, keep, 10 * n + int(keep * 100))
    d = Dev(h)
    for t in (1, 2):
        g = _grad32(n, h.seed, t)
        g_dirty = g.copy()
        g_dirty[h.mask == 0] = np.float32(np.nan)                 # never read
        d.g.copy_(dev_f32(g_dirty))
        if t == 1:                                               # garbage at pruned positions is replaced by +0
            dirty = h.w.copy()
            dirty[h.mask == 0] = 3.0
            d.w.copy_(dev_f32(dirty))
        samo.samo_fused_step_fp32(d.g, d.w, d.idx, d.seg_ptr, d.m, d.v, 1.0, samo.adam_cfg(t, **si.ADAM))
        oracle.step_fp32(g, h.w, h.idx, h.m, h.v, 1.0, OCFG, t)
        _check(d, h, "n=%d keep=%g t=%d" % (n, keep, t))


@pytest.mark.parametrize("n", [1, 4, 5, 1024, 4097, 50001])
def test_dense_layer_fp32(n):
    h = Host(n, 1.0, 77 + n, dense=True)
    d = Dev(h)
    for t in (1, 2, 3):
        g = _grad32(n, h.seed, t)
        d.g.copy_(dev_f32(g))
        samo.samo_fused_step_fp32(d.g, d.w, None, None, d.m, d.v, 0.5, samo.adam_cfg(t, lr=1e-3, weight_decay=0.01))
        oracle.step_fp32(g, h.w, h.idx, h.m, h.v, 0.5, oracle.AdamCfg(1e-3, 0.9, 0.999, 1e-8, 0.01, 0), t)
        _check(d, h, "dense n=%d t=%d" % (n, t))


def test_fp32_batched_mixed_model():
    specs = [(3 * 4096, 0.1, False), (1, 1.0, False), (5000, 0.0, False), (4097, 0.3, False), (100003, 0.05, False),
             (30001, 1.0, True), (40000, 0.97, False), (70_001, 1.0, False)]
    hosts = [Host(n, keep, 500 + i, dense) for i, (n, keep, dense) in enumerate(specs)]
    devs = [Dev(h) for h in hosts]
    plan = samo.Plan([d.layer(h) for d, h in zip(devs, hosts)])
    with pytest.raises(samo.SamoError) as e:                      # no compressed p, no fp16 buffers in this plan
        plan.samo_fused_step_batched(1.0, samo.adam_cfg(1, **si.ADAM))
    assert e.value.status == samo.SAMO_ERR_PLAN
    for t in (1, 2):
        grads = [_grad32(h.n, h.seed, t) for h in hosts]
        for d, g in zip(devs, grads):
            d.g.copy_(dev_f32(g))
        plan.samo_fused_step_fp32_batched(1.0, samo.adam_cfg(t, **si.ADAM))
        for d, h, g in zip(devs, hosts, grads):
            oracle.step_fp32(g, h.w, h.idx, h.m, h.v, 1.0, OCFG, t)
            _check(d, h, "batched t=%d n=%d" % (t, h.n))
    plan.close()


def test_fp32_batched_model_that_keeps_under_seven_percent():
    """A single-precision plan below 7 % kept gets tiles of one and a half times the weight (eight
    segments, a 32 KiB fp32 image): sizes that end inside a segment, an empty layer."""
    specs = [(200_003, 0.05, False), (9 * 1024, 0.0, False), (65_536, 0.03, False), (50_000, 0.06, False)]
    hosts = [Host(n, keep, 900 + i, dense) for i, (n, keep, dense) in enumerate(specs)]
    devs = [Dev(h) for h in hosts]
    plan = samo.Plan([d.layer(h) for d, h in zip(devs, hosts)])
    assert plan.num_tiles == sum(-(-(6144 * -(-h.n // 1024) + 24 * h.idx.shape[0]) // 49152) for h in hosts)
    for t in (1, 2):
        grads = [_grad32(h.n, h.seed, t) for h in hosts]
        for d, g in zip(devs, grads):
            d.g.copy_(dev_f32(g))
        plan.samo_fused_step_fp32_batched(1.0, samo.adam_cfg(t, **si.ADAM))
        for d, h, g in zip(devs, hosts, grads):
            oracle.step_fp32(g, h.w, h.idx, h.m, h.v, 1.0, OCFG, t)
            _check(d, h, "sparse plan t=%d n=%d" % (t, h.n))
    plan.close()


def test_fp32_statistics_clipping_and_overflow_skip():
    specs = [(50_000, 0.1, False), (4097, 0.3, False), (30001, 1.0, True), (200_003, 0.05, False)]
    hosts = [Host(n, keep, 800 + i, dense) for i, (n, keep, dense) in enumerate(specs)]
    devs = [Dev(h) for h in hosts]
    plan = samo.Plan([d.layer(h) for d, h in zip(devs, hosts)])
    stats = samo.GradStats(plan)
    factor, max_norm = 0.5, 0.01
    grads = [_grad32(h.n, h.seed, 1) for h in hosts]
    for d, h, g in zip(devs, hosts, grads):
        dirty = g.copy()
        dirty[h.mask == 0] = np.float32(np.inf)                  # pruned positions do not count
        d.g.copy_(dev_f32(dirty))
    plan.samo_grad_stats_batched(3, factor, stats)
    ss, bad = stats.read()
    ref_ss = sum(oracle.sum_squares(oracle.compress_f32(g, h.idx, factor)) for h, g in zip(hosts, grads))
    terms = sum(h.idx.shape[0] for h in hosts)
    assert not bad and abs(ss - ref_ss) <= 2 * terms * 2.0 ** -53 * ref_ss
    coef = oracle.clip_coefficient(ref_ss, max_norm)
    assert coef < 1.0
    plan.samo_fused_step_fp32_batched(factor, samo.adam_cfg(1, **si.ADAM), stats.guard(max_norm, True))
    for d, h, g in zip(devs, hosts, grads):
        gc = oracle.compress_f32(g, h.idx, factor)
        oracle.scale(gc, coef)
        pc = oracle.compress_f32(h.w, h.idx)
        oracle.adam(pc, h.m, h.v, gc, OCFG, 1)
        h.w = oracle.expand_f32(pc, h.idx, h.n)
        _check(d, h, "clipped n=%d" % h.n)
    # a non-finite value at a kept position: the guarded step leaves everything as it is
    before = [(d.w.clone(), d.m.clone(), d.v.clone()) for d in devs]
    bad_g = grads[0].copy()
    bad_g[hosts[0].idx[3]] = np.float32(np.nan)
    devs[0].g.copy_(dev_f32(bad_g))
    plan.samo_grad_stats_batched(3, factor, stats)
    assert stats.read()[1] is True
    plan.samo_fused_step_fp32_batched(factor, samo.adam_cfg(2, **si.ADAM), stats.guard(max_norm, True))
    for d, (w0, m0, v0) in zip(devs, before):
        assert torch.equal(d.w, w0) and torch.equal(d.m, m0) and torch.equal(d.v, v0)
    plan.close()


def test_fp32_step_is_deterministic():
    h = Host(300_007, 0.1, 9)
    outs = []
    for _ in range(2):
        d = Dev(h)
        d.g.copy_(dev_f32(_grad32(h.n, 9, 1)))
        samo.samo_fused_step_fp32(d.g, d.w, d.idx, d.seg_ptr, d.m, d.v, 1.0, samo.adam_cfg(1, **si.ADAM))
        outs.append((d.w.clone(), d.m.clone(), d.v.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
