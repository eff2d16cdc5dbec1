"""GPU parity of the widened path: compressed fp16 gradient (copy / accumulate), the Adam+expand
step that follows an all-reduce, gradient statistics with clipping and overflow skip, SGD."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import (DEV, INV, OCFG, DevLayer, HostLayer, assert_close, dev_f16_bits, dev_f32, dev_i32, host_bits)

pytestmark = pytest.mark.gpu

SIZES = [1, 3, 4, 5, 255, 256, 257, 4095, 4096, 4097, 100003]


def _layer(n, keep, seed, dense=False):
    if keep < 0:                              # -keep of the elements, in four dense stretches
        mask = np.zeros(n, np.uint8)
        run = max(1, int(-keep * n / 4))
        for start in np.random.default_rng(seed).integers(0, n - run, 4):
            mask[start:start + run] = 1
    else:
        mask = np.ones(n, np.uint8) if dense else si.bernoulli_mask(n, keep, seed)
    return HostLayer(n, mask, si.weights(n, seed), seed, dense=dense)


def _wide_range_grads(n, seed):
    """fp16 gradients whose exponents spread over the whole half range (rounding of sums matters)."""
    g = si.grads_fp16(n, seed, 2).view(np.float16)
    e = np.random.default_rng(seed).integers(-14, 3, n).astype(np.float16)
    return (g * np.float16(2.0) ** e).view(np.uint16)


# ------------------------------------------------------------------ compressed fp16 gradient
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("dense", [False, True])
def test_gather_fp16_copy_and_accumulate_bit_exact(n, dense):
    h = _layer(n, 0.3, 600 + n, dense)
    d_idx = None if dense else dev_i32(h.idx)
    g1, g2, g3 = h.grads(1), _wide_range_grads(n, 601 + n), h.grads(3)
    gc16 = torch.full((h.idx.shape[0],), float("nan"), dtype=torch.float16, device=DEV)
    samo.samo_gather_grads_fp16(dev_f16_bits(g1), d_idx, gc16, accumulate=False)
    ref = oracle.compress_f16(g1, h.idx)
    assert np.array_equal(host_bits(gc16), ref)
    for g in (g2, g3):
        samo.samo_gather_grads_fp16(dev_f16_bits(g), d_idx, gc16, accumulate=True)
        oracle.accumulate_f16(g, h.idx, ref)
        assert np.array_equal(host_bits(gc16), ref)


def test_accumulate_overflow_cancellation_and_pruned_garbage():
    g = np.array([0x7BFF, 0x7E00, 0x7BFF, 0x7C00, 0x3C00, 0x0001, 0x8001], np.uint16)
    idx = np.array([0, 2, 4, 5, 6], np.int32)                     # positions 1 and 3 are pruned: NaN / inf there
    acc0 = np.array([0x7BFF, 0xFBFF, 0xBC00, 0x0001, 0x0001], np.uint16)
    gc16 = dev_f16_bits(acc0)
    samo.samo_gather_grads_fp16(dev_f16_bits(g), dev_i32(idx), gc16, accumulate=True)
    ref = acc0.copy()
    oracle.accumulate_f16(g, idx, ref)
    assert ref.tolist() == [0x7C00, 0x0000, 0x0000, 0x0002, 0x0000]
    assert np.array_equal(host_bits(gc16), ref)


# ------------------------------------------------------------------ Adam + expand from the compressed fp16 gradient
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("dense", [False, True])
def test_adam_expand_step_matches_oracle_and_fused(n, dense):
    h = _layer(n, 0.2, 700 + n, dense)
    a, b = DevLayer(h), DevLayer(h)
    for t in (1, 2):
        g = h.grads(t)
        cfg = samo.adam_cfg(t, **si.ADAM)
        gc16 = dev_f16_bits(oracle.compress_f16(g, h.idx))
        a.w.fill_(float("nan"))
        samo.samo_adam_expand_step(gc16, a.w, a.idx, a.seg_ptr, a.p, a.m, a.v, INV, cfg)
        b.set_grads(g)
        samo.samo_fused_step(b.g, b.w, b.idx, b.seg_ptr, b.p, b.m, b.v, INV, cfg)
        gc = oracle.upcast(oracle.compress_f16(g, h.idx), INV)
        oracle.adam(h.p, h.m, h.v, gc, OCFG, t)
        got_p = a.p.cpu().numpy()
        assert_close(got_p, h.p, "p")
        assert_close(a.m.cpu().numpy(), h.m, "m")
        assert_close(a.v.cpu().numpy(), h.v, "v")
        assert np.array_equal(host_bits(a.w), oracle.decompress(got_p, h.idx, n))
        # same arithmetic as the fully fused step: identical bits
        assert torch.equal(a.p, b.p) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v)
        assert np.array_equal(host_bits(a.w), host_bits(b.w))


# ------------------------------------------------------------------ SGD with momentum
@pytest.mark.parametrize("nnz", [1, 5, 256, 257, 100003])
@pytest.mark.parametrize("mu,wd", [(0.9, 0.0), (0.9, 5e-4), (0.0, 0.0)])
def test_sgd_step(nnz, mu, wd):
    rng = np.random.default_rng(nnz)
    p = si.weights(nnz, nnz)
    buf = np.zeros_like(p)
    d_p, d_buf = dev_f32(p), dev_f32(buf)
    for t in range(4):
        gc = (rng.standard_normal(nnz) * 1e-2).astype(np.float32)
        samo.samo_sgd_step(d_p, d_buf, dev_f32(gc), samo.sgd_cfg(0.1, mu, wd))
        oracle.sgd(p, buf, gc, 0.1, mu, wd)
        assert_close(d_p.cpu().numpy(), p, "p")
        assert_close(d_buf.cpu().numpy(), buf, "buf")


@pytest.mark.parametrize("n", [1, 4097, 100003])
@pytest.mark.parametrize("dense", [False, True])
def test_fused_sgd_step(n, dense):
    h = _layer(n, 0.15, 800 + n, dense)
    d = DevLayer(h)
    buf = h.m                                               # zeros: the momentum buffer
    for t in (1, 2, 3):
        g = h.grads(t)
        d.w.fill_(float("nan"))
        d.set_grads(g)
        samo.samo_fused_sgd_step(d.g, d.w, d.idx, d.seg_ptr, d.p, d.m, INV, samo.sgd_cfg(0.05, 0.9, 1e-4))
        oracle.sgd(h.p, buf, oracle.gather(g, h.idx, INV), 0.05, 0.9, 1e-4)
        got_p = d.p.cpu().numpy()
        assert_close(got_p, h.p, "p")
        assert_close(d.m.cpu().numpy(), buf, "buf")
        assert np.array_equal(host_bits(d.w), oracle.decompress(got_p, h.idx, n))
    assert not d.v.any()                                    # the second Adam state is never touched


# ------------------------------------------------------------------ batched: DP-shaped split, statistics, guard
def _model(with_gc=True, specs=None):
    specs = specs or [(3 * 4096, 0.1, False), (1, 1.0, False), (5000, 0.0, False), (4097, 0.3, False), (100003, 0.05, False),
                      (30001, 1.0, True), (40000, 0.97, False)]
    hosts = [_layer(n, keep, 900 + i, dense) for i, (n, keep, dense) in enumerate(specs)]
    devs = [DevLayer(h, with_gc=with_gc, with_gc16=True) for h in hosts]
    return hosts, devs, samo.Plan([d.layer() for d in devs])


def _ref_stats(hosts, t, extra=None):
    total, bad = 0.0, False
    for i, h in enumerate(hosts):
        g = h.grads(t) if extra is None else extra[i]
        gc = oracle.gather(g, h.idx, INV)
        total += oracle.sum_squares(gc)
        bad |= oracle.has_nonfinite(gc)
    return total, bad


def test_a_model_that_keeps_under_seven_percent_is_cut_into_heavier_tiles():
    """Below 7 % kept overall a plan's tiles weigh twice as much (up to eleven segments, a larger LDS
    image): every tile kernel on such a plan, with a layer whose kept elements sit in a
    few dense stretches, an empty one and sizes that end inside a segment."""
    specs = [(200_003, 0.05, False), (9 * 1024, 0.0, False), (65_536, -0.03, False), (50_000, 0.06, False)]
    hosts, devs, plan = _model(specs=specs)
    n_total, nnz_total = plan.totals()
    assert nnz_total < 0.07 * n_total
    assert plan.num_tiles == sum(-(-(6144 * -(-h.n // 1024) + 24 * h.idx.shape[0]) // 65536) for h in hosts)
    for t in (1, 2, 3):
        for d, h in zip(devs, hosts):
            d.set_grads(h.grads(t))
            d.w.fill_(float("nan"))
        if t == 1:
            plan.samo_fused_step_batched(INV, samo.adam_cfg(t, **si.ADAM))
        elif t == 2:
            plan.samo_gather_fp16_batched(False, INV)
            plan.samo_adam_expand_batched(INV, samo.adam_cfg(t, **si.ADAM))
        else:
            plan.samo_gather_batched(INV)
            plan.samo_adam_batched(samo.adam_cfg(t, **si.ADAM))
            plan.samo_decompress_batched()
        for d, h in zip(devs, hosts):
            oracle.step(h.grads(t), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
            got_p = d.p.cpu().numpy()
            assert_close(got_p, h.p, "p t=%d" % t)
            assert_close(d.m.cpu().numpy(), h.m, "m t=%d" % t)
            assert_close(d.v.cpu().numpy(), h.v, "v t=%d" % t)
            assert np.array_equal(host_bits(d.w), oracle.decompress(got_p, h.idx, h.n)), "w t=%d" % t


@pytest.mark.parametrize("cost_k", [6, 20, 96])
def test_any_tile_weight_gives_the_same_model(cost_k):
    """The tuning aid SAMO_KNOB_TILE_COST: tiles of one segment, of the largest weight (sixteen segments, a
    32 KiB LDS image) and one in between; every tile kernel against the oracle."""
    samo.samo_debug_set(samo.KNOB_TILE_COST, cost_k)
    try:
        hosts, devs, plan = _model()
        for t in (1, 2):
            for d, h in zip(devs, hosts):
                d.set_grads(h.grads(t))
                d.w.fill_(float("nan"))
            if t == 1:
                plan.samo_fused_step_batched(INV, samo.adam_cfg(t, **si.ADAM))
            else:
                plan.samo_gather_fp16_batched(False, INV)
                plan.samo_adam_expand_batched(INV, samo.adam_cfg(t, **si.ADAM))
                for d in devs:
                    d.w.fill_(float("nan"))
                plan.samo_decompress_batched()
            for d, h in zip(devs, hosts):
                oracle.step(h.grads(t), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
                got_p = d.p.cpu().numpy()
                assert_close(got_p, h.p, "p t=%d" % t)
                assert_close(d.m.cpu().numpy(), h.m, "m t=%d" % t)
                assert_close(d.v.cpu().numpy(), h.v, "v t=%d" % t)
                assert np.array_equal(host_bits(d.w), oracle.decompress(got_p, h.idx, h.n)), "w t=%d" % t
    finally:
        samo.samo_debug_set(samo.KNOB_TILE_COST)


def test_dp_split_batched_with_statistics():
    hosts, devs, plan = _model()
    stats = samo.GradStats(plan)
    for t in (1, 2):
        for d, h in zip(devs, hosts):
            d.set_grads(h.grads(t))
            d.w.fill_(float("nan"))
        plan.samo_gather_fp16_batched(False, INV, stats)
        for d, h in zip(devs, hosts):
            assert np.array_equal(host_bits(d.gc16), oracle.compress_f16(h.grads(t), h.idx))
        ss, bad = stats.read()
        ref_ss, ref_bad = _ref_stats(hosts, t)
        assert abs(ss - ref_ss) <= 1e-12 * ref_ss and bad == ref_bad == False
        # the other two ways to the same statistics
        again = samo.GradStats(plan)
        plan.samo_grad_stats_batched(0, INV, again)
        assert again.read() == (ss, bad)                     # same partials, same order: same bits
        plan.samo_grad_stats_batched(1, INV, again)
        assert again.read() == (ss, bad)
        plan.samo_gather_batched(INV, again)
        assert again.read() == (ss, bad)
        plan.samo_grad_stats_batched(2, 1.0, again)
        assert again.read() == (ss, bad)
        plan.samo_adam_expand_batched(INV, samo.adam_cfg(t, **si.ADAM))
        for d, h in zip(devs, hosts):
            oracle.step(h.grads(t), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
            got_p = d.p.cpu().numpy()
            assert_close(got_p, h.p, "p")
            assert_close(d.m.cpu().numpy(), h.m, "m")
            assert_close(d.v.cpu().numpy(), h.v, "v")
            assert np.array_equal(host_bits(d.w), oracle.decompress(got_p, h.idx, h.n))


@pytest.mark.parametrize("n,keep", [(11_000_003, 0.25), (9_000_001, 0.13)])
def test_statistics_of_many_chunks(n, keep):
    """More chunk records than one reduction level takes, with a count that is not a multiple of
    eight (slots of the partials array stay unused), and a non-finite value in the last chunk."""
    mask = si.bernoulli_mask(n, keep, 4242)
    kept = np.flatnonzero(mask)
    chunks = -(-kept.shape[0] // 256)
    target = (chunks - 8) // 8 * 8 + 3                       # a count of chunk records that is 3 mod 8
    mask[kept[target * 256 - 100:]] = 0                      # ... the last of them ragged
    h = HostLayer(n, mask, si.weights(n, 4242), 4242)
    assert h.idx.shape[0] > 4 * 1024 * 256 and (-(-h.idx.shape[0] // 256)) % 8 == 3
    d = DevLayer(h, with_gc=True, with_gc16=True)
    plan = samo.Plan([d.layer()])
    stats = samo.GradStats(plan)
    g = h.grads(1)
    d.set_grads(g)
    gc = oracle.gather(g, h.idx, INV)
    ref_ss = oracle.sum_squares(gc)
    plan.samo_gather_fp16_batched(False, INV, stats)
    ss, bad = stats.read()
    # two fp64 summations of the same non-negative terms in different orders: each is within
    # (terms - 1) * 2^-53 relative of the exact sum
    assert abs(ss - ref_ss) <= 2 * gc.shape[0] * 2.0 ** -53 * ref_ss and not bad
    assert np.array_equal(host_bits(d.gc16), oracle.compress_f16(g, h.idx))
    again = samo.GradStats(plan)
    plan.samo_gather_batched(INV, again)
    assert again.read() == (ss, bad)
    assert np.array_equal(d.gc.cpu().numpy(), gc)
    g2 = g.copy()
    g2[h.idx[-1]] = 0x7C00                                   # +inf at the last kept position
    d.set_grads(g2)
    plan.samo_grad_stats_batched(0, INV, stats)
    assert stats.read()[1] is True


def test_compressed_fp16_gradients_of_all_layers_in_one_flat_bucket():
    """Section IV-A: the data-parallel all-reduce sends the compressed gradients as one message.
    alloc_model(bucket_gc16=True) lays every layer's gc16 out back to back in ONE buffer (slices on
    16-byte boundaries); after the batched gather (two micro-batches, the second accumulated) each
    slice equals the oracle's compressed gradient bit for bit and the padding is untouched, and the
    Adam + expand step that follows reads the bucket."""
    specs = [(3 * 4096, 0.1), (1, 1.0), (5003, 0.21), (4097, 0.3), (100003, 0.05), (40000, 0.97)]
    hosts = [_layer(n, keep, 950 + i) for i, (n, keep) in enumerate(specs)]
    built = [samo.samo_build_index(torch.from_numpy(h.mask).to(DEV)) for h in hosts]
    layers = samo.alloc_model([(h.n, h.idx.shape[0], False) for h in hosts], DEV, bucket_gc16=True)
    bucket = layers.gc16_bucket
    # one allocation, slices in layer order, each padded to a multiple of 8 halves
    at = 0
    for L, h in zip(layers, hosts):
        nnz = h.idx.shape[0]
        assert L.gc16.data_ptr() == bucket.data_ptr() + 2 * at and L.gc16.numel() == nnz
        assert L.gc16.data_ptr() % 16 == 0
        at += (nnz + 7) // 8 * 8
    assert bucket.numel() == at and bucket.is_contiguous()
    pad = torch.ones(at, dtype=torch.bool, device=DEV)
    for L in layers:
        pad[(L.gc16.data_ptr() - bucket.data_ptr()) // 2:][:L.gc16.numel()] = False
    bucket.view(torch.int16)[pad] = 0x1234                           # recognisable padding
    for L, h, ix in zip(layers, hosts, built):
        L.idx.copy_(ix.idx)
        L.seg_ptr.copy_(ix.seg_ptr)
        L.p.copy_(dev_f32(h.p))
    plan = samo.Plan(layers)
    refs = []
    for mb in (1, 2):
        for i, (L, h) in enumerate(zip(layers, hosts)):
            g = _wide_range_grads(h.n, 70 * mb + i)
            L.g.copy_(dev_f16_bits(g))
            if mb == 1:
                refs.append(oracle.compress_f16(g, h.idx))
            else:
                oracle.accumulate_f16(g, h.idx, refs[i])
        plan.samo_gather_fp16_batched(mb > 1, INV)
    whole = host_bits(bucket)
    for L, h, ref in zip(layers, hosts, refs):
        lo = (L.gc16.data_ptr() - bucket.data_ptr()) // 2
        assert np.array_equal(whole[lo:lo + ref.shape[0]], ref)
    assert bool((bucket.view(torch.int16)[pad] == 0x1234).all())
    plan.samo_adam_expand_batched(INV, samo.adam_cfg(1, **si.ADAM))
    for L, h, ref in zip(layers, hosts, refs):
        oracle.adam(h.p, h.m, h.v, oracle.upcast(ref, INV), OCFG, 1)
        got_p = L.p.cpu().numpy()
        assert_close(got_p, h.p, "p")
        assert_close(L.m.cpu().numpy(), h.m, "m")
        assert_close(L.v.cpu().numpy(), h.v, "v")
        assert np.array_equal(host_bits(L.w), oracle.decompress(got_p, h.idx, h.n))


def test_micro_batch_accumulation_batched():
    hosts, devs, plan = _model()
    refs = [None] * len(hosts)
    for mb in (1, 2, 3):
        for i, (d, h) in enumerate(zip(devs, hosts)):
            g = _wide_range_grads(h.n, 50 * mb + i)
            d.set_grads(g)
            if mb == 1:
                refs[i] = oracle.compress_f16(g, h.idx)
            else:
                oracle.accumulate_f16(g, h.idx, refs[i])
        plan.samo_gather_fp16_batched(mb > 1, INV)
        for d, ref in zip(devs, refs):
            assert np.array_equal(host_bits(d.gc16), ref)


@pytest.mark.parametrize("entry", ["adam_expand", "fused", "adam"])
@pytest.mark.parametrize("max_norm", [0.05, 1e6])
def test_clipping_by_global_norm(entry, max_norm):
    hosts, devs, plan = _model()
    stats = samo.GradStats(plan)
    for d, h in zip(devs, hosts):
        d.set_grads(h.grads(1))
    cfg = samo.adam_cfg(1, **si.ADAM)
    if entry == "adam_expand":
        plan.samo_gather_fp16_batched(False, INV, stats)
        plan.samo_adam_expand_batched(INV, cfg, stats.guard(max_grad_norm=max_norm))
    elif entry == "fused":
        plan.samo_grad_stats_batched(0, INV, stats)
        plan.samo_fused_step_batched(INV, cfg, stats.guard(max_grad_norm=max_norm))
    else:
        plan.samo_gather_batched(INV, stats)
        plan.samo_adam_batched(cfg, stats.guard(max_grad_norm=max_norm))
        plan.samo_decompress_batched()
    total, _ = _ref_stats(hosts, 1)
    coef = oracle.clip_coefficient(total, max_norm)
    assert (coef < 1.0) == (max_norm < np.sqrt(total))
    for d, h in zip(devs, hosts):
        gc = oracle.gather(h.grads(1), h.idx, INV)
        oracle.scale(gc, coef)
        oracle.adam(h.p, h.m, h.v, gc, OCFG, 1)
        got_p = d.p.cpu().numpy()
        assert_close(got_p, h.p, "p")
        assert_close(d.m.cpu().numpy(), h.m, "m")
        assert_close(d.v.cpu().numpy(), h.v, "v")
        assert np.array_equal(host_bits(d.w), oracle.decompress(got_p, h.idx, h.n))


@pytest.mark.parametrize("entry", ["adam_expand", "fused", "sgd"])
def test_overflow_skips_the_step_and_pruned_garbage_does_not(entry):
    hosts, devs, plan = _model()
    stats = samo.GradStats(plan)
    cfg = samo.adam_cfg(1, **si.ADAM)

    def run(grads):
        for d, g in zip(devs, grads):
            d.set_grads(g)
        if entry == "adam_expand":
            plan.samo_gather_fp16_batched(False, INV, stats)
            plan.samo_adam_expand_batched(INV, cfg, stats.guard(skip_on_nonfinite=True))
        elif entry == "fused":
            plan.samo_grad_stats_batched(0, INV, stats)
            plan.samo_fused_step_batched(INV, cfg, stats.guard(skip_on_nonfinite=True))
        else:
            plan.samo_grad_stats_batched(0, INV, stats)
            plan.samo_fused_sgd_step_batched(INV, samo.sgd_cfg(0.1), stats.guard(skip_on_nonfinite=True))

    plan.samo_decompress_batched()
    before = [(d.p.clone(), d.m.clone(), d.v.clone(), d.w.view(torch.int16).clone()) for d in devs]
    # an infinity at a KEPT position of one layer: the whole model's step is skipped
    grads = [h.grads(1) for h in hosts]
    grads[4] = grads[4].copy()
    grads[4][hosts[4].idx[17]] = 0x7C00
    run(grads)
    ss, bad = stats.read()
    assert bad and _ref_stats(hosts, 1, grads)[1]
    for d, (p, m, v, w) in zip(devs, before):
        assert torch.equal(d.p, p) and torch.equal(d.m, m) and torch.equal(d.v, v)
        assert torch.equal(d.w.view(torch.int16), w)
    # NaN / inf only at PRUNED positions: not an overflow, the step runs
    grads = [h.grads(1) for h in hosts]
    grads[4] = grads[4].copy()
    grads[4][hosts[4].mask == 0] = 0x7E00
    run(grads)
    ss, bad = stats.read()
    assert not bad and np.isfinite(ss)
    assert not torch.equal(devs[4].p, before[4][0])


def test_fused_sgd_step_batched_matches_oracle():
    hosts, devs, plan = _model()
    for t in (1, 2):
        for d, h in zip(devs, hosts):
            d.set_grads(h.grads(t))
            d.w.fill_(float("nan"))
        plan.samo_fused_sgd_step_batched(INV, samo.sgd_cfg(0.05, 0.9, 1e-4))
        for d, h in zip(devs, hosts):
            oracle.sgd(h.p, h.m, oracle.gather(h.grads(t), h.idx, INV), 0.05, 0.9, 1e-4)
            got_p = d.p.cpu().numpy()
            assert_close(got_p, h.p, "p")
            assert_close(d.m.cpu().numpy(), h.m, "buf")
            assert np.array_equal(host_bits(d.w), oracle.decompress(got_p, h.idx, h.n))


def test_statistics_need_their_workspace():
    hosts, devs, plan = _model()
    stats = samo.GradStats(plan)
    small = torch.empty(8, dtype=torch.uint8, device=DEV)
    rc = samo.lib().samo_grad_stats_batched(plan._handle, 0, 1.0, stats.ptr, small.data_ptr(), small.numel(), None)
    assert rc == samo.SAMO_ERR_WORKSPACE
    rc = samo.lib().samo_fused_step_batched(plan._handle, 1.0, samo.adam_cfg(1), samo.StepGuard(None, 1.0, 0), None)
    assert rc == samo.SAMO_ERR_NULL                        # clipping asked for without statistics
