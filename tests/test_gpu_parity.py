"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.
Bit-exact for index construction, expansion and gradient compression; <= 1e-6 relative for
the fp32 Adam state (see gpu_util.assert_close)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import (DEV, INV, OCFG, DevLayer, HostLayer, assert_close, dev_f16_bits, dev_f32, dev_i32, dev_u8,
                      host_bits, nan_f16, ref_seg_ptr)

pytestmark = pytest.mark.gpu

SIZES = [1, 15, 16, 17, 63, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 8192, 8193, 3 * 8192 + 777, 100003]


def _layer(n, keep, seed):
    return HostLayer(n, si.bernoulli_mask(n, keep, seed), si.weights(n, seed), seed)


# ------------------------------------------------------------------ a0: index construction
@pytest.mark.parametrize("n", SIZES)
def test_build_index_edge_masks(n):
    masks = dict(si.edge_masks(n))
    masks["bernoulli_0.1"] = si.bernoulli_mask(n, 0.1, n)
    masks["bernoulli_0.9"] = si.bernoulli_mask(n, 0.9, n + 1)
    for name, mask in masks.items():
        ref = oracle.build_index(mask)
        ix = samo.samo_build_index(dev_u8(mask))
        assert ix.nnz == ref.shape[0], name
        assert np.array_equal(ix.idx.cpu().numpy(), ref), name
        assert np.array_equal(ix.seg_ptr.cpu().numpy(), ref_seg_ptr(ref, n)), name
        assert samo.samo_validate_index(ix.idx, n, ix.seg_ptr), name


def test_build_index_config1_and_determinism():
    spec = si.config("fc1024")[0]
    mask = si.make_mask(spec, None)
    ref = oracle.build_index(mask)
    d_mask = dev_u8(mask)
    a = samo.samo_build_index(d_mask)
    b = samo.samo_build_index(d_mask)
    assert np.array_equal(a.idx.cpu().numpy(), ref)
    assert torch.equal(a.idx, b.idx) and torch.equal(a.seg_ptr, b.seg_ptr)


@pytest.mark.parametrize("n,keep", [(3_000_001, 0.1), (1024 * 1024 * 5 + 1, 0.5), (2_100_000, 0.999)])
def test_build_index_many_segments(n, keep):
    # more segments than scan threads: every thread of the scan owns a run of several entries
    mask = si.bernoulli_mask(n, keep, n % 1000)
    ref = oracle.build_index(mask)
    ix = samo.samo_build_index(dev_u8(mask))
    assert ix.nnz == ref.shape[0]
    assert np.array_equal(ix.idx.cpu().numpy(), ref)
    assert np.array_equal(ix.seg_ptr.cpu().numpy(), ref_seg_ptr(ref, n))


@pytest.mark.parametrize("passes", [1, 2, 4])
def test_build_index_every_block_size(passes):
    """A workgroup takes 64, 128 or 256 KiB of mask (one, two or four passes; the library picks by the
    launch's size): each forced here on layers of less than a block, exactly one block, a block and a
    bit, and many blocks with a ragged end, alone and as one batched call, with an index capacity that
    is too small on one of them."""
    block = 65536 * passes
    sizes = [1, 1025, block - 1, block, block + 1, 3 * block + 17 * 1024 + 5, 40 * block + 123457]
    masks = [si.bernoulli_mask(n, keep, 40 + i) for i, (n, keep) in enumerate(zip(sizes, [1.0, 0.5, 0.1, 0.03, 0.9, 0.2, 0.1]))]
    refs = [oracle.build_index(m) for m in masks]
    samo.samo_debug_set(samo.KNOB_INDEX_PASSES, passes)
    try:
        for mask, ref in zip(masks, refs):
            ix = samo.samo_build_index(dev_u8(mask))
            assert ix.nnz == ref.shape[0]
            assert np.array_equal(ix.idx.cpu().numpy(), ref)
            assert np.array_equal(ix.seg_ptr.cpu().numpy(), ref_seg_ptr(ref, mask.shape[0]))
        got = samo.samo_build_index_many([dev_u8(m) for m in masks])
        for ix, mask, ref in zip(got, masks, refs):
            assert np.array_equal(ix.idx.cpu().numpy(), ref)
            assert np.array_equal(ix.seg_ptr.cpu().numpy(), ref_seg_ptr(ref, mask.shape[0]))
        # capacity too small: the count is still the true one, nothing is stored beyond the capacity
        mask, ref = masks[-2], refs[-2]
        cap = ref.shape[0] // 2
        idx = torch.full((cap + 64,), -5, dtype=torch.int32, device=DEV)
        seg = torch.empty(samo.samo_seg_ptr_len(mask.shape[0]), dtype=torch.int32, device=DEV)
        nnz = torch.zeros(1, dtype=torch.int64, device=DEV)
        samo.samo_build_index_into(dev_u8(mask), idx[:cap], seg, nnz)
        assert int(nnz.item()) == ref.shape[0]
        assert np.array_equal(idx[:cap].cpu().numpy(), ref[:cap]) and bool((idx[cap:] == -5).all())
    finally:
        samo.samo_debug_set(samo.KNOB_INDEX_PASSES)


def test_build_index_batched_many_jobs():
    # more jobs than one launch group holds (48), with empty, tiny, ragged and multi-segment layers
    rng = np.random.default_rng(7)
    sizes = [0, 1, 15, 16, 1023, 1024, 1025, 4097, 70001, 300007] + [int(x) for x in rng.integers(1, 20000, 95)]
    masks = [si.bernoulli_mask(n, float(rng.uniform(0.0, 1.0)), 900 + i) for i, n in enumerate(sizes)]
    got = samo.samo_build_index_many([dev_u8(m) for m in masks])
    assert len(got) == len(masks) == 105
    for ix, mask in zip(got, masks):
        ref = oracle.build_index(mask)
        assert ix.nnz == ref.shape[0] and ix.n == mask.shape[0]
        assert np.array_equal(ix.idx.cpu().numpy(), ref)
        assert np.array_equal(ix.seg_ptr.cpu().numpy(), ref_seg_ptr(ref, mask.shape[0]))
    assert samo.samo_build_index_many([]) == []


def test_build_index_gives_up_cleanly_when_the_wait_is_cut_short():
    """With no patience at all for a predecessor, a workgroup gives up instead of waiting: the
    call must still end, and report either the right index or the failure — never a wrong one.
    The layer is 611 blocks, more than two per compute unit: the workgroups that start together
    cannot all find their predecessor's count published at their first look, so the give-up path
    is taken in at least one of the three builds."""
    n = 40_000_003
    mask = si.bernoulli_mask(n, 0.1, 31)
    d_mask = dev_u8(mask)
    outcomes = set()
    samo.samo_debug_set(samo.KNOB_INDEX_SPIN_LIMIT, 0)
    try:
        for _ in range(3):
            try:
                ix = samo.samo_build_index(d_mask)
                assert np.array_equal(ix.idx.cpu().numpy(), oracle.build_index(mask))
                outcomes.add("ok")
            except samo.SamoError as e:
                assert e.status == samo.SAMO_ERR_INDEX
                outcomes.add("gave up")
    finally:
        samo.samo_debug_set(samo.KNOB_INDEX_SPIN_LIMIT)
    assert "gave up" in outcomes
    ix = samo.samo_build_index(d_mask)                  # and the library is fine afterwards
    assert np.array_equal(ix.idx.cpu().numpy(), oracle.build_index(mask))


def test_build_index_empty_layer():
    ix = samo.samo_build_index(torch.empty(0, dtype=torch.uint8, device=DEV))
    assert ix.nnz == 0 and ix.seg_ptr.cpu().tolist() == [0]


def test_build_index_capacity_too_small_reports_true_count():
    n = 50000
    mask = si.bernoulli_mask(n, 0.5, 3)
    ref = oracle.build_index(mask)
    cap = 1000
    idx = torch.full((cap + 64,), -7, dtype=torch.int32, device=DEV)
    seg_ptr = torch.empty(samo.samo_seg_ptr_len(n), dtype=torch.int32, device=DEV)
    nnz = torch.zeros(1, dtype=torch.int64, device=DEV)
    samo.samo_build_index_into(dev_u8(mask), idx[:cap], seg_ptr, nnz)
    assert int(nnz.item()) == ref.shape[0]
    got = idx.cpu().numpy()
    assert np.array_equal(got[:cap], ref[:cap])
    assert np.all(got[cap:] == -7)                      # nothing stored beyond the capacity


def test_seg_ptr_from_foreign_index_and_validation():
    n = 70001
    mask = si.bernoulli_mask(n, 0.07, 5)
    ref = oracle.build_index(mask)
    d_idx = dev_i32(ref)
    seg_ptr = samo.samo_build_seg_ptr(d_idx, n)
    assert np.array_equal(seg_ptr.cpu().numpy(), ref_seg_ptr(ref, n))
    assert samo.samo_validate_index(d_idx, n, seg_ptr)
    assert samo.samo_validate_index(d_idx, n)
    bad = ref.copy()
    bad[100], bad[101] = bad[101], bad[100]             # not ascending
    assert not samo.samo_validate_index(dev_i32(bad), n)
    dup = ref.copy()
    dup[7] = dup[6]                                     # duplicate
    assert not samo.samo_validate_index(dev_i32(dup), n)
    assert not samo.samo_validate_index(d_idx, int(ref[-1]))          # out of range
    wrong = seg_ptr.clone()
    wrong[3] += 1
    assert not samo.samo_validate_index(d_idx, n, wrong)


# ------------------------------------------------------------------ a1: expansion
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("keep", [0.0, 0.1, 0.5, 1.0])
def test_decompress_bit_exact(n, keep):
    h = _layer(n, keep, 100 + n)
    d = DevLayer(h)
    samo.samo_decompress(d.p, d.idx, d.seg_ptr, d.w)
    assert np.array_equal(host_bits(d.w), oracle.decompress(h.p, h.idx, n))


def test_decompress_special_values():
    # subnormal halves, ties, overflow to infinity, signed zeros, NaN
    vals = np.array([0.0, -0.0, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, -(2.0 ** -26), 2.0 ** -14, 6e-5, -6e-8,
                     65504.0, 65519.996, 65520.0, -1e9, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, np.inf, -np.inf,
                     1e-45, 1.17e-38], np.float32)
    n = 5000
    idx = (np.arange(vals.shape[0], dtype=np.int32) * 257 + 3)
    d_idx = dev_i32(idx)
    w = nan_f16(n)
    samo.samo_decompress(dev_f32(vals), d_idx, samo.samo_build_seg_ptr(d_idx, n), w)
    assert np.array_equal(host_bits(w), oracle.decompress(vals, idx, n))
    nan_p = np.array([np.nan], np.float32)
    d_idx = dev_i32(np.array([9], np.int32))
    samo.samo_decompress(dev_f32(nan_p), d_idx, samo.samo_build_seg_ptr(d_idx, 16), w[:16])
    got = host_bits(w[:16])
    assert (got[9] & 0x7C00) == 0x7C00 and (got[9] & 0x3FF) != 0 and not np.delete(got, 9).any()


def test_config1_exercises_subnormal_halves():
    spec = si.config("fc1024")[0]
    data = si.make_layer(spec)
    h = HostLayer(spec.n, data.mask, data.w32, spec.seed)
    d = DevLayer(h)
    samo.samo_decompress(d.p, d.idx, d.seg_ptr, d.w)
    bits = host_bits(d.w)
    assert np.array_equal(bits, oracle.decompress(h.p, h.idx, spec.n))
    kept = bits[h.idx]
    assert np.count_nonzero(((kept & 0x7C00) == 0) & ((kept & 0x3FF) != 0)) > 50


# ------------------------------------------------------------------ a2: gradient compression
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("inv", [INV, 1.0, 1.0 / 3.0])
def test_gather_bit_exact(n, inv):
    h = _layer(n, 0.13, 200 + n)
    g = h.grads(1)
    gc = torch.full((h.idx.shape[0],), float("nan"), device=DEV)
    samo.samo_gather_grads(dev_f16_bits(g), dev_i32(h.idx), inv, gc)
    ref = oracle.gather(g, h.idx, inv)
    assert np.array_equal(gc.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_gather_ignores_pruned_positions_and_keeps_subnormals():
    n = 20000
    h = _layer(n, 0.2, 31)
    g = h.grads(1)
    g[h.idx[:6]] = np.array([0x0001, 0x8001, 0x03FF, 0x8000, 0x0000, 0x7BFF], np.uint16)
    poisoned = g.copy()
    poisoned[h.mask == 0] = 0x7E00
    gc = torch.empty(h.idx.shape[0], device=DEV)
    samo.samo_gather_grads(dev_f16_bits(poisoned), dev_i32(h.idx), 1.0, gc)
    assert np.array_equal(gc.cpu().numpy().view(np.uint32), oracle.gather(g, h.idx, 1.0).view(np.uint32))


# ------------------------------------------------------------------ a3: compressed Adam
@pytest.mark.parametrize("nnz", [1, 3, 4, 5, 255, 256, 257, 1023, 2048, 2049, 100003])
@pytest.mark.parametrize("wd,decoupled", [(0.0, 0), (0.1, 0), (0.1, 1)])
def test_adam_within_tolerance(nnz, wd, decoupled):
    rng = np.random.default_rng(nnz)
    p = si.weights(nnz, nnz)
    m = (rng.standard_normal(nnz) * 1e-3).astype(np.float32)
    v = (rng.standard_normal(nnz) ** 2 * 1e-6).astype(np.float32)
    d_p, d_m, d_v = dev_f32(p), dev_f32(m), dev_f32(v)
    ocfg = OCFG._replace(weight_decay=wd, decoupled_wd=decoupled)
    for t in (1, 2, 7):
        gc = (rng.standard_normal(nnz) * 1e-3).astype(np.float32)
        samo.samo_adam_step(d_p, d_m, d_v, dev_f32(gc), samo.adam_cfg(t, **ocfg._asdict()))
        oracle.adam(p, m, v, gc, ocfg, t)
        assert_close(d_p.cpu().numpy(), p, "p t=%d" % t)
        assert_close(d_m.cpu().numpy(), m, "m t=%d" % t)
        assert_close(d_v.cpu().numpy(), v, "v t=%d" % t)


def test_adam_zero_gradient_keeps_zero_state():
    nnz = 4096
    p = si.weights(nnz, 1)
    d_p, d_m, d_v = dev_f32(p), dev_f32(np.zeros(nnz)), dev_f32(np.zeros(nnz))
    samo.samo_adam_step(d_p, d_m, d_v, dev_f32(np.zeros(nnz)), samo.adam_cfg(1, **si.ADAM))
    assert np.array_equal(d_p.cpu().numpy(), p) and not d_m.any() and not d_v.any()


# ------------------------------------------------------------------ a4: fused optimizer phase, config 1
def _check_fused_outputs(d, h, n, t):
    got_p = d.p.cpu().numpy()
    assert_close(got_p, h.p, "p t=%d" % t)
    assert_close(d.m.cpu().numpy(), h.m, "m t=%d" % t)
    assert_close(d.v.cpu().numpy(), h.v, "v t=%d" % t)
    # the dense fp16 weights are exactly the expansion of the GPU's own fp32 parameters ...
    w_bits = host_bits(d.w)
    assert np.array_equal(w_bits, oracle.decompress(got_p, h.idx, n)), "w t=%d" % t
    # ... and pruned positions are +0 bit patterns
    assert not w_bits[h.mask == 0].any()


def test_config1_three_steps_fused_and_unfused():
    spec = si.config("fc1024")[0]
    data = si.make_layer(spec)
    h = HostLayer(spec.n, data.mask, data.w32, spec.seed)
    fused, unfused = DevLayer(h), DevLayer(h, with_gc=True)
    for t in (1, 2, 3):
        g = h.grads(t)
        cfg = samo.adam_cfg(t, **si.ADAM)
        fused.w.fill_(float("nan"))
        fused.set_grads(g)
        samo.samo_fused_step(fused.g, fused.w, fused.idx, fused.seg_ptr, fused.p, fused.m, fused.v, INV, cfg)
        unfused.w.fill_(float("nan"))
        unfused.set_grads(g)
        samo.samo_gather_grads(unfused.g, unfused.idx, INV, unfused.gc)
        samo.samo_adam_step(unfused.p, unfused.m, unfused.v, unfused.gc, cfg)
        samo.samo_decompress(unfused.p, unfused.idx, unfused.seg_ptr, unfused.w)
        oracle.step(g, spec.n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
        _check_fused_outputs(fused, h, spec.n, t)
        _check_fused_outputs(unfused, h, spec.n, t)
        # same arithmetic in both paths of the library: identical bits
        for a, b in ((fused.p, unfused.p), (fused.m, unfused.m), (fused.v, unfused.v)):
            assert torch.equal(a, b)
        assert np.array_equal(host_bits(fused.w), host_bits(unfused.w))


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("keep", [0.0, 0.05, 0.5, 1.0])
def test_fused_step_ragged_sizes(n, keep):
    h = _layer(n, keep, 300 + n)
    d = DevLayer(h)
    for t in (1, 2):
        g = h.grads(t)
        d.w.fill_(float("nan"))
        d.set_grads(g)
        samo.samo_fused_step(d.g, d.w, d.idx, d.seg_ptr, d.p, d.m, d.v, INV, samo.adam_cfg(t, **si.ADAM))
        oracle.step(g, n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
        _check_fused_outputs(d, h, n, t)


@pytest.mark.parametrize("n", [1, 7, 8, 9, 4095, 4096, 4104, 8191, 8192, 8200, 50001])
def test_dense_layer_fused_and_decompress(n):
    h = HostLayer(n, np.ones(n, np.uint8), si.weights(n, n), 400 + n, dense=True)
    d = DevLayer(h)
    samo.samo_decompress(d.p, None, None, d.w)
    assert np.array_equal(host_bits(d.w), oracle.decompress(h.p, h.idx, n))
    for t in (1, 2):
        g = h.grads(t)
        d.w.fill_(float("nan"))
        d.set_grads(g)
        samo.samo_fused_step(d.g, d.w, None, None, d.p, d.m, d.v, INV, samo.adam_cfg(t, **si.ADAM))
        oracle.step(g, n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
        _check_fused_outputs(d, h, n, t)


def test_fused_step_is_deterministic():
    h = _layer(200000, 0.1, 77)
    outs = []
    for _ in range(2):
        d = DevLayer(h)
        d.set_grads(h.grads(1))
        samo.samo_fused_step(d.g, d.w, d.idx, d.seg_ptr, d.p, d.m, d.v, INV, samo.adam_cfg(1, **si.ADAM))
        outs.append((d.p.clone(), d.m.clone(), d.v.clone(), d.w.view(torch.int16).clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# ------------------------------------------------------------------ batched forms
def _mixed_model():
    specs = [(8192 * 3, 0.1), (1, 1.0), (5000, 0.0), (8193, 0.3), (100003, 0.05), (1024, 0.5), (40000, 0.97)]
    layers = [_layer(n, keep, 500 + i) for i, (n, keep) in enumerate(specs)]
    n = 30001
    layers.insert(3, HostLayer(n, np.ones(n, np.uint8), si.weights(n, 599), 599, dense=True))
    return layers


def test_batched_entries_match_oracle():
    hosts = _mixed_model()
    devs = [DevLayer(h, with_gc=True) for h in hosts]
    plan = samo.Plan([d.layer() for d in devs])
    assert plan.totals() == (sum(h.n for h in hosts), sum(h.idx.shape[0] for h in hosts))

    plan.samo_decompress_batched()
    for d, h in zip(devs, hosts):
        assert np.array_equal(host_bits(d.w), oracle.decompress(h.p, h.idx, h.n))

    # unfused batched step 1, fused batched step 2
    for d, h in zip(devs, hosts):
        d.set_grads(h.grads(1))
        d.w.fill_(float("nan"))
    plan.samo_gather_batched(INV)
    for d, h in zip(devs, hosts):
        assert np.array_equal(d.gc.cpu().numpy().view(np.uint32), oracle.gather(h.grads(1), h.idx, INV).view(np.uint32))
    plan.samo_adam_batched(samo.adam_cfg(1, **si.ADAM))
    plan.samo_decompress_batched()
    for d, h in zip(devs, hosts):
        oracle.step(h.grads(1), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, 1)
        _check_fused_outputs(d, h, h.n, 1)

    for d, h in zip(devs, hosts):
        d.set_grads(h.grads(2))
        d.w.fill_(float("nan"))
    plan.samo_fused_step_batched(INV, samo.adam_cfg(2, **si.ADAM))
    for d, h in zip(devs, hosts):
        oracle.step(h.grads(2), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, 2)
        _check_fused_outputs(d, h, h.n, 2)
    plan.close()


def _uneven_masks():
    """Masks whose local density swings between nothing kept and everything kept, so that a
    plan's tiles range from one segment to the largest a workgroup takes."""
    rng = np.random.default_rng(77)
    out = []
    n = 300_007                                          # long empty and full stretches, ragged end
    m = np.zeros(n, np.uint8)
    m[20_000:29_000] = 1
    m[100_000:100_003] = 1
    m[150_001:260_000] = rng.random(109_999) < 0.5
    m[-5:] = 1
    out.append(m)
    out.append(si.row_clustered_mask(96, 4096, 0.9, 5))  # hot rows 10x denser than the rest
    out.append(si.row_clustered_mask(40, 3000, 0.8, 6))  # rows that do not line up with segments
    out.append(np.ones(70_001, np.uint8))                # everything kept, through the index
    out.append(np.zeros(50_000, np.uint8))               # nothing kept
    return out


def test_plan_tiles_follow_local_density():
    hosts = [HostLayer(m.shape[0], m, si.weights(m.shape[0], 700 + i), 700 + i) for i, m in enumerate(_uneven_masks())]
    devs = [DevLayer(h, with_gc16=True) for h in hosts]
    plan = samo.Plan([d.layer() for d in devs])
    plan.samo_decompress_batched()
    for d, h in zip(devs, hosts):
        assert np.array_equal(host_bits(d.w), oracle.decompress(h.p, h.idx, h.n))
    for t in (1, 2):
        for d, h in zip(devs, hosts):
            d.set_grads(h.grads(t))
            d.w.fill_(float("nan"))
        if t == 1:
            plan.samo_fused_step_batched(INV, samo.adam_cfg(t, **si.ADAM))
        else:                                            # the split form walks the same tiles
            plan.samo_gather_fp16_batched(False, INV)
            plan.samo_adam_expand_batched(INV, samo.adam_cfg(t, **si.ADAM))
        for d, h in zip(devs, hosts):
            oracle.step(h.grads(t), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, t)
            _check_fused_outputs(d, h, h.n, t)
    plan.close()


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_plan_tiles_cover_random_piecewise_masks(seed):
    """Many layers of random size whose density jumps between stretches (nothing, a few, half, all
    kept): whatever the cut into tiles, every segment must be expanded and updated exactly once."""
    rng = np.random.default_rng(1000 + seed)
    hosts = []
    for i in range(24):
        n = int(rng.choice([1, 7, 1023, 1024, 1025, 5000, 33_333, 70_000, 200_001]))
        mask = np.zeros(n, np.uint8)
        lo = 0
        while lo < n:
            hi = min(n, lo + int(rng.integers(1, 20_000)))
            d = float(rng.choice([0.0, 0.003, 0.05, 0.5, 1.0]))
            mask[lo:hi] = rng.random(hi - lo) < d
            lo = hi
        hosts.append(HostLayer(n, mask, si.weights(n, 3000 + 100 * seed + i), 3000 + 100 * seed + i))
    devs = [DevLayer(h) for h in hosts]
    plan = samo.Plan([d.layer() for d in devs])
    plan.samo_decompress_batched()
    for d, h in zip(devs, hosts):
        assert np.array_equal(host_bits(d.w), oracle.decompress(h.p, h.idx, h.n))
    for d, h in zip(devs, hosts):
        d.set_grads(h.grads(1))
        d.w.fill_(float("nan"))
    plan.samo_fused_step_batched(INV, samo.adam_cfg(1, **si.ADAM))
    for d, h in zip(devs, hosts):
        oracle.step(h.grads(1), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, 1)
        _check_fused_outputs(d, h, h.n, 1)
    plan.close()


def test_checkpoint_resume_from_the_compressed_state(tmp_path):
    """The compressed state (idx, p, m, v and the step counter) is the whole checkpoint: theta16 is
    recomputed by expansion, seg_ptr from idx, and training continues bit for bit."""
    h = _layer(150_001, 0.1, 61)
    d = DevLayer(h)
    for t in (1, 2):
        d.set_grads(h.grads(t))
        samo.samo_fused_step(d.g, d.w, d.idx, d.seg_ptr, d.p, d.m, d.v, INV, samo.adam_cfg(t, **si.ADAM))
    path = tmp_path / "ckpt.npz"
    np.savez(path, idx=d.idx.cpu().numpy(), p=d.p.cpu().numpy(), m=d.m.cpu().numpy(), v=d.v.cpu().numpy(), t=2, n=h.n)
    w_before = host_bits(d.w).copy()
    d.set_grads(h.grads(3))
    samo.samo_fused_step(d.g, d.w, d.idx, d.seg_ptr, d.p, d.m, d.v, INV, samo.adam_cfg(3, **si.ADAM))

    ck = np.load(path)
    n = int(ck["n"])
    idx = dev_i32(ck["idx"])
    seg_ptr = samo.samo_build_seg_ptr(idx, n)
    assert samo.samo_validate_index(idx, n, seg_ptr)
    p, m, v = dev_f32(ck["p"]), dev_f32(ck["m"]), dev_f32(ck["v"])
    w = nan_f16(n)
    samo.samo_decompress(p, idx, seg_ptr, w)
    assert np.array_equal(host_bits(w), w_before)                 # theta16 is recomputable
    g = nan_f16(n)
    g.copy_(dev_f16_bits(h.grads(3)))
    samo.samo_fused_step(g, w, idx, seg_ptr, p, m, v, INV, samo.adam_cfg(int(ck["t"]) + 1, **si.ADAM))
    assert torch.equal(p, d.p) and torch.equal(m, d.m) and torch.equal(v, d.v)
    assert torch.equal(w.view(torch.int16), d.w.view(torch.int16))


def test_plan_reports_missing_buffers():
    h = _layer(5000, 0.2, 9)
    d = DevLayer(h)                                     # no gc
    plan = samo.Plan([d.layer()])
    with pytest.raises(samo.SamoError) as e:
        plan.samo_gather_batched(INV)
    assert e.value.status == samo.SAMO_ERR_PLAN
    plan.samo_fused_step_batched(INV, samo.adam_cfg(1, **si.ADAM))     # has all it needs
    torch.cuda.synchronize()


def test_empty_plan_is_a_no_op():
    plan = samo.Plan([])
    plan.samo_fused_step_batched(INV, samo.adam_cfg(1, **si.ADAM))
    plan.samo_decompress_batched()
    assert plan.totals() == (0, 0)


def test_stream_copy():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    samo.samo_stream_copy(dst, src)
    assert torch.equal(dst, src)
    dst2 = torch.zeros(1000, dtype=torch.int32, device=DEV)
    samo.samo_stream_copy(dst2, src[:1000])
    assert torch.equal(dst2, src[:1000])


def test_mfma_rate_probe_runs_and_counts_its_flops():
    """The measurement aid beside the weight-gradient kernels: every workgroup does the same work, the
    accumulated value grows with the iteration count, and the reported flops are those of the launch."""
    sink = torch.zeros(5, dtype=torch.float32, device=DEV)
    assert samo.samo_mfma_rate_probe(1, sink) == 5 * 8 * 8 * 2.0 * 32 * 32 * 16
    one = sink.cpu().numpy().copy()
    assert np.all(np.isfinite(one)) and one[0] != 0.0 and np.all(one == one[0])
    assert samo.samo_mfma_rate_probe(64, sink) == 64 * 5 * 8 * 8 * 2.0 * 32 * 32 * 16
    many = sink.cpu().numpy()
    assert np.all(many == many[0]) and abs(many[0] - 64 * one[0]) <= 1e-4 * abs(64 * one[0])
    assert samo.samo_mfma_rate_probe(0, sink[:0]) == 0.0


def test_runs_on_a_side_stream():
    h = _layer(300000, 0.1, 55)
    d = DevLayer(h)
    d.set_grads(h.grads(1))
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        samo.samo_fused_step(d.g, d.w, d.idx, d.seg_ptr, d.p, d.m, d.v, INV, samo.adam_cfg(1, **si.ADAM))
    s.synchronize()
    oracle.step(h.grads(1), h.n, h.idx, h.p, h.m, h.v, INV, OCFG, 1)
    _check_fused_outputs(d, h, h.n, 1)
