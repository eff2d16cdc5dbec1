"""GPU parity of the weight gradient formed and compressed in one kernel (compression fused into
the backward pass: Section III-C, and Section VI-C on its compute overhead) against the
CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import DEV, dev_f16_bits, dev_i32, host_bits, ref_seg_ptr

pytestmark = pytest.mark.gpu

# (tokens, out, in): single blocks, ragged tails in every direction, several tiles of either shape,
# one to fourteen stages of 32 tokens, one to seven of 64 (the ring's start-up, wrap-around and drain), with and without a tail
SHAPES = [(1, 8, 8), (7, 8, 16), (31, 16, 8), (32, 24, 40), (33, 136, 264), (100, 256, 512),
          (64, 384, 520), (257, 128, 256), (96, 264, 776), (45, 520, 72), (130, 520, 528),
          (64, 8, 8), (65, 16, 16), (128, 264, 8), (160, 8, 264), (289, 24, 24), (421, 264, 520)]


def _mask(kind, out_f, in_f, seed):
    n = out_f * in_f
    if kind == "bernoulli10":
        return si.bernoulli_mask(n, 0.1, seed)
    if kind == "bernoulli50":
        return si.bernoulli_mask(n, 0.5, seed)
    if kind == "rows":
        return si.row_clustered_mask(out_f, in_f, 0.8, seed)
    if kind == "edges":                       # first and last element of every row, nothing else
        m = np.zeros((out_f, in_f), np.uint8)
        m[:, 0] = 1
        m[:, -1] = 1
        return m.reshape(-1)
    if kind == "dense_idx":                   # every element kept, with an explicit index
        return np.ones(n, np.uint8)
    raise KeyError(kind)


def _bracket(dy, x, tokens, out_f, in_f, idx):
    """fp16 bit patterns between which a result must lie: the exact sum moved down and up by the
    worst rounding error of tokens fp32 additions in any order (2^-23 of the magnitude sum per
    addition covers truncating adders too), each rounded to fp16 — rounding is monotonic."""
    exact = oracle.linear_weight_grad(dy, x, tokens, out_f, in_f)[idx]
    mag = oracle.linear_weight_grad_magnitude(dy, x, tokens, out_f, in_f)[idx]
    slack = (tokens + 2) * 2.0 ** -23 * mag
    with np.errstate(over="ignore"):
        return (exact - slack).astype(np.float16), (exact + slack).astype(np.float16)


def _check_f16(got_bits, lo, hi, want_bits, what):
    got = got_bits.view(np.float16)
    bad = ~((got >= lo) & (got <= hi))
    assert not bad.any(), "%s: %d of %d outside the rounding bracket, first at %d: got %r, bracket %r..%r" % (
        what, int(bad.sum()), got.size, int(np.flatnonzero(bad)[0]), got[bad][0], lo[bad][0], hi[bad][0])
    # where the bracket is a single value the result is fixed to the bit (also the sign of zero)
    fixed = lo.view(np.uint16) == hi.view(np.uint16)
    assert np.array_equal(got_bits[fixed], want_bits[fixed]), what + ": differs from the oracle where rounding is unambiguous"
    # the bracket is a worst case; fp32 sums of these inputs land on the correctly rounded value
    # of the exact sum nearly always
    if got.size >= 1000:
        assert (got_bits == want_bits).mean() > 0.98, what + ": too few results equal the correctly rounded exact sum"


def _problem(tokens, out_f, in_f, kind, seed):
    dy = si.output_grads_fp16(tokens, out_f, seed)
    x = si.activations_fp16(tokens, in_f, seed)
    mask = _mask(kind, out_f, in_f, seed)
    idx = oracle.build_index(mask)
    d_dy = dev_f16_bits(dy).view(tokens, out_f)
    d_x = dev_f16_bits(x).view(tokens, in_f)
    return dy, x, idx, d_dy, d_x, dev_i32(idx), dev_i32(ref_seg_ptr(idx, out_f * in_f))


@pytest.fixture(params=["128", "256", "mixed"])
def tile(request):
    """Both kernels (128 x 128 tiles by two wave groups that split each stage's tokens, 256 x 256
    tiles) on every case, and the library's own rule with a round of 4 tiles, so that layers of 5,
    6 or 9 large tiles here are split between the two as a layer of 300 is on 256 compute units."""
    if request.param == "mixed":
        samo.samo_debug_set(samo.KNOB_WGRAD_ROUND, 4)
    else:
        samo.samo_debug_set(samo.KNOB_WGRAD_TILE, int(request.param))
    yield request.param
    samo.samo_debug_set(samo.KNOB_WGRAD_TILE)
    samo.samo_debug_set(samo.KNOB_WGRAD_ROUND)


@pytest.mark.parametrize("kind", ["bernoulli10", "bernoulli50", "rows", "edges", "dense_idx"])
@pytest.mark.parametrize("tokens,out_f,in_f", SHAPES)
def test_compressed_weight_gradient_matches_the_oracle(tokens, out_f, in_f, kind, tile):
    seed = 1000 + tokens + out_f + in_f
    dy, x, idx, d_dy, d_x, d_idx, d_seg = _problem(tokens, out_f, in_f, kind, seed)
    nnz = idx.shape[0]
    want = oracle.wgrad_compress(dy, x, tokens, out_f, in_f, idx)
    lo, hi = _bracket(dy, x, tokens, out_f, in_f, idx)

    gc16 = torch.full((nnz + 8,), float("nan"), dtype=torch.float16, device=DEV)
    samo.samo_wgrad_gather_fp16(d_dy, d_x, d_idx, d_seg, gc16[:nnz])
    torch.cuda.synchronize()
    _check_f16(host_bits(gc16[:nnz]), lo, hi, want, "gc16")
    assert torch.isnan(gc16[nnz:]).all(), "wrote past the compressed gradient"

    inv = np.float32(1.0 / si.LOSS_SCALE)
    gc = torch.full((nnz + 8,), float("nan"), dtype=torch.float32, device=DEV)
    samo.samo_wgrad_gather(d_dy, d_x, d_idx, d_seg, float(inv), gc[:nnz])
    torch.cuda.synchronize()
    got = gc[:nnz].cpu().numpy()
    # the fp32 output is the fp16 output widened and multiplied once in fp32
    assert np.array_equal(got.view(np.uint32), (host_bits(gc16[:nnz]).view(np.float16).astype(np.float32) * inv).view(np.uint32))
    assert torch.isnan(gc[nnz:]).all()


def test_unpruned_layer_without_an_index(tile):
    tokens, out_f, in_f = 70, 136, 264
    dy, x, _, d_dy, d_x, _, _ = _problem(tokens, out_f, in_f, "dense_idx", 5)
    n = out_f * in_f
    idx = np.arange(n, dtype=np.int32)
    gc16 = torch.full((n,), float("nan"), dtype=torch.float16, device=DEV)
    samo.samo_wgrad_gather_fp16(d_dy, d_x, None, None, gc16)
    torch.cuda.synchronize()
    lo, hi = _bracket(dy, x, tokens, out_f, in_f, idx)
    _check_f16(host_bits(gc16), lo, hi, oracle.wgrad_compress(dy, x, tokens, out_f, in_f, idx), "dense gc16")


def test_micro_batches_accumulate_in_half_precision(tile):
    """Second micro-batch added to the stored fp16 gradient: one correctly rounded half addition of
    the kernel's own fp16 weight gradient (Section II-E micro-batches, Section III-A storage)."""
    tokens, out_f, in_f = 90, 136, 520
    dy, x, idx, d_dy, d_x, d_idx, d_seg = _problem(tokens, out_f, in_f, "bernoulli10", 77)
    nnz = idx.shape[0]
    first = torch.empty(nnz, dtype=torch.float16, device=DEV)
    samo.samo_wgrad_gather_fp16(d_dy, d_x, d_idx, d_seg, first)
    dy2 = si.output_grads_fp16(tokens, out_f, 77, step=2)
    x2 = si.activations_fp16(tokens, in_f, 77, step=2)
    d_dy2, d_x2 = dev_f16_bits(dy2).view(tokens, out_f), dev_f16_bits(x2).view(tokens, in_f)
    second = torch.empty(nnz, dtype=torch.float16, device=DEV)
    samo.samo_wgrad_gather_fp16(d_dy2, d_x2, d_idx, d_seg, second)
    acc = first.clone()
    samo.samo_wgrad_gather_fp16(d_dy2, d_x2, d_idx, d_seg, acc, accumulate=True)
    torch.cuda.synchronize()
    a, b = host_bits(first), host_bits(second)
    # oracle's accumulation: dense fp16 tensor holding b at idx, added into a copy of a
    dense = np.zeros(out_f * in_f, np.uint16)
    dense[idx] = b
    want = a.copy()
    oracle.accumulate_f16(dense, idx, want)
    assert np.array_equal(host_bits(acc), want)
    lo, hi = _bracket(dy2, x2, tokens, out_f, in_f, idx)
    _check_f16(b, lo, hi, oracle.wgrad_compress(dy2, x2, tokens, out_f, in_f, idx), "second micro-batch")


def test_no_tokens_and_no_kept_elements(tile):
    out_f, in_f = 136, 264
    n = out_f * in_f
    idx = oracle.build_index(si.bernoulli_mask(n, 0.2, 3))
    d_idx, d_seg = dev_i32(idx), dev_i32(ref_seg_ptr(idx, n))
    empty_dy = torch.empty((0, out_f), dtype=torch.float16, device=DEV)
    empty_x = torch.empty((0, in_f), dtype=torch.float16, device=DEV)
    gc = torch.full((idx.shape[0],), float("nan"), dtype=torch.float32, device=DEV)
    samo.samo_wgrad_gather(empty_dy, empty_x, d_idx, d_seg, 1.0, gc)
    torch.cuda.synchronize()
    assert not gc.view(torch.int32).cpu().numpy().any()              # +0 everywhere
    # nothing kept: nothing is written, nothing is read
    none = torch.empty(0, dtype=torch.int32, device=DEV)
    seg0 = dev_i32(ref_seg_ptr(np.empty(0, np.int32), n))
    dy = dev_f16_bits(si.output_grads_fp16(9, out_f, 1)).view(9, out_f)
    x = dev_f16_bits(si.activations_fp16(9, in_f, 1)).view(9, in_f)
    samo.samo_wgrad_gather(dy, x, none, seg0, 1.0, torch.empty(0, dtype=torch.float32, device=DEV))
    torch.cuda.synchronize()


def test_overflow_rounds_to_infinity_and_specials_propagate(tile):
    tokens, out_f, in_f = 40, 8, 8
    dy = np.full((tokens, out_f), 64.0, np.float16)
    x = np.full((tokens, in_f), 64.0, np.float16)
    x[3, 5] = np.inf
    dy[0, 2] = np.nan
    idx = np.arange(out_f * in_f, dtype=np.int32)
    d_idx, d_seg = dev_i32(idx), dev_i32(ref_seg_ptr(idx, out_f * in_f))
    gc16 = torch.empty(out_f * in_f, dtype=torch.float16, device=DEV)
    samo.samo_wgrad_gather_fp16(dev_f16_bits(dy.reshape(-1).view(np.uint16)).view(tokens, out_f),
                                dev_f16_bits(x.reshape(-1).view(np.uint16)).view(tokens, in_f), d_idx, d_seg, gc16)
    torch.cuda.synchronize()
    got = host_bits(gc16).view(np.float16).reshape(out_f, in_f)
    want = oracle.wgrad_compress(dy.reshape(-1).view(np.uint16), x.reshape(-1).view(np.uint16), tokens, out_f, in_f,
                                 idx).view(np.float16).reshape(out_f, in_f)
    assert np.array_equal(np.isnan(got), np.isnan(want))             # row 2 of dW
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])                         # 40 * 4096 > 65504: +inf; column 5: +inf


def test_several_layers_in_one_call_share_the_tile_list(tile):
    """Five layers of different shapes, token counts and masks in one batched call, one of them with
    nothing kept and one without an index: each layer's result against the oracle; with the round of
    4 tiles the 14 large tiles of the list are three rounds of large ones and two as small quarters,
    and layer boundaries fall inside rounds."""
    layers = [(64, 384, 264, "bernoulli10"), (33, 136, 264, "rows"), (70, 24, 40, "none"), (130, 520, 264, "bernoulli50"),
              (45, 264, 8, "dense")]
    jobs16, jobs32, checks = [], [], []
    inv = np.float32(1.0 / si.LOSS_SCALE)
    for j, (tokens, out_f, in_f, kind) in enumerate(layers):
        n = out_f * in_f
        dy = si.output_grads_fp16(tokens, out_f, 40 + j)
        x = si.activations_fp16(tokens, in_f, 40 + j)
        d_dy = dev_f16_bits(dy).view(tokens, out_f)
        d_x = dev_f16_bits(x).view(tokens, in_f)
        if kind == "none":
            idx = np.zeros(0, dtype=np.int32)
        elif kind == "dense":
            idx = np.arange(n, dtype=np.int32)
        else:
            idx = oracle.build_index(_mask(kind, out_f, in_f, 40 + j))
        nnz = idx.shape[0]
        d_idx = None if kind == "dense" else dev_i32(idx)
        d_seg = None if kind == "dense" else dev_i32(ref_seg_ptr(idx, n))
        gc16 = torch.full((nnz + 8,), float("nan"), dtype=torch.float16, device=DEV)
        gc = torch.full((nnz + 8,), float("nan"), dtype=torch.float32, device=DEV)
        jobs16.append((d_dy, d_x, d_idx, d_seg, gc16[:nnz]))
        jobs32.append((d_dy, d_x, d_idx, d_seg, gc[:nnz]))
        checks.append((dy, x, tokens, out_f, in_f, idx, gc16, gc))
    samo.samo_wgrad_gather_fp16_batched(jobs16)
    samo.samo_wgrad_gather_batched(jobs32, float(inv))
    torch.cuda.synchronize()
    for dy, x, tokens, out_f, in_f, idx, gc16, gc in checks:
        nnz = idx.shape[0]
        assert torch.isnan(gc16[nnz:]).all() and torch.isnan(gc[nnz:]).all(), "wrote past a layer's compressed gradient"
        if nnz == 0:
            continue
        lo, hi = _bracket(dy, x, tokens, out_f, in_f, idx)
        got = host_bits(gc16[:nnz])
        _check_f16(got, lo, hi, oracle.wgrad_compress(dy, x, tokens, out_f, in_f, idx), "batched gc16 %dx%d" % (out_f, in_f))
        assert np.array_equal(gc[:nnz].cpu().numpy().view(np.uint32), (got.view(np.float16).astype(np.float32) * inv).view(np.uint32))
    # second micro-batch: accumulate into the same buffers, all layers at once
    before = [host_bits(c[6][:c[5].shape[0]]).view(np.float16).copy() for c in checks]
    samo.samo_wgrad_gather_fp16_batched(jobs16, accumulate=True)
    torch.cuda.synchronize()
    for c, h in zip(checks, before):
        nnz = c[5].shape[0]
        if nnz:
            assert np.array_equal(host_bits(c[6][:nnz]), (h + h).astype(np.float16).view(np.uint16)), "accumulate: twice the first result"
    samo.samo_wgrad_gather_batched([], 1.0)                  # no jobs: nothing to do
    with pytest.raises(RuntimeError):
        samo.samo_wgrad_gather_batched(jobs32 + jobs32, 1.0)  # ten jobs


def test_rejections():
    dy = torch.zeros((4, 8), dtype=torch.float16, device=DEV)
    x = torch.zeros((4, 12), dtype=torch.float16, device=DEV)
    gc = torch.zeros(96, dtype=torch.float32, device=DEV)
    with pytest.raises(samo.SamoError):
        samo.samo_wgrad_gather(dy, x, None, None, 1.0, gc)           # in = 12 is not a multiple of 8
    x = torch.zeros((5, 16), dtype=torch.float16, device=DEV)
    with pytest.raises(ValueError):
        samo.samo_wgrad_gather(dy, x, None, None, 1.0, gc)           # token counts differ
    x = torch.zeros((4, 16), dtype=torch.float16, device=DEV)
    with pytest.raises(samo.SamoError):
        samo.samo_wgrad_gather(dy, x, None, None, 1.0, gc[:100 - 10])   # no index, yet fewer than out * in outputs
    idx = torch.zeros(90, dtype=torch.int32, device=DEV)
    with pytest.raises(samo.SamoError):
        samo.samo_wgrad_gather(dy, x, idx, None, 1.0, gc[:90])       # an index without seg_ptr
    with pytest.raises(samo.SamoError):
        samo.samo_wgrad_gather(dy, x, None, None, 0.0, torch.zeros(128, dtype=torch.float32, device=DEV))


def test_fused_backward_compression_feeds_statistics_and_the_optimizer():
    """Two micro-batches of a three-layer model, the gradient of every layer compressed inside its
    backward kernel into the stored fp16 gradient (the second micro-batch accumulated), then the
    batched statistics, clipping and Adam + expansion — against the oracle's unfused route through
    a dense fp16 gradient.  Small-integer operands make every weight gradient exact in fp16, so
    the comparison does not depend on the order of the kernel's sums."""
    from gpu_util import INV, OCFG, DevLayer, HostLayer, assert_close
    shapes = [(136, 264, 0.2, False), (264, 72, 0.5, False), (24, 40, 1.0, True)]      # (out, in, keep, unpruned)
    tokens = 70
    hosts, devs, ops = [], [], []
    rng = np.random.default_rng(31)
    for k, (out_f, in_f, keep, dense) in enumerate(shapes):
        n = out_f * in_f
        mask = np.ones(n, np.uint8) if dense else si.bernoulli_mask(n, keep, 40 + k)
        hosts.append(HostLayer(n, mask, si.weights(n, 40 + k), 40 + k, dense=dense))
        devs.append(DevLayer(hosts[-1], with_gc16=True))
        ops.append([(rng.integers(-2, 3, (tokens, out_f)).astype(np.float16), rng.integers(-3, 4, (tokens, in_f)).astype(np.float16))
                    for _ in range(2)])
    plan = samo.Plan([d.layer() for d in devs])
    stats = samo.GradStats(plan)
    # backward passes: micro-batch 0 overwrites, micro-batch 1 accumulates
    ref_gc16 = []
    for (out_f, in_f, _, _), h, d, mb in zip(shapes, hosts, devs, ops):
        acc = None
        for j, (dy, x) in enumerate(mb):
            dyb, xb = dy.reshape(-1).view(np.uint16), x.reshape(-1).view(np.uint16)
            samo.samo_wgrad_gather_fp16(dev_f16_bits(dyb).view(tokens, out_f), dev_f16_bits(xb).view(tokens, in_f),
                                        d.idx, d.seg_ptr, d.gc16, accumulate=j > 0)
            dense16 = oracle.linear_weight_grad(dyb, xb, tokens, out_f, in_f).astype(np.float16).view(np.uint16)
            if acc is None:
                acc = oracle.compress_f16(dense16, h.idx)
            else:
                oracle.accumulate_f16(dense16, h.idx, acc)
        ref_gc16.append(acc)
        assert np.array_equal(host_bits(d.gc16), acc)                   # exact sums: bit-exact
    # statistics over the stored fp16 gradient, then clipped Adam + expansion
    plan.samo_grad_stats_batched(1, INV, stats)
    total = sum(oracle.sum_squares(oracle.upcast(g, INV)) for g in ref_gc16)
    ss, bad = stats.read()
    assert not bad and abs(ss - total) <= 1e-12 * total
    max_norm = 0.25 * total ** 0.5
    plan.samo_adam_expand_batched(INV, samo.adam_cfg(1, **si.ADAM), stats.guard(max_grad_norm=max_norm))
    torch.cuda.synchronize()
    coef = oracle.clip_coefficient(total, max_norm)
    for h, d, g in zip(hosts, devs, ref_gc16):
        gc = oracle.upcast(g, INV)
        oracle.scale(gc, coef)
        oracle.adam(h.p, h.m, h.v, gc, OCFG, 1)
        assert_close(d.p.cpu().numpy(), h.p, "p")
        assert_close(d.m.cpu().numpy(), h.m, "m")
        assert_close(d.v.cpu().numpy(), h.v, "v")
        assert np.array_equal(host_bits(d.w), oracle.decompress(d.p.cpu().numpy(), h.idx, h.n))
    plan.close()


def test_fused_weight_gradient_under_hip_graph_replay():
    """The backward kernel, the statistics and the guarded optimizer phase captured once and
    replayed with eager work in between; every replay equals the eager result bit for bit."""
    from gpu_util import INV, DevLayer, HostLayer
    out_f, in_f, tokens = 264, 520, 100
    n = out_f * in_f
    h = HostLayer(n, si.bernoulli_mask(n, 0.15, 71), si.weights(n, 71), 71)
    a, b = DevLayer(h, with_gc16=True), DevLayer(h, with_gc16=True)
    plan_a, plan_b = samo.Plan([a.layer()]), samo.Plan([b.layer()])
    stats_a, stats_b = samo.GradStats(plan_a), samo.GradStats(plan_b)
    dy = torch.empty((tokens, out_f), dtype=torch.float16, device=DEV)
    x = torch.empty((tokens, in_f), dtype=torch.float16, device=DEV)
    cfg = samo.adam_cfg(1, **si.ADAM)

    def work(d, plan, stats):
        samo.samo_wgrad_gather_fp16(dy, x, d.idx, d.seg_ptr, d.gc16)
        plan.samo_grad_stats_batched(1, INV, stats)
        plan.samo_adam_expand_batched(INV, cfg, stats.guard(max_grad_norm=0.5, skip_on_nonfinite=True))

    def feed(step):
        dy.copy_(dev_f16_bits(si.output_grads_fp16(tokens, out_f, 71, step)).view(tokens, out_f))
        x.copy_(dev_f16_bits(si.activations_fp16(tokens, in_f, 71, step)).view(tokens, in_f))

    feed(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work(a, plan_a, stats_a)                                       # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work(a, plan_a, stats_a)
    work(b, plan_b, stats_b)                                           # both sides have taken step 1 once...
    graph.replay()
    work(b, plan_b, stats_b)                                           # ...and twice
    for step in (2, 3, 4):
        feed(step)
        a.w.fill_(float("nan"))
        b.w.fill_(float("nan"))
        torch.cuda.synchronize()
        work(b, plan_b, stats_b)
        graph.replay()
        torch.cuda.synchronize()
        assert stats_a.read() == stats_b.read(), step
        assert torch.equal(a.gc16.view(torch.int16), b.gc16.view(torch.int16)), step
        assert torch.equal(a.p, b.p) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v), step
        assert torch.equal(a.w.view(torch.int16), b.w.view(torch.int16)), step
    # the eager side once more against the oracle: its last compressed gradient
    lo, hi = _bracket(si.output_grads_fp16(tokens, out_f, 71, 4), si.activations_fp16(tokens, in_f, 71, 4), tokens, out_f, in_f, h.idx)
    got = host_bits(b.gc16).view(np.float16)
    assert np.all((got >= lo) & (got <= hi))
    plan_a.close()
    plan_b.close()
