"""GPU parity at the benchmark's full sizes and launch configuration: every weight matrix of
a model processed by ONE batched launch, compared with the CPU oracle element by element
(the C oracle finishes a 2.7B-shape step in a few seconds, so nothing is sampled)."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import DEV, INV, OCFG, assert_close, host_bits

pytestmark = pytest.mark.gpu


def note(text):
    """A progress line that reaches the terminal through pytest's capture (long tests stay visibly alive)."""
    sys.__stdout__.write("  [%s]\n" % text)
    sys.__stdout__.flush()


class Model:
    """All layers of a configuration on the GPU (index built by the library) and on the host
    (index built by the oracle).

    steps_ahead = k: the oracle's k optimizer steps (the same gradient every step, as in
    oracle_step) are taken while the layers stream through the generator, and only the oracle's
    index and final p, m, v stay on the host — 16 bytes per kept element instead of 3 more per
    dense one — so that the largest configurations are checked whole with bounded host memory."""

    def __init__(self, specs, with_gc=False, workers=12, with_gc16=False, steps_ahead=0):
        self.specs = specs
        self.host = []      # [spec, mask, idx, p, m, v, g16]
        masks = []
        on_dev = []          # (p, g) of every layer, on the GPU, until the arena exists

        def consume(i, data):
            spec = data.spec
            ref_idx = oracle.build_index(data.mask)
            p_host = np.ascontiguousarray(data.w32[ref_idx])
            masks.append(None if spec.mask_kind == "dense" else torch.from_numpy(data.mask).to(DEV))
            h = [spec, data.mask, ref_idx, p_host, np.zeros_like(p_host), np.zeros_like(p_host), data.g16]
            if steps_ahead:
                on_dev.append((torch.from_numpy(p_host).to(DEV),
                               torch.from_numpy(data.g16.view(np.int16)).to(DEV).view(torch.float16)))
                h[3] = p_host.copy()
                for t in range(1, steps_ahead + 1):
                    oracle.step(data.g16, spec.n, ref_idx, h[3], h[4], h[5], INV, OCFG, t)
                h[1] = h[6] = None
                if i % 16 == 15:
                    note("%d of %d matrices generated, oracle %d steps ahead" % (i + 1, len(specs), steps_ahead))
            self.host.append(h)

        si.generate(specs, consume, workers=workers)
        # same set-up as bench.py: batched index build, one layer-major allocation, one plan
        built = iter(samo.samo_build_index_many([m for m in masks if m is not None]))
        self.layers = samo.alloc_model([(h[0].n, h[2].shape[0], m is None) for h, m in zip(self.host, masks)], DEV,
                                       with_gc=with_gc, with_gc16=with_gc16)
        for L, h, m in zip(self.layers, self.host, masks):
            if m is not None:
                ix = next(built)
                assert ix.nnz == h[2].shape[0], h[0].name
                assert np.array_equal(ix.idx.cpu().numpy(), h[2]), h[0].name          # bit-exact index
                L.idx.copy_(ix.idx)
                L.seg_ptr.copy_(ix.seg_ptr)
            if steps_ahead:
                d_p, d_g = on_dev.pop(0)
                L.p.copy_(d_p)
                L.g.copy_(d_g)
                del d_p, d_g
            else:
                L.p.copy_(torch.from_numpy(h[3]))
                L.g.copy_(torch.from_numpy(h[6].view(np.int16)).view(torch.float16))
            L.w.fill_(float("nan"))
            if with_gc:
                L.gc.fill_(float("nan"))
        del masks
        self.plan = samo.Plan(self.layers)

    def oracle_step(self, t):
        for spec, mask, idx, p, m, v, g16 in self.host:
            oracle.step(g16, spec.n, idx, p, m, v, INV, OCFG, t)

    def check(self, t):
        for L, (spec, mask, idx, p, m, v, g16) in zip(self.layers, self.host):
            got_p = L.p.cpu().numpy()
            assert_close(got_p, p, "%s p t=%d" % (spec.name, t))
            assert_close(L.m.cpu().numpy(), m, "%s m t=%d" % (spec.name, t))
            assert_close(L.v.cpu().numpy(), v, "%s v t=%d" % (spec.name, t))
            w_bits = host_bits(L.w)
            assert np.array_equal(w_bits, oracle.decompress(got_p, idx, spec.n)), "%s w t=%d" % (spec.name, t)

    def poison_w(self):
        for L in self.layers:
            L.w.fill_(float("nan"))


def test_gpt2p7b_90pct_every_batched_entry_at_full_size():
    """The configuration bench.py times: 128 matrices, N = 2,516,582,400, one launch per step."""
    model = Model(si.config("gpt2.7b", 0.9), with_gc=True, with_gc16=True)
    n_total, nnz_total = model.plan.totals()
    assert n_total == 2_516_582_400 and nnz_total == 251_658_240
    for t in (1, 2):
        model.poison_w()
        model.plan.samo_fused_step_batched(INV, samo.adam_cfg(t, **si.ADAM))
        model.oracle_step(t)
        model.check(t)
    # step 3 as the separate passes of the paper, step 4 as the split around an all-reduce with the
    # gradient statistics reduced on the way (the other entries bench.py times, same launch shapes)
    model.poison_w()
    model.plan.samo_gather_batched(INV)
    model.plan.samo_adam_batched(samo.adam_cfg(3, **si.ADAM))
    model.plan.samo_decompress_batched()
    model.oracle_step(3)
    model.check(3)
    model.poison_w()
    stats = samo.GradStats(model.plan)
    model.plan.samo_gather_fp16_batched(False, INV, stats)
    model.plan.samo_adam_expand_batched(INV, samo.adam_cfg(4, **si.ADAM), stats.guard(0.0, True))
    ref_ss = sum(oracle.sum_squares(oracle.gather(h[6], h[2], INV)) for h in model.host)
    ss, bad = stats.read()
    assert not bad and abs(ss - ref_ss) <= 2 * nnz_total * 2.0 ** -53 * ref_ss
    # the statistics a data-parallel run takes from the reduced compressed gradient (a kernel of its
    # own, several chunk records per wave) and those of the unscaled fp32 one: same partials, same bits
    again = samo.GradStats(model.plan)
    model.plan.samo_grad_stats_batched(1, INV, again)
    assert again.read() == (ss, bad)
    model.plan.samo_grad_stats_batched(2, 1.0, again)          # gc as step 3's gather left it: the same gradient
    assert again.read() == (ss, bad)
    for L, h in zip(model.layers[:8], model.host[:8]):
        assert np.array_equal(host_bits(L.gc16), oracle.compress_f16(h[6], h[2])), h[0].name
    model.oracle_step(4)
    model.check(4)


def test_gpt350m_unfused_then_fused():
    model = Model(si.config("gpt350m", 0.9), with_gc=True)
    assert model.plan.totals() == (301_989_888, 30_198_984)
    model.plan.samo_decompress_batched()
    for L, h in zip(model.layers, model.host):
        assert np.array_equal(host_bits(L.w), oracle.decompress(h[3], h[2], h[0].n)), h[0].name
    model.poison_w()
    model.plan.samo_gather_batched(INV)
    for L, h in zip(model.layers, model.host):
        assert np.array_equal(L.gc.cpu().numpy().view(np.uint32), oracle.gather(h[6], h[2], INV).view(np.uint32))
    model.plan.samo_adam_batched(samo.adam_cfg(1, **si.ADAM))
    model.plan.samo_decompress_batched()
    model.oracle_step(1)
    model.check(1)
    model.poison_w()
    model.plan.samo_fused_step_batched(INV, samo.adam_cfg(2, **si.ADAM))
    model.oracle_step(2)
    model.check(2)


def test_gpt2p7b_single_precision_slice():
    """Eight layers (32 matrices, 629 M elements) of the 2.7B shape at 90 % through the batched
    single-precision step, two steps, every element against the oracle."""
    specs = si.config("gpt2.7b", 0.9, layers=8)
    host, masks = [], []

    def consume(i, data):
        idx = oracle.build_index(data.mask)
        w = np.where(data.mask != 0, data.w32, np.float32(0)).astype(np.float32)
        host.append([data.spec, data.mask, idx, w, np.zeros(idx.shape[0], np.float32), np.zeros(idx.shape[0], np.float32)])
        masks.append(torch.from_numpy(data.mask).to(DEV))

    si.generate(specs, consume, workers=12)
    built = samo.samo_build_index_many(masks)
    del masks
    layers = samo.alloc_model_fp32([(ix.n, ix.nnz, False) for ix in built], DEV)
    for L, ix, h in zip(layers, built, host):
        assert np.array_equal(ix.idx.cpu().numpy(), h[2]), h[0].name
        L.idx.copy_(ix.idx)
        L.seg_ptr.copy_(ix.seg_ptr)
        dirty = h[3].copy()
        dirty[h[1] == 0] = 5.0                                    # garbage at pruned positions goes away
        L.w32.copy_(torch.from_numpy(dirty))
    del built
    plan = samo.Plan(layers)
    for t in (1, 2):
        for L, h in zip(layers, host):
            L.g32.copy_(torch.from_numpy(si.grads_fp32(h[0].n, h[0].seed, t)))
        plan.samo_fused_step_fp32_batched(1.0, samo.adam_cfg(t, **si.ADAM))
        for L, h in zip(layers, host):
            spec, mask, idx, w, m, v = h
            oracle.step_fp32(si.grads_fp32(spec.n, spec.seed, t), w, idx, m, v, 1.0, OCFG, t)
            got = L.w32.cpu().numpy()
            assert_close(got[idx], w[idx], "%s w32 t=%d" % (spec.name, t))
            assert not got.view(np.uint32)[mask == 0].any(), spec.name
            assert_close(L.m.cpu().numpy(), m, "%s m t=%d" % (spec.name, t))
            assert_close(L.v.cpu().numpy(), v, "%s v t=%d" % (spec.name, t))
    plan.close()


def _whole_model_two_fused_steps(specs, workers=12):
    """Two fused steps of ONE batched launch each over every matrix of `specs`, then every element
    of p, m, v and w against the oracle (which took its two steps while the layers were generated)."""
    model = Model(specs, workers=workers, steps_ahead=2)
    note("%d matrices resident, N = %d, nnz = %d" % ((len(specs),) + model.plan.totals()))
    for t in (1, 2):
        model.poison_w()
        model.plan.samo_fused_step_batched(INV, samo.adam_cfg(t, **si.ADAM))
    torch.cuda.synchronize()
    note("two batched steps done, comparing")
    model.check(2)
    return model


def test_gpt1p3b_fused_full_size():
    """BASELINE configuration 3: 24 layers x 4 matrices, hidden 2048, 90 % magnitude-pruned."""
    model = _whole_model_two_fused_steps(si.config("gpt1.3b", 0.9))
    assert model.plan.totals() == (1_207_959_552, 120_795_960)


@pytest.mark.parametrize("sparsity", [0.8, 0.95])
def test_gpt2p7b_sparsity_sweep_full_size(sparsity):
    """All 32 layers (128 matrices) of the 2.7B shape at the other sparsities of the sweep."""
    model = _whole_model_two_fused_steps(si.config("gpt2.7b", sparsity))
    n_total, nnz_total = model.plan.totals()
    assert n_total == 2_516_582_400
    assert nnz_total == sum(si.kept_count(s.n, sparsity) for s in model.specs) == round((1 - sparsity) * n_total)


def test_gpt6p7b_row_clustered_full_size_with_dense_embedding():
    """BASELINE configuration 5 whole: 32 layers x 4 matrices with 128 different per-matrix sparsities
    in [0.8, 0.97], row-clustered masks, plus the dense 50304x4096 embedding.
    SAMO_TEST_6P7B_LAYERS caps the number of transformer layers (default: all 32)."""
    nl = min(32, int(os.environ.get("SAMO_TEST_6P7B_LAYERS", "32")))
    specs = si.config("gpt6.7b", layers=nl)
    assert specs[-1].mask_kind == "dense" and specs[-1].n == 50304 * 4096
    if nl == 32:
        ps = [s.sparsity for s in specs[:-1]]
        assert len(set(ps)) == 128 and 0.8 <= min(ps) < 0.81 and 0.96 < max(ps) <= 0.97
    model = _whole_model_two_fused_steps(specs, workers=8)
    # hot rows are ~10x denser than cold rows: tiles differ widely in their compressed slice
    spec, idx = model.host[0][0], model.host[0][2]
    per_row = np.bincount(idx // spec.cols, minlength=spec.rows)
    assert per_row.max() > 5 * np.median(per_row)


def test_largest_layer_int32_index_limit():
    """One layer of N = 2^31 - 1 elements, the largest flat size a 32-bit index allows (Section III-B):
    index, expansion and one fused step, bit-exact / within tolerance on every element."""
    n = 2**31 - 1
    chunk = 1 << 26
    mask = np.empty(n, np.uint8)
    g16 = np.empty(n, np.uint16)
    for c, lo in enumerate(range(0, n, chunk)):
        hi = min(n, lo + chunk)
        mask[lo:hi] = si.bernoulli_mask(hi - lo, 0.04, 7000 + c)
        g16[lo:hi] = si.grads_fp16(hi - lo, 7000 + c)
    mask[0] = mask[-1] = 1                                        # first and last position kept
    ref_idx = oracle.build_index(mask)
    assert ref_idx[0] == 0 and ref_idx[-1] == n - 1
    nnz = ref_idx.shape[0]

    d_mask = torch.from_numpy(mask).to(DEV)
    ix = samo.samo_build_index(d_mask)
    del d_mask
    assert ix.nnz == nnz
    assert np.array_equal(ix.idx.cpu().numpy(), ref_idx)
    assert samo.samo_validate_index(ix.idx, n, ix.seg_ptr)

    p_host = si.weights(nnz, 7100)
    p = torch.from_numpy(p_host).to(DEV)
    m, v = torch.zeros_like(p), torch.zeros_like(p)
    w = torch.full((n,), float("nan"), dtype=torch.float16, device=DEV)
    samo.samo_decompress(p, ix.idx, ix.seg_ptr, w)
    ref_w = oracle.decompress(p_host, ref_idx, n)
    assert np.array_equal(host_bits(w), ref_w)

    g = torch.from_numpy(g16.view(np.int16)).to(DEV).view(torch.float16)
    w.fill_(float("nan"))
    samo.samo_fused_step(g, w, ix.idx, ix.seg_ptr, p, m, v, INV, samo.adam_cfg(1, **si.ADAM))
    ref_m, ref_v = np.zeros_like(p_host), np.zeros_like(p_host)
    oracle.step(g16, n, ref_idx, p_host, ref_m, ref_v, INV, OCFG, 1, ref_w)
    got_p = p.cpu().numpy()
    assert_close(got_p, p_host, "p")
    assert_close(m.cpu().numpy(), ref_m, "m")
    assert_close(v.cpu().numpy(), ref_v, "v")
    assert np.array_equal(host_bits(w), oracle.decompress(got_p, ref_idx, n, ref_w))


def test_fused_step_under_hip_graph_replay():
    """The batched entry only enqueues kernels on the caller's stream, so it can be captured into a
    HIP graph; every replay must give what the eager launch gives."""
    specs = si.config("gpt350m", 0.9, layers=2)
    eager, graphed = Model(specs), Model(specs)
    cfg = samo.adam_cfg(1, **si.ADAM)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graphed.plan.samo_fused_step_batched(INV, cfg)          # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graphed.plan.samo_fused_step_batched(INV, cfg)
    eager.plan.samo_fused_step_batched(INV, cfg)                # eager has done 1 step, graphed 1 step
    for rep in range(3):
        eager.poison_w()
        graphed.poison_w()
        torch.cuda.synchronize()
        eager.plan.samo_fused_step_batched(INV, cfg)
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager.layers, graphed.layers):
            assert torch.equal(a.p, b.p) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v), rep
            assert torch.equal(a.w.view(torch.int16), b.w.view(torch.int16)), rep
    # and the eager side still matches the oracle after its 4 steps with a fixed step counter
    for _ in range(4):
        eager.oracle_step(1)
    eager.check(1)


def test_index_build_statistics_and_guarded_split_step_under_hip_graph_replay():
    """Index construction (init + chained kernel), the compressed fp16 gather with gradient
    statistics (gather, two-level reduction) and the clipped Adam+expand step are kernels only —
    no memset, no allocation — so they replay from a HIP graph; every replay is checked against
    the eager result, with eager work and synchronisations between replays."""
    specs = si.config("gpt350m", 0.9, layers=1)
    n_masks = len(specs)
    host = [si.make_layer(s) for s in specs]
    masks = [torch.from_numpy(h.mask).to(DEV) for h in host]
    first = samo.samo_build_index_many(masks)                       # sizes the buffers (eager)
    layers = samo.alloc_model([(ix.n, ix.nnz, False) for ix in first], DEV, with_gc16=True)
    ref = samo.alloc_model([(ix.n, ix.nnz, False) for ix in first], DEV, with_gc16=True)
    for group in (layers, ref):
        for L, ix, h in zip(group, first, host):
            L.idx.copy_(ix.idx)
            L.seg_ptr.copy_(ix.seg_ptr)
            L.p.copy_(torch.from_numpy(np.ascontiguousarray(h.w32[h.mask != 0])))
            L.g.copy_(torch.from_numpy(h.g16.view(np.int16)).view(torch.float16))
    plan, ref_plan = samo.Plan(layers), samo.Plan(ref)
    stats, ref_stats = samo.GradStats(plan), samo.GradStats(ref_plan)
    cfg = samo.adam_cfg(1, **si.ADAM)
    nnz_out = torch.zeros(n_masks, dtype=torch.int64, device=DEV)
    max_norm = 0.5                                                 # well below the gradient's norm: clipping acts

    def work(pl, st, group):
        samo.samo_build_index_batched(masks, [L.idx for L in group], [L.seg_ptr for L in group], nnz_out)
        pl.samo_gather_fp16_batched(False, INV, st)
        pl.samo_adam_expand_batched(INV, cfg, st.guard(max_norm, True))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work(plan, stats, layers)                                   # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work(plan, stats, layers)
    work(ref_plan, ref_stats, ref)                                  # both sides have done one step
    for rep in range(3):
        for group in (layers, ref):
            for L in group:
                L.w.fill_(float("nan"))
                L.idx.fill_(-1)                                     # the replay has to rebuild these
                L.seg_ptr.fill_(-7)
        nnz_out.fill_(-3)
        torch.cuda.synchronize()
        work(ref_plan, ref_stats, ref)
        expect_nnz = nnz_out.clone()
        nnz_out.fill_(-3)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(nnz_out, expect_nnz) and nnz_out.tolist() == [ix.nnz for ix in first], rep
        assert stats.read() == ref_stats.read(), rep
        for a, b, ix in zip(layers, ref, first):
            assert torch.equal(a.idx, ix.idx) and torch.equal(a.seg_ptr, ix.seg_ptr), rep
            assert torch.equal(a.idx, b.idx) and torch.equal(a.seg_ptr, b.seg_ptr), rep
            assert torch.equal(a.gc16.view(torch.int16), b.gc16.view(torch.int16)), rep
            assert torch.equal(a.p, b.p) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v), rep
            assert torch.equal(a.w.view(torch.int16), b.w.view(torch.int16)), rep
    ss, bad = stats.read()
    assert not bad and ss ** 0.5 > max_norm
    # the eager side against the oracle: four identical clipped steps with t = 1
    total = sum(oracle.sum_squares(oracle.gather(h.g16, np.flatnonzero(h.mask).astype(np.int32), INV)) for h in host)
    coef = oracle.clip_coefficient(total, max_norm)
    for L, h in zip(ref, host):
        idx = oracle.build_index(h.mask)
        p = np.ascontiguousarray(h.w32[idx])
        m, v = np.zeros_like(p), np.zeros_like(p)
        for _ in range(4):
            gc = oracle.gather(h.g16, idx, INV)
            oracle.scale(gc, coef)
            oracle.adam(p, m, v, gc, OCFG, 1)
        assert_close(L.p.cpu().numpy(), p, "p")
        assert_close(L.m.cpu().numpy(), m, "m")
        assert_close(L.v.cpu().numpy(), v, "v")


def _check_rows_against_oracle(got, idx, dy, x, tokens, out_f, in_f, at_least, seed, name=""):
    """Every kept output in a set of whole rows of dW against the oracle's rounding bracket:
    the exact sum s and the magnitude sum S in fp64; any fp32 summation order lands within
    (tokens + 2) * 2^-23 * S of s, and rounding to fp16 is monotonic."""
    rng = np.random.default_rng(seed)
    edges = [r for b in range(0, out_f + 1, 128) for r in (b - 1, b) if 0 <= r < out_f]
    bounds = np.searchsorted(idx, np.arange(out_f + 1, dtype=np.int64) * in_f, side="left")
    per_row = np.diff(bounds)                                            # kept outputs in every row of dW
    chosen = np.zeros(out_f, bool)
    chosen[[0, out_f - 1] + edges] = True
    for r in rng.permutation(out_f):                                     # random rows until enough outputs are covered
        if per_row[chosen].sum() >= at_least:
            break
        chosen[r] = True
    rows = np.flatnonzero(chosen).astype(np.int64)
    checked, exact_hits = 0, 0
    for r0 in range(0, rows.shape[0], 64):                              # 64 rows per fp64 product
        block = rows[r0:r0 + 64]
        val, mag = oracle.wgrad_rows(dy, x, tokens, out_f, in_f, block)
        lo_k = np.searchsorted(idx, block * in_f, side="left")
        hi_k = np.searchsorted(idx, (block + 1) * in_f, side="left")
        for r in range(block.shape[0]):
            ks = np.arange(lo_k[r], hi_k[r])
            cols = idx[ks] - block[r] * in_f
            s_, S_ = val[r, cols], mag[r, cols]
            slack = (tokens + 2) * 2.0 ** -23 * S_
            g = got[ks]
            lo, hi = (s_ - slack).astype(np.float16), (s_ + slack).astype(np.float16)
            assert np.all((g >= lo) & (g <= hi)), "%s row %d: outputs outside the rounding bracket of the exact sums" % (name, block[r])
            exact_hits += int((g == s_.astype(np.float16)).sum())
            checked += ks.shape[0]
    assert checked >= at_least, (checked, at_least)
    assert exact_hits > 0.98 * checked


@pytest.mark.parametrize("layer,tokens", [("fc1", 2048), ("fc1", 4096 + 24), ("qkv", 2048)])
def test_gpt2p7b_weight_gradient_compressed_in_the_backward_kernel(layer, tokens):
    """Full-size layers of the 2.7B model, magnitude-pruned to 10 %: FC1 (dW 2560 x 10240, 400 tiles
    of 256 x 256: all of them large) in the launch configuration bench.py times — one 2048-token
    sequence — and on a longer run with a ragged end; QKV (300 tiles: one round of 256 large ones,
    the other 44 as 128 x 128 quarters).  Against the oracle on sampled outputs, and against the
    unfused route of this library (a library GEMM into the dense fp16 tensor, then
    samo_gather_grads) on every output."""
    spec = [s for s in si.config("gpt2.7b", 0.9, layers=1) if s.name.endswith(layer)][0]
    out_f, in_f = spec.rows, spec.cols
    data = si.make_layer(spec)
    idx = oracle.build_index(data.mask)
    nnz = idx.shape[0]
    dy = si.output_grads_fp16(tokens, out_f, spec.seed)
    x = si.activations_fp16(tokens, in_f, spec.seed)
    d_dy = torch.from_numpy(dy.view(np.int16)).to(DEV).view(torch.float16).view(tokens, out_f)
    d_x = torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.float16).view(tokens, in_f)
    ix = samo.samo_build_index(torch.from_numpy(data.mask).to(DEV))
    assert ix.nnz == nnz
    gc16 = torch.full((nnz,), float("nan"), dtype=torch.float16, device=DEV)
    samo.samo_wgrad_gather_fp16(d_dy, d_x, ix.idx, ix.seg_ptr, gc16)
    gc = torch.full((nnz,), float("nan"), dtype=torch.float32, device=DEV)
    samo.samo_wgrad_gather(d_dy, d_x, ix.idx, ix.seg_ptr, INV, gc)
    torch.cuda.synchronize()
    got = host_bits(gc16)
    # the oracle on whole rows of dW: the first and last row, rows on both sides of every 128-row
    # and 256-row tile boundary, and random ones, until at least 200 000 kept outputs are covered
    _check_rows_against_oracle(got.view(np.float16), idx, dy, x, tokens, out_f, in_f, at_least=200_000, seed=12)
    # fp32 output = the fp16 one widened, times 1/loss scale
    assert np.array_equal(gc.cpu().numpy().view(np.uint32),
                          (got.view(np.float16).astype(np.float32) * np.float32(INV)).view(np.uint32))
    # every output against the unfused route: same products, fp32 sums in another order.  Each
    # route's fp32 sum is within (tokens + 2) * 2^-23 * sum|dY X| of the exact one, and that sum is
    # at most the product of the two columns' norms; then each rounds once to fp16.
    dense = torch.empty((out_f, in_f), dtype=torch.float16, device=DEV)
    torch.matmul(d_dy.t(), d_x, out=dense)
    ref = torch.empty(nnz, dtype=torch.float32, device=DEV)
    samo.samo_gather_grads(dense.view(-1), ix.idx, 1.0, ref)
    torch.cuda.synchronize()
    a, b = got.view(np.float16).astype(np.float32), ref.cpu().numpy()
    assert (a == b).mean() > 0.995
    norm_dy = np.sqrt((dy.reshape(tokens, out_f).astype(np.float64) ** 2).sum(axis=0))
    norm_x = np.sqrt((x.reshape(tokens, in_f).astype(np.float64) ** 2).sum(axis=0))
    slack = (tokens + 2) * 2.0 ** -23 * norm_dy[idx // in_f] * norm_x[idx % in_f]
    ulp = np.maximum(np.abs(b), 2.0 ** -14) * 2.0 ** -10
    assert np.all(np.abs(a.astype(np.float64) - b) <= ulp + 2 * slack), "further from the library GEMM's result than two roundings allow"


def test_gpt2p7b_layer_weight_gradients_in_one_batched_call():
    """The four pruned matrices of one transformer layer of the 2.7B model (QKV, projection, FC1, FC2:
    1200 tiles of 256 x 256 as one list) in one samo_wgrad_gather_fp16_batched call at 2048 tokens,
    the configuration bench.py times: sampled outputs of every matrix against the oracle, and every
    output against the one-call-per-matrix result (the same products; a tile may be summed by the
    other kernel, so in another order)."""
    tokens = 2048
    specs = si.config("gpt2.7b", 0.9, layers=1)
    jobs, single, keep = [], [], []
    for spec in specs:
        out_f, in_f = spec.rows, spec.cols
        data = si.make_layer(spec)
        idx = oracle.build_index(data.mask)
        dy = si.output_grads_fp16(tokens, out_f, spec.seed)
        x = si.activations_fp16(tokens, in_f, spec.seed)
        d_dy = torch.from_numpy(dy.view(np.int16)).to(DEV).view(torch.float16).view(tokens, out_f)
        d_x = torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.float16).view(tokens, in_f)
        ix = samo.samo_build_index(torch.from_numpy(data.mask).to(DEV))
        assert ix.nnz == idx.shape[0]
        gc16 = torch.full((ix.nnz,), float("nan"), dtype=torch.float16, device=DEV)
        one = torch.full((ix.nnz,), float("nan"), dtype=torch.float16, device=DEV)
        jobs.append((d_dy, d_x, ix.idx, ix.seg_ptr, gc16))
        single.append(one)
        keep.append((spec, idx, dy, x, ix))
    samo.samo_wgrad_gather_fp16_batched(jobs)
    for (d_dy, d_x, idx_d, seg_d, _), one in zip(jobs, single):
        samo.samo_wgrad_gather_fp16(d_dy, d_x, idx_d, seg_d, one)
    torch.cuda.synchronize()
    rng = np.random.default_rng(21)
    for (spec, idx, dy, x, _), (_, _, _, _, gc16), one in zip(keep, jobs, single):
        out_f, in_f, nnz = spec.rows, spec.cols, idx.shape[0]
        got = host_bits(gc16).view(np.float16)
        _check_rows_against_oracle(got, idx, dy, x, tokens, out_f, in_f, at_least=200_000, seed=21, name=spec.name)
        a, b = got.astype(np.float32), host_bits(one).view(np.float16).astype(np.float32)
        assert (a == b).mean() > 0.995, spec.name
        norm_dy = np.sqrt((dy.reshape(tokens, out_f).astype(np.float64) ** 2).sum(axis=0))
        norm_x = np.sqrt((x.reshape(tokens, in_f).astype(np.float64) ** 2).sum(axis=0))
        bound = (tokens + 2) * 2.0 ** -23 * norm_dy[idx // in_f] * norm_x[idx % in_f]
        ulp = np.maximum(np.abs(b), 2.0 ** -14) * 2.0 ** -10
        assert np.all(np.abs(a.astype(np.float64) - b) <= ulp + 2 * bound), spec.name + ": batched and single results further apart than two roundings allow"

