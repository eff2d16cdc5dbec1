"""The boundary's conventions on the GPU: every entry point only enqueues kernels on the caller's
stream — no allocation, copy or synchronisation inside the library — so index construction, plan
set-up and the optimizer step can sit in ONE HIP graph and follow a re-pruning on replay."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import DEV, INV, OCFG, assert_close, host_bits

pytestmark = pytest.mark.gpu


def _masks(specs, sparsity, salt):
    """Magnitude masks of every matrix from weights of another seed: a different pruning of the same shapes."""
    return [si.magnitude_mask(si.weights(s.n, s.seed + salt), sparsity) for s in specs]


def test_index_build_plan_init_and_fused_step_in_one_hip_graph_across_repruning():
    """Capture build index -> init plan -> fused step once; replay it after the masks changed (a
    re-pruning that keeps fewer elements than the buffers have room for).  Every replay is compared
    bit for bit with the same three calls made eagerly on buffers of their own, and with the oracle."""
    samo.samo_init()
    specs = si.config("gpt350m", 0.9, layers=1)                     # QKV, proj, FC1, FC2 of one layer
    weights = [si.weights(s.n, s.seed) for s in specs]
    grads = [si.grads_fp16(s.n, s.seed) for s in specs]
    prunings = [_masks(specs, 0.90, 0), _masks(specs, 0.93, 17), _masks(specs, 0.90, 29)]
    capacity = [int(m.sum()) for m in prunings[0]]
    cfg = samo.adam_cfg(1, **si.ADAM)

    class Side:
        def __init__(self):
            self.masks = [torch.zeros(s.n, dtype=torch.uint8, device=DEV) for s in specs]
            self.layers = samo.alloc_model([(s.n, c, False) for s, c in zip(specs, capacity)], DEV)
            self.nnz_out = torch.zeros(len(specs), dtype=torch.int64, device=DEV)
            self.jobs = samo.IndexJobs(self.masks, [L.idx for L in self.layers], [L.seg_ptr for L in self.layers],
                                       self.nnz_out)
            for L in self.layers:                                    # a valid (empty) index before the first build
                L.seg_ptr.zero_()
            self.plan = samo.Plan(self.layers)

        def load(self, masks):
            """What the training loop does after re-pruning: new masks, the kept weights compressed, fresh state."""
            for d_mask, mask, L, w in zip(self.masks, masks, self.layers, weights):
                d_mask.copy_(torch.from_numpy(mask))
                kept = np.ascontiguousarray(w[mask != 0])
                L.p.fill_(float("nan"))
                L.p[:kept.shape[0]].copy_(torch.from_numpy(kept))
                L.m.zero_()
                L.v.zero_()
                L.w.fill_(float("nan"))
                L.idx.fill_(-1)
                L.seg_ptr.fill_(-7)
            self.nnz_out.fill_(-3)

        def work(self):
            self.jobs.launch()
            self.plan.init()
            self.plan.samo_fused_step_batched(INV, cfg)

    graphed, eager = Side(), Side()
    for side in (graphed, eager):
        for L, g in zip(side.layers, grads):
            L.g.copy_(torch.from_numpy(g.view(np.int16)).view(torch.float16))
        side.load(prunings[0])
    side_stream = torch.cuda.Stream()
    side_stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side_stream):
        graphed.work()                                               # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    graphed.load(prunings[0])
    with torch.cuda.graph(graph):
        graphed.work()
    for rep, masks in enumerate(prunings):
        graphed.load(masks)
        eager.load(masks)
        torch.cuda.synchronize()
        eager.work()
        graph.replay()
        torch.cuda.synchronize()
        counts = [int(m.sum()) for m in masks]
        assert graphed.nnz_out.tolist() == counts == eager.nnz_out.tolist(), rep
        for a, b, s, mask, w, g, k in zip(graphed.layers, eager.layers, specs, masks, weights, grads, counts):
            assert k <= a.p.numel()
            idx = oracle.build_index(mask)
            assert np.array_equal(a.idx[:k].cpu().numpy(), idx), (rep, s.name)
            assert torch.equal(a.seg_ptr, b.seg_ptr), (rep, s.name)
            for ta, tb in ((a.p, b.p), (a.m, b.m), (a.v, b.v)):
                assert torch.equal(ta[:k], tb[:k]), (rep, s.name)
            assert torch.equal(a.w.view(torch.int16), b.w.view(torch.int16)), (rep, s.name)
            # nothing beyond the kept elements was touched
            assert torch.isnan(a.p[k:]).all() and not a.m[k:].any() and not a.v[k:].any(), (rep, s.name)
            p = np.ascontiguousarray(w[idx])
            m, v = np.zeros_like(p), np.zeros_like(p)
            oracle.step(g, s.n, idx, p, m, v, INV, OCFG, 1)
            got_p = a.p[:k].cpu().numpy()
            assert_close(got_p, p, "%s p, pruning %d" % (s.name, rep))
            assert_close(a.m[:k].cpu().numpy(), m, "%s m, pruning %d" % (s.name, rep))
            assert_close(a.v[:k].cpu().numpy(), v, "%s v, pruning %d" % (s.name, rep))
            assert np.array_equal(host_bits(a.w), oracle.decompress(got_p, idx, s.n)), (rep, s.name)


def test_plan_in_a_caller_workspace_and_too_small_workspaces():
    """samo_plan_init writes into the workspace it is given (here a slice of a larger buffer), the
    same plan can be initialised again after the index changed, and a workspace one byte short is
    rejected before anything is enqueued."""
    n, seed = 300_007, 41
    mask = si.bernoulli_mask(n, 0.2, seed)
    idx = oracle.build_index(mask)
    ix = samo.samo_build_index(torch.from_numpy(mask).to(DEV))
    layers = samo.alloc_model([(n, ix.nnz, False)], DEV)
    L = layers[0]
    L.idx.copy_(ix.idx)
    L.seg_ptr.copy_(ix.seg_ptr)
    p = np.ascontiguousarray(si.weights(n, seed)[idx])
    L.p.copy_(torch.from_numpy(p))
    big = torch.full((1 << 20,), 0x5A, dtype=torch.uint8, device=DEV)
    probe = samo.Plan(layers)
    need = probe.workspace_bytes
    assert 0 < need < big.numel() - 512
    plan = samo.Plan(layers, workspace=big[256:256 + need])
    plan.samo_decompress_batched()
    assert np.array_equal(host_bits(L.w), oracle.decompress(p, idx, n))
    assert bool((big[:256] == 0x5A).all()) and bool((big[256 + need:] == 0x5A).all())      # nothing outside the slice
    import ctypes
    out = samo.PlanDesc()
    rc = samo.lib().samo_plan_init(plan._descs, 1, big.data_ptr(), need - 1, None, ctypes.byref(out))
    assert rc == samo.SAMO_ERR_WORKSPACE and not out.d_layers
