"""The entry point that allocates nothing: samo_grad_stats_batched_static keeps its partial sums in
a static array inside the library's device image instead of a caller workspace.  Checked against
the workspace entry (bit-equal) and the oracle, on two calls in a row, the second on a smaller
model — the array keeps the first call's contents."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si
from gpu_util import DEV, INV

pytestmark = pytest.mark.gpu


def _model(sizes, seed):
    hosts, shapes = [], []
    for i, (n, keep) in enumerate(sizes):
        mask = si.bernoulli_mask(n, keep, seed + i)
        idx = oracle.build_index(mask)
        g = si.grads_fp16(n, seed + i)
        hosts.append((n, idx, g))
        shapes.append((n, idx.shape[0], False))
    layers = samo.alloc_model(shapes, DEV, with_gc16=True)
    for L, (n, idx, g) in zip(layers, hosts):
        L.idx.copy_(torch.from_numpy(idx))
        L.seg_ptr.copy_(samo.samo_build_seg_ptr(L.idx, n))
        L.g.copy_(torch.from_numpy(g.view(np.int16)).view(torch.float16))
        L.p.zero_()
    return hosts, layers, samo.Plan(layers)


def test_static_scratch_statistics_twice_second_call_smaller():
    samo.samo_init()
    assert samo.lib().samo_static_scratch_bytes() == 16 << 20
    first = [(2_000_003, 0.1), (1_048_576, 0.2), (300_007, 0.05), (4097, 1.0 - 1e-9)]     # ~ 430 k kept: two-level reduction
    second = [(100_003, 0.1), (5000, 0.3)]                                                  # ~ 11 k kept: one level
    for sizes, seed in ((first, 100), (second, 200)):
        hosts, layers, plan = _model(sizes, seed)
        for source in (0, 1):
            if source == 1:
                plan.samo_gather_fp16_batched(False, INV)
            with_ws, static = samo.GradStats(plan), samo.GradStats(plan)
            static.buf.fill_(float("nan"))
            plan.samo_grad_stats_batched(source, INV, with_ws)
            plan.samo_grad_stats_batched_static(source, INV, static)
            a, b = with_ws.read(), static.read()
            assert a == b and not b[1], (sizes, source)
            ref = sum(oracle.sum_squares(oracle.gather(g, idx, INV)) for n, idx, g in hosts)
            kept = sum(idx.shape[0] for _, idx, _ in hosts)
            assert abs(b[0] - ref) <= 2 * kept * 2.0 ** -53 * ref, (sizes, source)
        # a non-finite kept gradient is seen through the static array as well
        n, idx, g = hosts[0]
        g2 = g.copy()
        g2[idx[-1]] = 0x7C00
        layers[0].g.copy_(torch.from_numpy(g2.view(np.int16)).view(torch.float16))
        static = samo.GradStats(plan)
        plan.samo_grad_stats_batched_static(0, INV, static)
        assert static.read()[1] is True


def test_static_scratch_rejects_plans_beyond_its_size():
    """More partial sums than the static array holds: rejected on the host, nothing enqueued."""
    too_big = samo.PlanDesc()
    too_big.num_chunks = (16 << 20) // 16
    too_big.buffers = 0xFFFFFFFF
    stats = torch.zeros(2, dtype=torch.float64, device=DEV)
    rc = samo.lib().samo_grad_stats_batched_static(ctypes.byref(too_big), 0, 1.0, stats.data_ptr(), None)
    assert rc == samo.SAMO_ERR_SIZE
    assert "size" in samo.status_string(rc)
