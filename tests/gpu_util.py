"""Helpers shared by the GPU parity tests (host<->device moves and the comparison rules)."""
import numpy as np
import torch

import oracle
import paper_2302_05045_amd as samo
import samo_inputs as si

DEV = torch.device("cuda:0")
OCFG = oracle.AdamCfg(**si.ADAM)
INV = 1.0 / si.LOSS_SCALE
TOL = 1e-6          # relative tolerance on fp32 p, m, v fixed by the benchmark spec


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def dev_f16_bits(bits):
    """uint16 fp16 bit patterns -> torch.float16 tensor on the GPU, bits preserved."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.float16)


def host_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def nan_f16(n):
    return torch.full((n,), float("nan"), dtype=torch.float16, device=DEV)


def ref_seg_ptr(idx, n):
    """Defining property of seg_ptr: number of kept positions below each multiple of 1024."""
    nseg = (n + samo.SEG_ELEMS - 1) // samo.SEG_ELEMS
    return np.searchsorted(idx, np.arange(nseg + 1, dtype=np.int64) * samo.SEG_ELEMS, side="left").astype(np.int32)


def assert_close(got, ref, what, tol=TOL):
    """|a-b| <= tol * max(|a|,|b|) + tol * rms(ref): relative 1e-6, with an absolute floor that
    absorbs cancellation in beta*m + (1-beta)*g for entries far below the tensor's scale."""
    got64, ref64 = got.astype(np.float64), ref.astype(np.float64)
    assert got.shape == ref.shape, what
    if ref.size == 0:
        return
    atol = tol * float(np.sqrt(np.mean(ref64 * ref64)))
    err = np.abs(got64 - ref64)
    bound = tol * np.maximum(np.abs(got64), np.abs(ref64)) + atol
    bad = np.flatnonzero(~(err <= bound))
    assert bad.size == 0, "%s: %d of %d outside tolerance, first at %d: got %r ref %r" % (
        what, bad.size, ref.size, bad[0], got[bad[0]], ref[bad[0]])


class HostLayer:
    """One layer's inputs on the host plus the oracle's compressed state."""

    def __init__(self, n, mask, w32, seed, dense=False):
        self.n, self.mask, self.seed, self.dense = n, mask, seed, dense
        self.idx = oracle.build_index(mask)
        self.p = np.ascontiguousarray(w32[self.idx])
        self.m = np.zeros_like(self.p)
        self.v = np.zeros_like(self.p)

    def grads(self, t):
        return si.grads_fp16(self.n, self.seed, t)


class DevLayer:
    """The same layer resident on the GPU; the index is built by the library from the mask."""

    def __init__(self, h: HostLayer, with_gc=False, with_gc16=False):
        self.h = h
        if h.dense:
            self.idx = self.seg_ptr = None
        else:
            ix = samo.samo_build_index(dev_u8(h.mask))
            self.idx, self.seg_ptr = ix.idx, ix.seg_ptr
            assert ix.nnz == h.idx.shape[0]
        self.p, self.m, self.v = dev_f32(h.p), dev_f32(h.m), dev_f32(h.v)
        self.w = nan_f16(h.n)
        self.g = nan_f16(h.n)
        self.gc = torch.full((h.p.shape[0],), float("nan"), device=DEV) if with_gc else None
        self.gc16 = torch.full((h.p.shape[0],), float("nan"), dtype=torch.float16, device=DEV) if with_gc16 else None

    def set_grads(self, bits):
        self.g.copy_(dev_f16_bits(bits))

    def layer(self):
        return samo.Layer(self.h.n, self.idx, self.seg_ptr, self.p, self.m, self.v, self.w, self.g, self.gc, self.gc16)
