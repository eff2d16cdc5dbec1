"""Seeded synthetic inputs for the SAMO pipeline: shapes, masks, weights, gradients.

This module serves both the CPU oracle's tests and the GPU path's tests/bench.
It holds none of the method's arithmetic: it only draws random tensors and
pruning masks with the shapes and sparsity structure of the paper's GPT-3
workloads (Table I; 90 % pruning, Section V), using numpy on the host.

Everything is a pure function of its integer seeds.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Callable, Iterator, NamedTuple

import numpy as np

# Hyper-parameters common to every configuration (inputs of the method, not part of it).
LOSS_SCALE = 1024.0
ADAM = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, decoupled_wd=0)
W_STD = 0.02
G_STD = 1e-3

_STREAM_W, _STREAM_MASK, _STREAM_G, _STREAM_ROWS, _STREAM_P, _STREAM_X, _STREAM_DY = range(7)


def _rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), stream, int(sub)])))


# ------------------------------------------------------------------ tensors
def _to_fp16_bits(x: np.ndarray) -> np.ndarray:
    """IEEE round-to-nearest-even fp32 -> fp16 bit patterns (torch's vectorised CPU cast; numpy's
    scalar cast gives the same bits but is an order of magnitude slower on model-sized tensors)."""
    import torch
    return torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)


def weights(n: int, seed: int) -> np.ndarray:
    """fp32 master weights ~ N(0, 0.02)."""
    w = _rng(seed, _STREAM_W).standard_normal(n, dtype=np.float32)
    w *= np.float32(W_STD)
    return w


def grads_fp16(n: int, seed: int, step: int = 1, loss_scale: float = LOSS_SCALE) -> np.ndarray:
    """Dense fp16 gradient bits (uint16): fp16(N(0, 1e-3) * loss_scale), a fresh draw per step.

    Non-zero everywhere, so pruned positions carry garbage the method must ignore."""
    g = _rng(seed, _STREAM_G, step).standard_normal(n, dtype=np.float32)
    g *= np.float32(G_STD * loss_scale)
    return _to_fp16_bits(g)


def grads_fp32(n: int, seed: int, step: int = 1) -> np.ndarray:
    """Dense fp32 gradient ~ N(0, 1e-3) for single-precision SAMO (no loss scale), fresh per step."""
    g = _rng(seed, _STREAM_G, step).standard_normal(n, dtype=np.float32)
    g *= np.float32(G_STD)
    return g


def activations_fp16(tokens: int, features: int, seed: int, step: int = 1) -> np.ndarray:
    """Input of a fully connected layer, tokens x features row-major fp16 bits ~ N(0, 1)
    (what a layer norm hands to the layer)."""
    x = _rng(seed, _STREAM_X, step).standard_normal(tokens * features, dtype=np.float32)
    return _to_fp16_bits(x)


def output_grads_fp16(tokens: int, features: int, seed: int, step: int = 1,
                      loss_scale: float = LOSS_SCALE) -> np.ndarray:
    """Gradient arriving at a fully connected layer's output, tokens x features row-major fp16
    bits ~ N(0, G_STD * loss_scale / sqrt(tokens)), so that the weight gradient it forms with
    activations_fp16 has the spread of grads_fp16."""
    dy = _rng(seed, _STREAM_DY, step).standard_normal(tokens * features, dtype=np.float32)
    dy *= np.float32(G_STD * loss_scale / np.sqrt(float(tokens)))
    return _to_fp16_bits(dy)


# ------------------------------------------------------------------ masks (uint8, != 0 keeps)
def bernoulli_mask(n: int, keep: float, seed: int) -> np.ndarray:
    return (_rng(seed, _STREAM_MASK).random(n) < keep).astype(np.uint8)


def kept_count(n: int, sparsity: float) -> int:
    """Number of kept entries at a given pruned fraction: round-half-up of (1 - p) * n."""
    return int(np.floor((1.0 - sparsity) * n + 0.5))


def magnitude_mask(w: np.ndarray, sparsity: float) -> np.ndarray:
    """Keep the k largest |w| (k = kept_count); ties at the threshold keep the lower flat index."""
    n = w.shape[0]
    k = kept_count(n, sparsity)
    mask = np.zeros(n, np.uint8)
    if k <= 0:
        return mask
    if k >= n:
        mask[:] = 1
        return mask
    a = np.abs(w)
    thr = np.partition(a, n - k)[n - k]
    above = a > thr
    mask[above] = 1
    need = k - int(np.count_nonzero(above))
    if need > 0:
        ties = np.flatnonzero(a == thr)[:need]
        mask[ties] = 1
    return mask


def row_clustered_mask(rows: int, cols: int, sparsity: float, seed: int) -> np.ndarray:
    """10 % of the rows ("hot") are 10x denser than the rest; overall density = 1 - sparsity.

    d_cold = (1-p)/1.9, d_hot = min(1, 10 d_cold); if d_hot clamps, d_cold is
    re-solved from 0.1 d_hot + 0.9 d_cold = 1-p.  Bernoulli within rows."""
    dens = 1.0 - sparsity
    d_cold = dens / 1.9
    d_hot = min(1.0, 10.0 * d_cold)
    if d_hot >= 1.0:
        d_cold = (dens - 0.1 * d_hot) / 0.9
    n_hot = int(round(0.1 * rows))
    hot = _rng(seed, _STREAM_ROWS).permutation(rows)[:n_hot]
    row_d = np.full(rows, d_cold, np.float32)
    row_d[hot] = d_hot
    rng = _rng(seed, _STREAM_MASK)
    mask = np.empty(rows * cols, np.uint8)
    chunk = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        u = rng.random((r1 - r0, cols), dtype=np.float32)
        mask[r0 * cols:r1 * cols] = (u < row_d[r0:r1, None]).reshape(-1)
    return mask


def edge_masks(n: int) -> dict:
    """Degenerate masks every index/scatter/gather implementation must survive."""
    out = {
        "all_zero": np.zeros(n, np.uint8),
        "all_one": np.ones(n, np.uint8),
        "first_only": np.zeros(n, np.uint8),
        "last_only": np.zeros(n, np.uint8),
        "alternating": (np.arange(n) & 1).astype(np.uint8),
        "every_64": (np.arange(n) % 64 == 0).astype(np.uint8),
        "every_65": (np.arange(n) % 65 == 64).astype(np.uint8),
        "nonunit_values": ((np.arange(n) % 7 == 3) * 0x80).astype(np.uint8),
    }
    if n:
        out["first_only"][0] = 1
        out["last_only"][-1] = 1
    return out


# ------------------------------------------------------------------ model shapes
class Matrix(NamedTuple):
    name: str
    rows: int
    cols: int
    seed: int
    sparsity: float      # pruned fraction p; < 0 means "left dense"
    mask_kind: str       # "bernoulli" | "magnitude" | "row_clustered" | "dense"

    @property
    def n(self) -> int:
        return self.rows * self.cols


def gpt_layer_shapes(hidden: int, ffn: int) -> list:
    """The four weight matrices of one transformer layer: QKV, attention proj, FC1, FC2."""
    return [("qkv", hidden, 3 * hidden), ("proj", hidden, hidden),
            ("fc1", hidden, ffn), ("fc2", ffn, hidden)]


def matrix_seed(base: int, layer: int, m: int) -> int:
    return base * 1_000_000 + 4 * layer + m


def gpt_matrices(layers: int, hidden: int, ffn: int, sparsity: float, base_seed: int,
                 mask_kind: str = "magnitude") -> list:
    out = []
    for l in range(layers):
        for mi, (name, r, c) in enumerate(gpt_layer_shapes(hidden, ffn)):
            out.append(Matrix("l%d.%s" % (l, name), r, c, matrix_seed(base_seed, l, mi), sparsity, mask_kind))
    return out


def config(name: str, sparsity: float = 0.9, layers: int | None = None) -> list:
    """The benchmark configurations, as lists of Matrix descriptors.

    fc1024    one 1024x1024 FC layer, Bernoulli keep 0.1, seed 0
    gpt350m   24 layers, hidden 1024, FFN 4096, magnitude masks
    gpt1.3b   24 layers, hidden 2048, FFN 8192
    gpt2.7b   32 layers, hidden 2560, FFN 10240 (sparsity 0.80 / 0.90 / 0.95)
    gpt6.7b   32 layers, hidden 4096, FFN 16384, per-matrix sparsity ~ U[0.8, 0.97],
              row-clustered masks, plus a dense 50304x4096 embedding
    `layers` truncates the model (for bounded samples of the same workload)."""
    if name == "fc1024":
        return [Matrix("fc", 1024, 1024, 0, 0.9, "bernoulli")]
    table = {"gpt350m": (24, 1024, 4096, 2), "gpt1.3b": (24, 2048, 8192, 3),
             "gpt2.7b": (32, 2560, 10240, 4), "gpt6.7b": (32, 4096, 16384, 5)}
    if name not in table:
        raise KeyError(name)
    nl, h, ffn, base = table[name]
    nl = nl if layers is None else min(nl, layers)
    if name != "gpt6.7b":
        return gpt_matrices(nl, h, ffn, sparsity, base)
    mats = []
    ps = _rng(base, _STREAM_P).uniform(0.8, 0.97, size=32 * 4)
    for l in range(nl):
        for mi, (nm, r, c) in enumerate(gpt_layer_shapes(h, ffn)):
            mats.append(Matrix("l%d.%s" % (l, nm), r, c, matrix_seed(base, l, mi),
                               float(ps[4 * l + mi]), "row_clustered"))
    mats.append(Matrix("embedding", 50304, 4096, matrix_seed(base, 999, 0), -1.0, "dense"))
    return mats


class LayerData(NamedTuple):
    spec: Matrix
    w32: np.ndarray      # fp32[n] dense master weights before pruning
    mask: np.ndarray     # uint8[n]
    g16: np.ndarray      # uint16[n] fp16 bits of the dense scaled gradient


def make_mask(spec: Matrix, w32: np.ndarray | None) -> np.ndarray:
    if spec.mask_kind == "bernoulli":
        return bernoulli_mask(spec.n, 1.0 - spec.sparsity, spec.seed)
    if spec.mask_kind == "magnitude":
        return magnitude_mask(w32 if w32 is not None else weights(spec.n, spec.seed), spec.sparsity)
    if spec.mask_kind == "row_clustered":
        return row_clustered_mask(spec.rows, spec.cols, spec.sparsity, spec.seed)
    if spec.mask_kind == "dense":
        return np.ones(spec.n, np.uint8)
    raise KeyError(spec.mask_kind)


def make_layer(spec: Matrix, step: int = 1) -> LayerData:
    w32 = weights(spec.n, spec.seed)
    return LayerData(spec, w32, make_mask(spec, w32), grads_fp16(spec.n, spec.seed, step))


def generate(specs: list, consume: Callable[[int, LayerData], None], workers: int = 8,
             step: int = 1) -> None:
    """Generate layers on a small thread pool and hand each to `consume(i, data)` in order.

    At most `workers` layers are alive at once, so model-sized configurations stream
    through host memory instead of being held whole."""
    if workers <= 1:
        for i, s in enumerate(specs):
            consume(i, make_layer(s, step))
        return
    with ThreadPoolExecutor(max_workers=workers) as pool:
        pending = []
        it: Iterator = iter(enumerate(specs))
        for _ in range(workers):
            nxt = next(it, None)
            if nxt is None:
                break
            pending.append((nxt[0], pool.submit(make_layer, nxt[1], step)))
        while pending:
            i, fut = pending.pop(0)
            data = fut.result()
            nxt = next(it, None)
            if nxt is not None:
                pending.append((nxt[0], pool.submit(make_layer, nxt[1], step)))
            consume(i, data)
            del data
