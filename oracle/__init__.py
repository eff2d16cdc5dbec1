"""CPU oracle for the SAMO compressed-parameter pipeline — TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy wrapper over ``samo_oracle.c`` (plain scalar C loops written
from Section III of the paper) plus the analytic memory model of Section III-D.
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the GPU package
and the GPU package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import NamedTuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "samo_oracle.c")
_LIB = os.path.join(_HERE, "libsamo_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  No fast-math, no contraction, no OpenMP."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i64, i32, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_float
        vp = ctypes.c_void_p
        lib.samo_oracle_f32_to_f16.restype = ctypes.c_uint16
        lib.samo_oracle_f32_to_f16.argtypes = [f32]
        lib.samo_oracle_f16_to_f32.restype = f32
        lib.samo_oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.samo_oracle_f32_to_f16_array.restype = None
        lib.samo_oracle_f32_to_f16_array.argtypes = [vp, vp, i64]
        lib.samo_oracle_f16_to_f32_array.restype = None
        lib.samo_oracle_f16_to_f32_array.argtypes = [vp, vp, i64]
        lib.samo_oracle_build_index.restype = i64
        lib.samo_oracle_build_index.argtypes = [vp, i64, vp]
        lib.samo_oracle_decompress.restype = None
        lib.samo_oracle_decompress.argtypes = [vp, vp, i64, vp, i64]
        lib.samo_oracle_gather.restype = None
        lib.samo_oracle_gather.argtypes = [vp, vp, i64, f32, vp]
        lib.samo_oracle_compress_f16.restype = None
        lib.samo_oracle_compress_f16.argtypes = [vp, vp, i64, vp]
        lib.samo_oracle_f64_to_f16.restype = ctypes.c_uint16
        lib.samo_oracle_f64_to_f16.argtypes = [ctypes.c_double]
        lib.samo_oracle_accumulate_f16.restype = None
        lib.samo_oracle_accumulate_f16.argtypes = [vp, vp, i64, vp]
        lib.samo_oracle_upcast.restype = None
        lib.samo_oracle_upcast.argtypes = [vp, i64, f32, vp]
        lib.samo_oracle_sum_squares.restype = ctypes.c_double
        lib.samo_oracle_sum_squares.argtypes = [vp, i64]
        lib.samo_oracle_has_nonfinite.restype = i32
        lib.samo_oracle_has_nonfinite.argtypes = [vp, i64]
        lib.samo_oracle_scale.restype = None
        lib.samo_oracle_scale.argtypes = [vp, i64, f32]
        lib.samo_oracle_sgd.restype = None
        lib.samo_oracle_sgd.argtypes = [vp, vp, vp, i64, f32, f32, f32]
        lib.samo_oracle_adam.restype = None
        lib.samo_oracle_adam.argtypes = [vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i32, i32]
        lib.samo_oracle_step.restype = None
        lib.samo_oracle_step.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp, vp, f32,
                                         f32, f32, f32, f32, f32, i32, i32]
        lib.samo_oracle_compress_f32.restype = None
        lib.samo_oracle_compress_f32.argtypes = [vp, vp, i64, f32, vp]
        lib.samo_oracle_expand_f32.restype = None
        lib.samo_oracle_expand_f32.argtypes = [vp, vp, i64, vp, i64]
        lib.samo_oracle_step_fp32.restype = None
        lib.samo_oracle_step_fp32.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp, vp, f32,
                                              f32, f32, f32, f32, f32, i32, i32]
        _lib = lib
    return _lib


def _arr(a: np.ndarray, dtype, writable: bool = False) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != np.dtype(dtype) or a.ndim != 1 \
            or not a.flags.c_contiguous:
        raise TypeError("oracle expects a contiguous 1-D numpy array of %s" % np.dtype(dtype))
    if writable and not a.flags.writeable:
        raise TypeError("oracle output array is read-only")
    return a


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


class AdamCfg(NamedTuple):
    """Adam hyper-parameters; every field is rounded to fp32 before use."""
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    decoupled_wd: int = 0


# ----------------------------------------------------------------- fp16 <-> fp32
def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of IEEE binary16 bit patterns (RNE)."""
    x = _arr(x, np.float32)
    out = np.empty(x.shape[0], np.uint16)
    _load().samo_oracle_f32_to_f16_array(_ptr(x), _ptr(out), x.shape[0])
    return out


def f16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    h = _arr(h, np.uint16)
    out = np.empty(h.shape[0], np.float32)
    _load().samo_oracle_f16_to_f32_array(_ptr(h), _ptr(out), h.shape[0])
    return out


# ----------------------------------------------------------------- the pipeline
def build_index(mask: np.ndarray) -> np.ndarray:
    """Section III: ind_i — ascending flat positions j with mask[j] != 0, int32."""
    mask = _arr(mask, np.uint8)
    n = mask.shape[0]
    if n > 2**31 - 1:
        raise ValueError("a layer's flat size must fit int32 (Section III-B)")
    lib = _load()
    nnz = lib.samo_oracle_build_index(_ptr(mask), n, None)
    idx = np.empty(nnz, np.int32)
    got = lib.samo_oracle_build_index(_ptr(mask), n, _ptr(idx))
    assert got == nnz
    return idx


def decompress(p: np.ndarray, idx: np.ndarray, n: int, w: np.ndarray | None = None) -> np.ndarray:
    """Section III-C "expansion": dense fp16 bits (uint16[n]), zeros off the index."""
    p = _arr(p, np.float32)
    idx = _arr(idx, np.int32)
    if p.shape[0] != idx.shape[0]:
        raise ValueError("p and idx differ in length")
    if w is None:
        w = np.empty(n, np.uint16)
    w = _arr(w, np.uint16, writable=True)
    if w.shape[0] != n:
        raise ValueError("w has the wrong length")
    _check_index(idx, n)
    _load().samo_oracle_decompress(_ptr(p), _ptr(idx), idx.shape[0], _ptr(w), n)
    return w


def gather(g: np.ndarray, idx: np.ndarray, inv_loss_scale: float) -> np.ndarray:
    """Section III-C compression of a layer's dense fp16 gradient + fp32 up-cast + unscale."""
    g = _arr(g, np.uint16)
    idx = _arr(idx, np.int32)
    _check_index(idx, g.shape[0])
    gc = np.empty(idx.shape[0], np.float32)
    _load().samo_oracle_gather(_ptr(g), _ptr(idx), idx.shape[0], np.float32(inv_loss_scale), _ptr(gc))
    return gc


def compress_f16(dense: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Section III-B compression of a dense fp16 tensor: the values at ind."""
    dense = _arr(dense, np.uint16)
    idx = _arr(idx, np.int32)
    _check_index(idx, dense.shape[0])
    out = np.empty(idx.shape[0], np.uint16)
    _load().samo_oracle_compress_f16(_ptr(dense), _ptr(idx), idx.shape[0], _ptr(out))
    return out


def f64_to_f16_bits_scalar(x: float) -> int:
    return int(_load().samo_oracle_f64_to_f16(float(x)))


def accumulate_f16(g: np.ndarray, idx: np.ndarray, gc16: np.ndarray) -> None:
    """gc16[i] <- fp16(gc16[i] + g[idx[i]]), correctly rounded: one more micro-batch into the
    stored compressed fp16 gradient (Section III-A; micro-batches, Section II-E)."""
    g = _arr(g, np.uint16)
    idx = _arr(idx, np.int32)
    gc16 = _arr(gc16, np.uint16, True)
    if gc16.shape[0] != idx.shape[0]:
        raise ValueError("gc16 and idx differ in length")
    _check_index(idx, g.shape[0])
    _load().samo_oracle_accumulate_f16(_ptr(g), _ptr(idx), idx.shape[0], _ptr(gc16))


def upcast(gc16: np.ndarray, inv_loss_scale: float) -> np.ndarray:
    """Section III-C optimizer step, first operation: compressed fp16 -> fp32, times 1/loss scale."""
    gc16 = _arr(gc16, np.uint16)
    gc = np.empty(gc16.shape[0], np.float32)
    _load().samo_oracle_upcast(_ptr(gc16), gc16.shape[0], np.float32(inv_loss_scale), _ptr(gc))
    return gc


def sum_squares(gc: np.ndarray) -> float:
    gc = _arr(gc, np.float32)
    return float(_load().samo_oracle_sum_squares(_ptr(gc), gc.shape[0]))


def has_nonfinite(gc: np.ndarray) -> bool:
    gc = _arr(gc, np.float32)
    return bool(_load().samo_oracle_has_nonfinite(_ptr(gc), gc.shape[0]))


def clip_coefficient(total_sum_squares: float, max_norm: float) -> np.float32:
    """Gradient clipping by global norm, as torch.nn.utils.clip_grad_norm_ defines it:
    coef = min(1, max_norm / (norm + 1e-6)), rounded to fp32."""
    norm = float(np.sqrt(total_sum_squares))
    return np.float32(min(1.0, max_norm / (norm + 1e-6)))


def scale(gc: np.ndarray, coef: float) -> None:
    gc = _arr(gc, np.float32, True)
    _load().samo_oracle_scale(_ptr(gc), gc.shape[0], np.float32(coef))


def sgd(p: np.ndarray, buf: np.ndarray, gc: np.ndarray, lr: float, momentum: float, weight_decay: float = 0.0) -> None:
    """In-place SGD with momentum on the compressed fp32 tensors (one state per parameter)."""
    p = _arr(p, np.float32, True)
    buf = _arr(buf, np.float32, True)
    gc = _arr(gc, np.float32)
    if not (buf.shape[0] == gc.shape[0] == p.shape[0]):
        raise ValueError("compressed tensors differ in length")
    _load().samo_oracle_sgd(_ptr(p), _ptr(buf), _ptr(gc), p.shape[0], lr, momentum, weight_decay)


def adam(p: np.ndarray, m: np.ndarray, v: np.ndarray, gc: np.ndarray, cfg: AdamCfg, step: int) -> None:
    """In-place Adam on the compressed fp32 tensors (Section III-C, III-D)."""
    p = _arr(p, np.float32, True)
    m = _arr(m, np.float32, True)
    v = _arr(v, np.float32, True)
    gc = _arr(gc, np.float32)
    nnz = p.shape[0]
    if not (m.shape[0] == v.shape[0] == gc.shape[0] == nnz):
        raise ValueError("compressed tensors differ in length")
    if step < 1:
        raise ValueError("Adam's step counter starts at 1")
    _load().samo_oracle_adam(_ptr(p), _ptr(m), _ptr(v), _ptr(gc), nnz,
                             cfg.lr, cfg.beta1, cfg.beta2, cfg.eps,
                             cfg.weight_decay, int(cfg.decoupled_wd), int(step))


def step(g: np.ndarray, n: int, idx: np.ndarray, p: np.ndarray, m: np.ndarray, v: np.ndarray,
         inv_loss_scale: float, cfg: AdamCfg, t: int, w: np.ndarray | None = None) -> np.ndarray:
    """gather -> adam -> decompress for one layer; updates p, m, v in place, returns w bits."""
    g = _arr(g, np.uint16)
    idx = _arr(idx, np.int32)
    p = _arr(p, np.float32, True)
    m = _arr(m, np.float32, True)
    v = _arr(v, np.float32, True)
    nnz = idx.shape[0]
    if g.shape[0] != n or not (p.shape[0] == m.shape[0] == v.shape[0] == nnz):
        raise ValueError("shape mismatch")
    if t < 1:
        raise ValueError("Adam's step counter starts at 1")
    _check_index(idx, n)
    if w is None:
        w = np.empty(n, np.uint16)
    w = _arr(w, np.uint16, True)
    gc = np.empty(nnz, np.float32)
    _load().samo_oracle_step(_ptr(g), _ptr(w), n, _ptr(idx), nnz, _ptr(p), _ptr(m), _ptr(v),
                             _ptr(gc), np.float32(inv_loss_scale),
                             cfg.lr, cfg.beta1, cfg.beta2, cfg.eps,
                             cfg.weight_decay, int(cfg.decoupled_wd), int(t))
    return w


# ----------------------------------------------------------------- single-precision SAMO
def compress_f32(dense: np.ndarray, idx: np.ndarray, factor: float = 1.0) -> np.ndarray:
    """Values of a dense fp32 tensor at idx, times `factor` (one fp32 multiply)."""
    dense = _arr(dense, np.float32)
    idx = _arr(idx, np.int32)
    _check_index(idx, dense.shape[0])
    out = np.empty(idx.shape[0], np.float32)
    _load().samo_oracle_compress_f32(_ptr(dense), _ptr(idx), idx.shape[0], np.float32(factor), _ptr(out))
    return out


def expand_f32(c: np.ndarray, idx: np.ndarray, n: int) -> np.ndarray:
    """Dense fp32 tensor of n elements: c at idx, +0 elsewhere."""
    c = _arr(c, np.float32)
    idx = _arr(idx, np.int32)
    if c.shape[0] != idx.shape[0]:
        raise ValueError("shape mismatch")
    _check_index(idx, n)
    dense = np.empty(n, np.float32)
    _load().samo_oracle_expand_f32(_ptr(c), _ptr(idx), idx.shape[0], _ptr(dense), n)
    return dense


def step_fp32(g32: np.ndarray, w32: np.ndarray, idx: np.ndarray, m: np.ndarray, v: np.ndarray,
              grad_factor: float, cfg: AdamCfg, t: int) -> None:
    """One single-precision optimizer phase of a layer: updates the dense w32 (kept positions
    stepped, every other position +0) and the compressed m, v in place."""
    g32 = _arr(g32, np.float32)
    w32 = _arr(w32, np.float32, True)
    idx = _arr(idx, np.int32)
    m = _arr(m, np.float32, True)
    v = _arr(v, np.float32, True)
    n, nnz = w32.shape[0], idx.shape[0]
    if g32.shape[0] != n or not (m.shape[0] == v.shape[0] == nnz):
        raise ValueError("shape mismatch")
    if t < 1:
        raise ValueError("Adam's step counter starts at 1")
    _check_index(idx, n)
    gc = np.empty(nnz, np.float32)
    pc = np.empty(nnz, np.float32)
    _load().samo_oracle_step_fp32(_ptr(g32), _ptr(w32), n, _ptr(idx), nnz, _ptr(m), _ptr(v), _ptr(gc), _ptr(pc),
                                  np.float32(grad_factor), cfg.lr, cfg.beta1, cfg.beta2, cfg.eps,
                                  cfg.weight_decay, int(cfg.decoupled_wd), int(t))


# ----------------------------------------------------------------- compression in the backward pass
def _f16_matrix(bits: np.ndarray, rows: int, cols: int) -> np.ndarray:
    bits = _arr(bits, np.uint16)
    if bits.shape[0] != rows * cols:
        raise ValueError("matrix of %d x %d needs %d elements, got %d" % (rows, cols, rows * cols, bits.shape[0]))
    return bits.view(np.float16).reshape(rows, cols).astype(np.float64)


def linear_weight_grad(dy: np.ndarray, x: np.ndarray, tokens: int, out_features: int, in_features: int) -> np.ndarray:
    """Gradient of a fully connected layer's weight (Section I: a linear transform of the layer's
    input; taken as Y = X W^T for W of shape out x in, the usual framework convention):
    dW[o, i] = sum over tokens t of dY[t, o] * X[t, i], in double precision from the fp16
    operands (dy: tokens x out, x: tokens x in, both row-major fp16 bit patterns).
    Returned flattened row-major, as the layer's index counts positions."""
    a = _f16_matrix(dy, tokens, out_features)
    b = _f16_matrix(x, tokens, in_features)
    return (a.T @ b).reshape(-1)


def linear_weight_grad_magnitude(dy: np.ndarray, x: np.ndarray, tokens: int, out_features: int,
                                 in_features: int) -> np.ndarray:
    """sum_t |dY[t, o]| * |X[t, i]|: what the rounding error of any summation order of
    linear_weight_grad is proportional to (used by tests to size their tolerance)."""
    a = np.abs(_f16_matrix(dy, tokens, out_features))
    b = np.abs(_f16_matrix(x, tokens, in_features))
    return (a.T @ b).reshape(-1)


def wgrad_compress(dy: np.ndarray, x: np.ndarray, tokens: int, out_features: int, in_features: int,
                   idx: np.ndarray) -> np.ndarray:
    """What the backward pass followed by compression leaves (Section III-C: the dense fp16
    gradient of a layer is compressed as soon as it is produced): the weight gradient rounded
    once to fp16, taken at idx.  Returns fp16 bit patterns."""
    idx = _arr(idx, np.int32)
    _check_index(idx, out_features * in_features)
    dense = linear_weight_grad(dy, x, tokens, out_features, in_features)
    with np.errstate(over="ignore"):
        return dense[idx].astype(np.float16).view(np.uint16)


def wgrad_at(dy: np.ndarray, x: np.ndarray, tokens: int, out_features: int, in_features: int,
             positions: np.ndarray) -> tuple:
    """linear_weight_grad and its magnitude sum at a few flattened positions only, one dot product
    per position (for layers too large to form densely on the host)."""
    a = _arr(dy, np.uint16).view(np.float16).reshape(tokens, out_features)
    b = _arr(x, np.uint16).view(np.float16).reshape(tokens, in_features)
    positions = np.asarray(positions, np.int64)
    if positions.size and (positions.min() < 0 or positions.max() >= out_features * in_features):
        raise ValueError("position outside the weight matrix")
    rows, cols = positions // in_features, positions % in_features
    val = np.empty(positions.shape[0], np.float64)
    mag = np.empty(positions.shape[0], np.float64)
    for k in range(positions.shape[0]):
        u = a[:, rows[k]].astype(np.float64)
        w = b[:, cols[k]].astype(np.float64)
        val[k] = np.dot(u, w)
        mag[k] = np.dot(np.abs(u), np.abs(w))
    return val, mag


def wgrad_rows(dy: np.ndarray, x: np.ndarray, tokens: int, out_features: int, in_features: int,
               rows: np.ndarray) -> tuple:
    """linear_weight_grad and its magnitude sum for whole rows of dW (the output features in
    `rows`): returns two fp64 arrays of len(rows) x in_features, entry [r][i] =
    sum_t dY[t][rows[r]] * X[t][i] and sum_t |dY[t][rows[r]] * X[t][i]| — the same definition as
    linear_weight_grad, one fp64 matrix product over the chosen output features only, so that a
    few hundred thousand outputs of a full-size layer can be checked without forming all of dW."""
    a = _arr(dy, np.uint16).view(np.float16).reshape(tokens, out_features)
    b = _arr(x, np.uint16).view(np.float16).reshape(tokens, in_features).astype(np.float64)
    rows = np.asarray(rows, np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= out_features):
        raise ValueError("row outside the weight matrix")
    u = a[:, rows].astype(np.float64)                       # tokens x len(rows)
    return u.T @ b, np.abs(u).T @ np.abs(b)


def _check_index(idx: np.ndarray, n: int) -> None:
    if idx.shape[0] == 0:
        return
    if idx[0] < 0 or idx[-1] >= n or (idx.shape[0] > 1 and not np.all(idx[1:] > idx[:-1])):
        raise ValueError("index must be strictly ascending and within [0, n)")


# ----------------------------------------------------------------- Section III-D
class MemoryModel(NamedTuple):
    default_bytes: int      # M^default = 20 phi
    samo_bytes: int         # M^SAMO    = 24 f phi + 2 phi   (Eq. 1-2)
    saved_bytes: int        # (24 p - 6) phi                 (Eq. 4-5)
    saved_fraction: float   # saved / default


def memory_model(phi: int, nnz: int) -> MemoryModel:
    """Model-state bytes of Section III-D for phi parameters of which nnz are unpruned.

    Default mixed precision: theta16 2, grad16 2, theta32 4, grad32 4, os 8 bytes
    per parameter.  SAMO: 18 bytes per unpruned parameter (grad16 2, theta32 4,
    grad32 4, os 8), a 4-byte index and a 2-byte temporary fp16 copy per unpruned
    parameter, plus the dense theta16 at 2 bytes per parameter.
    """
    default = (2 + 2 + 4 + 4 + 8) * phi
    samo = 18 * nnz + 4 * nnz + 2 * phi + 2 * nnz
    return MemoryModel(default, samo, default - samo, (default - samo) / default if phi else 0.0)


def resident_bytes(phi: int, nnz: int) -> int:
    """Bytes the fused single-GPU pipeline keeps resident: idx + p + m + v per
    unpruned parameter (4 each) and the dense fp16 weights (2 per parameter);
    the fp16/fp32 compressed gradients and the temporary fp16 copy of Section
    III-D are never materialised by a fused step."""
    return 16 * nnz + 2 * phi
