"""Python binding of libsamo — the SAMO compressed-parameter pipeline for MI355X.

Argument marshalling only: every function takes torch tensors that already live
on the GPU, passes their device pointers and the current HIP stream through the
C ABI declared in ``include/samo.h``, and returns.  All arithmetic and data
movement happens in the library's HIP kernels.  There is no CPU fallback: if the
shared library has not been built, importing the first symbol raises.

Names and semantics follow ``samo.h`` one to one (Section III of the paper):
``samo_build_index``, ``samo_decompress``, ``samo_gather_grads``,
``samo_adam_step``, ``samo_fused_step`` and the ``*_batched`` forms on a ``Plan``.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SAMO_LIBRARY_PATH") or os.path.join(_PKG, "libsamo.so")
SEG_ELEMS = 1024

ABI_VERSION = 4

SAMO_OK = 0
(SAMO_ERR_NULL, SAMO_ERR_SIZE, SAMO_ERR_ARG, SAMO_ERR_WORKSPACE, SAMO_ERR_ALIGN, SAMO_ERR_INDEX, SAMO_ERR_HIP,
 SAMO_ERR_PLAN) = -1, -2, -3, -4, -5, -6, -7, -8

# samo_debug_set knobs
(KNOB_OCC_TILE_STEP, KNOB_OCC_TILE_STEP32, KNOB_OCC_TILE_DECOMP, KNOB_OCC_TILE_C16, KNOB_OCC_FLAT_GATHER,
 KNOB_OCC_FLAT_STATS, KNOB_OCC_FLAT_STEP, KNOB_INDEX_SPIN_LIMIT, KNOB_WGRAD_TILE, KNOB_WGRAD_ROUND,
 KNOB_INDEX_PASSES, KNOB_TILE_COST) = range(12)
KNOB_DEFAULT = -1


class SamoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


class AdamCfg(ctypes.Structure):
    """samo_adam_cfg"""
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("decoupled_wd", ctypes.c_int32), ("step", ctypes.c_int32)]


class LayerDesc(ctypes.Structure):
    """samo_layer"""
    _fields_ = [("n", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("idx", ctypes.c_void_p), ("seg_ptr", ctypes.c_void_p),
                ("p", ctypes.c_void_p), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("w", ctypes.c_void_p), ("g", ctypes.c_void_p), ("gc", ctypes.c_void_p),
                ("gc16", ctypes.c_void_p), ("w32", ctypes.c_void_p), ("g32", ctypes.c_void_p)]


class PlanDesc(ctypes.Structure):
    """samo_plan"""
    _fields_ = [("d_layers", ctypes.c_void_p), ("d_tiles", ctypes.c_void_p), ("d_chunks", ctypes.c_void_p),
                ("num_tiles", ctypes.c_int64), ("num_chunks", ctypes.c_int64),
                ("n_total", ctypes.c_int64), ("nnz_total", ctypes.c_int64),
                ("num_layers", ctypes.c_int32), ("buffers", ctypes.c_uint32)]


class SgdCfg(ctypes.Structure):
    """samo_sgd_cfg"""
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float)]


class WgradJob(ctypes.Structure):
    """samo_wgrad_job"""
    _fields_ = [("d_dy", ctypes.c_void_p), ("d_x", ctypes.c_void_p), ("tokens", ctypes.c_int64),
                ("out", ctypes.c_int64), ("in_", ctypes.c_int64), ("d_idx", ctypes.c_void_p),
                ("d_seg_ptr", ctypes.c_void_p), ("nnz", ctypes.c_int64), ("d_gc", ctypes.c_void_p)]


SAMO_WGRAD_MAX_JOBS = 8


class StepGuard(ctypes.Structure):
    """samo_step_guard"""
    _fields_ = [("d_stats", ctypes.c_void_p), ("max_grad_norm", ctypes.c_float), ("skip_on_nonfinite", ctypes.c_int32)]


class IndexJob(ctypes.Structure):
    """samo_index_job"""
    _fields_ = [("mask", ctypes.c_void_p), ("n", ctypes.c_int64), ("idx", ctypes.c_void_p),
                ("idx_capacity", ctypes.c_int64), ("seg_ptr", ctypes.c_void_p), ("nnz", ctypes.c_void_p)]


_lib = None

_SIGNATURES = {
    "samo_status_string": (ctypes.c_char_p, [ctypes.c_int32]),
    "samo_abi_version": (ctypes.c_int32, []),
    "samo_init": (ctypes.c_int32, []),
    "samo_debug_set": (ctypes.c_int32, [ctypes.c_int32, ctypes.c_int32]),
    "samo_seg_ptr_len": (ctypes.c_int64, [ctypes.c_int64]),
    "samo_index_workspace_bytes": (ctypes.c_int32, [ctypes.c_int64, ctypes.POINTER(ctypes.c_size_t)]),
    "samo_count_nonzero": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p]),
    "samo_build_index": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "samo_build_index_batched": (ctypes.c_int32, [ctypes.POINTER(IndexJob), ctypes.c_int32, ctypes.c_void_p]),
    "samo_build_seg_ptr": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                            ctypes.c_void_p]),
    "samo_validate_index": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p]),
    "samo_decompress": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]),
    "samo_gather_grads": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                           ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p]),
    "samo_gather_grads_fp16": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                                ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]),
    "samo_sgd_step": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                       ctypes.POINTER(SgdCfg), ctypes.c_void_p]),
    "samo_adam_expand_step": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_float, ctypes.POINTER(AdamCfg),
                                               ctypes.c_void_p]),
    "samo_fused_sgd_step": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_float, ctypes.POINTER(SgdCfg), ctypes.c_void_p]),
    "samo_adam_step": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.POINTER(AdamCfg), ctypes.c_void_p]),
    "samo_fused_step": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_float, ctypes.POINTER(AdamCfg), ctypes.c_void_p]),
    "samo_fused_step_fp32": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_float, ctypes.POINTER(AdamCfg), ctypes.c_void_p]),
    "samo_fused_step_fp32_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_float, ctypes.POINTER(AdamCfg),
                                                      ctypes.POINTER(StepGuard), ctypes.c_void_p]),
    "samo_plan_workspace_bytes": (ctypes.c_int32, [ctypes.POINTER(LayerDesc), ctypes.c_int32,
                                                   ctypes.POINTER(ctypes.c_size_t)]),
    "samo_plan_init": (ctypes.c_int32, [ctypes.POINTER(LayerDesc), ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                        ctypes.c_void_p, ctypes.POINTER(PlanDesc)]),
    "samo_plan_stats_workspace_bytes": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.POINTER(ctypes.c_size_t)]),
    "samo_decompress_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_void_p]),
    "samo_gather_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_size_t, ctypes.c_void_p]),
    "samo_gather_fp16_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "samo_grad_stats_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                                                 ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "samo_static_scratch_bytes": (ctypes.c_size_t, []),
    "samo_grad_stats_batched_static": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_int32, ctypes.c_float,
                                                        ctypes.c_void_p, ctypes.c_void_p]),
    "samo_adam_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.POINTER(AdamCfg), ctypes.POINTER(StepGuard),
                                           ctypes.c_void_p]),
    "samo_fused_step_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_float, ctypes.POINTER(AdamCfg),
                                                 ctypes.POINTER(StepGuard), ctypes.c_void_p]),
    "samo_adam_expand_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_float, ctypes.POINTER(AdamCfg),
                                                  ctypes.POINTER(StepGuard), ctypes.c_void_p]),
    "samo_fused_sgd_step_batched": (ctypes.c_int32, [ctypes.POINTER(PlanDesc), ctypes.c_float, ctypes.POINTER(SgdCfg),
                                                     ctypes.POINTER(StepGuard), ctypes.c_void_p]),
    "samo_memory_model": (ctypes.c_int32, [ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64),
                                           ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
    "samo_wgrad_gather": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                           ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p]),
    "samo_wgrad_gather_fp16": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                                ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]),
    "samo_wgrad_gather_batched": (ctypes.c_int32, [ctypes.c_int32, ctypes.POINTER(WgradJob), ctypes.c_float,
                                                   ctypes.c_void_p]),
    "samo_wgrad_gather_fp16_batched": (ctypes.c_int32, [ctypes.c_int32, ctypes.POINTER(WgradJob), ctypes.c_int32,
                                                        ctypes.c_void_p]),
    "samo_stream_copy": (ctypes.c_int32, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]),
    "samo_mfma_rate_probe": (ctypes.c_int32, [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32,
                                              ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]),
}


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built — there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libsamo.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or `python -m paper_2302_05045_amd._build`) first; there is no CPU fallback")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        if handle.samo_abi_version() != ABI_VERSION:
            raise ImportError("libsamo.so has an unexpected ABI version")
        _lib = handle
    return _lib


def samo_init() -> None:
    """Per-device set-up outside stream capture (function attributes, static scratch address)."""
    _check(lib().samo_init(), "samo_init")


def samo_debug_set(knob: int, value: int = KNOB_DEFAULT) -> None:
    """Tuning / testing knob of the library (KNOB_*); KNOB_DEFAULT restores the built-in choice."""
    _check(lib().samo_debug_set(int(knob), int(value)), "samo_debug_set")


def samo_index_workspace_bytes(n: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().samo_index_workspace_bytes(int(n), ctypes.byref(out)), "samo_index_workspace_bytes")
    return out.value


def status_string(status: int) -> str:
    return lib().samo_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != SAMO_OK:
        raise SamoError(status, where)


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, name: str, length: Optional[int] = None) -> Optional[int]:
    """Device pointer of a contiguous 1-D CUDA tensor of the given dtype (None passes NULL)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a tensor on the GPU" % name)
    if t.dtype != dtype or t.dim() != 1 or not t.is_contiguous():
        raise TypeError("%s must be a contiguous 1-D %s tensor" % (name, dtype))
    if length is not None and t.numel() < length:
        raise ValueError("%s holds %d elements, needs %d" % (name, t.numel(), length))
    return t.data_ptr() if t.numel() else None


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


_F16 = torch.float16


def adam_cfg(step: int, lr: float = 1e-4, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
             weight_decay: float = 0.0, decoupled_wd: int = 0) -> AdamCfg:
    return AdamCfg(lr, beta1, beta2, eps, weight_decay, int(decoupled_wd), int(step))


def samo_seg_ptr_len(n: int) -> int:
    r = lib().samo_seg_ptr_len(int(n))
    if r < 0:
        raise SamoError(SAMO_ERR_SIZE, "samo_seg_ptr_len")
    return r


class Index(NamedTuple):
    idx: torch.Tensor       # int32[nnz]
    seg_ptr: torch.Tensor   # int32[ceil(n / 1024) + 1]
    nnz: int
    n: int


def samo_count_nonzero(mask: torch.Tensor, seg_ptr: torch.Tensor, nnz_out: torch.Tensor) -> None:
    n = mask.numel()
    _check(lib().samo_count_nonzero(_dev(mask, torch.uint8, "mask"), n,
                                    _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)),
                                    _dev(nnz_out, torch.int64, "nnz_out", 1), _stream()), "samo_count_nonzero")


def samo_build_index(mask: torch.Tensor) -> Index:
    """mask: uint8[n] on the GPU (non-zero keeps).  Counts, allocates idx, fills it.

    Reads the count back to size the index (one host synchronisation; the index is built
    once per pruning, not per iteration)."""
    n = mask.numel()
    seg_ptr = torch.empty(samo_seg_ptr_len(n), dtype=torch.int32, device=mask.device)
    nnz_out = torch.empty(1, dtype=torch.int64, device=mask.device)
    samo_count_nonzero(mask, seg_ptr, nnz_out)
    nnz = int(nnz_out.item())
    if nnz < 0:
        raise SamoError(SAMO_ERR_INDEX, "samo_count_nonzero (the device-side scan gave up)")
    idx = torch.empty(nnz, dtype=torch.int32, device=mask.device)
    samo_build_index_into(mask, idx, seg_ptr, nnz_out)
    return Index(idx, seg_ptr, nnz, n)


def samo_build_index_into(mask: torch.Tensor, idx: torch.Tensor, seg_ptr: torch.Tensor,
                          nnz_out: torch.Tensor) -> None:
    """Raw form: caller-provided idx (capacity = idx.numel()), seg_ptr and nnz_out (int64[1])."""
    n = mask.numel()
    _check(lib().samo_build_index(_dev(mask, torch.uint8, "mask"), n, _dev(idx, torch.int32, "idx"), idx.numel(),
                                  _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)),
                                  _dev(nnz_out, torch.int64, "nnz_out", 1), _stream()), "samo_build_index")


class IndexJobs:
    """The marshalled argument of samo_build_index_batched: the C job table plus references that
    keep its tensors alive.  Build it once, launch it as often as needed."""

    def __init__(self, masks: Sequence[torch.Tensor], idxs: Sequence[Optional[torch.Tensor]],
                 seg_ptrs: Sequence[torch.Tensor], nnz_out: torch.Tensor):
        k = len(masks)
        if not (len(idxs) == len(seg_ptrs) == k):
            raise ValueError("masks, idxs and seg_ptrs differ in length")
        nnz_ptr = _dev(nnz_out, torch.int64, "nnz_out", k) if k else None
        jobs = (IndexJob * max(k, 1))()
        for i in range(k):
            n = masks[i].numel()
            jobs[i].mask = _dev(masks[i], torch.uint8, "mask")
            jobs[i].n = n
            jobs[i].idx = _dev(idxs[i], torch.int32, "idx")
            jobs[i].idx_capacity = idxs[i].numel() if idxs[i] is not None else 0
            jobs[i].seg_ptr = _dev(seg_ptrs[i], torch.int32, "seg_ptr", samo_seg_ptr_len(n))
            jobs[i].nnz = nnz_ptr + 8 * i
        self.jobs, self.count = jobs, k
        self._keep = (list(masks), list(idxs), list(seg_ptrs), nnz_out)

    def launch(self) -> None:
        _check(lib().samo_build_index_batched(self.jobs, self.count, _stream()), "samo_build_index_batched")


def samo_build_index_batched(masks: Sequence[torch.Tensor], idxs: Sequence[Optional[torch.Tensor]],
                             seg_ptrs: Sequence[torch.Tensor], nnz_out: torch.Tensor) -> None:
    """Raw batched form: one job per mask; idxs[i] may be None (count only); nnz_out is int64[len(masks)]."""
    IndexJobs(masks, idxs, seg_ptrs, nnz_out).launch()


def samo_build_index_many(masks: Sequence[torch.Tensor]) -> list:
    """Index of every mask with a handful of launches: batched count, one read-back of the
    counts to size the indices, batched count + fill."""
    if not masks:
        return []
    dev = masks[0].device
    seg_ptrs = [torch.empty(samo_seg_ptr_len(m.numel()), dtype=torch.int32, device=dev) for m in masks]
    nnz_out = torch.empty(len(masks), dtype=torch.int64, device=dev)
    samo_build_index_batched(masks, [None] * len(masks), seg_ptrs, nnz_out)
    counts = nnz_out.cpu().tolist()
    if any(c < 0 for c in counts):
        raise SamoError(SAMO_ERR_INDEX, "samo_build_index_batched (the device-side scan gave up)")
    idxs = [torch.empty(c, dtype=torch.int32, device=dev) for c in counts]
    samo_build_index_batched(masks, idxs, seg_ptrs, nnz_out)
    return [Index(i, s, c, m.numel()) for i, s, c, m in zip(idxs, seg_ptrs, counts, masks)]


def samo_build_seg_ptr(idx: torch.Tensor, n: int) -> torch.Tensor:
    seg_ptr = torch.empty(samo_seg_ptr_len(n), dtype=torch.int32, device=idx.device)
    _check(lib().samo_build_seg_ptr(_dev(idx, torch.int32, "idx"), idx.numel(), int(n),
                                    _dev(seg_ptr, torch.int32, "seg_ptr"), _stream()), "samo_build_seg_ptr")
    return seg_ptr


def samo_validate_index(idx: torch.Tensor, n: int, seg_ptr: Optional[torch.Tensor] = None) -> bool:
    ok = torch.empty(1, dtype=torch.int32, device=idx.device)
    _check(lib().samo_validate_index(_dev(idx, torch.int32, "idx"), idx.numel(), int(n),
                                     _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)),
                                     _dev(ok, torch.int32, "ok"), _stream()), "samo_validate_index")
    return bool(ok.item())


def samo_decompress(p: torch.Tensor, idx: Optional[torch.Tensor], seg_ptr: Optional[torch.Tensor],
                    w: torch.Tensor) -> None:
    n, nnz = w.numel(), p.numel()
    _check(lib().samo_decompress(_dev(p, torch.float32, "p"), _dev(idx, torch.int32, "idx", nnz),
                                 _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)), nnz,
                                 _dev(w, _F16, "w"), n, _stream()), "samo_decompress")


def samo_gather_grads(g: torch.Tensor, idx: Optional[torch.Tensor], inv_loss_scale: float, gc: torch.Tensor) -> None:
    n, nnz = g.numel(), gc.numel()
    _check(lib().samo_gather_grads(_dev(g, _F16, "g"), n, _dev(idx, torch.int32, "idx", nnz), nnz,
                                   float(inv_loss_scale), _dev(gc, torch.float32, "gc"), _stream()),
           "samo_gather_grads")


def samo_gather_grads_fp16(g: torch.Tensor, idx: Optional[torch.Tensor], gc16: torch.Tensor,
                           accumulate: bool = False) -> None:
    n, nnz = g.numel(), gc16.numel()
    _check(lib().samo_gather_grads_fp16(_dev(g, _F16, "g"), n, _dev(idx, torch.int32, "idx", nnz), nnz,
                                        _dev(gc16, _F16, "gc16"), int(bool(accumulate)), _stream()),
           "samo_gather_grads_fp16")


def _dev_matrix(t: torch.Tensor, name: str) -> tuple:
    """(device pointer, rows, columns) of a contiguous 2-D fp16 CUDA tensor."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a tensor on the GPU" % name)
    if t.dtype != _F16 or t.dim() != 2 or not t.is_contiguous():
        raise TypeError("%s must be a contiguous 2-D float16 tensor" % name)
    return (t.data_ptr() if t.numel() else None), t.shape[0], t.shape[1]


def _wgrad_args(dy: torch.Tensor, x: torch.Tensor, idx: Optional[torch.Tensor], seg_ptr: Optional[torch.Tensor],
                nnz: int) -> tuple:
    dy_ptr, tokens, out_features = _dev_matrix(dy, "dy")
    x_ptr, tokens_x, in_features = _dev_matrix(x, "x")
    if tokens != tokens_x:
        raise ValueError("dy has %d rows (tokens), x has %d" % (tokens, tokens_x))
    n = out_features * in_features
    seg = _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)) if idx is not None else None
    return (dy_ptr, x_ptr, tokens, out_features, in_features, _dev(idx, torch.int32, "idx", nnz), seg, nnz)


def samo_wgrad_gather(dy: torch.Tensor, x: torch.Tensor, idx: Optional[torch.Tensor], seg_ptr: Optional[torch.Tensor],
                      inv_loss_scale: float, gc: torch.Tensor) -> None:
    """gc = the weight gradient dy^T x (tokens x out, tokens x in -> out x in), rounded to fp16, at idx,
    times inv_loss_scale."""
    nnz = gc.numel()
    _check(lib().samo_wgrad_gather(*_wgrad_args(dy, x, idx, seg_ptr, nnz), float(inv_loss_scale),
                                   _dev(gc, torch.float32, "gc"), _stream()), "samo_wgrad_gather")


def samo_wgrad_gather_fp16(dy: torch.Tensor, x: torch.Tensor, idx: Optional[torch.Tensor],
                           seg_ptr: Optional[torch.Tensor], gc16: torch.Tensor, accumulate: bool = False) -> None:
    """gc16 = that weight gradient, rounded to fp16, at idx; added to gc16 (in fp16) if accumulate."""
    nnz = gc16.numel()
    _check(lib().samo_wgrad_gather_fp16(*_wgrad_args(dy, x, idx, seg_ptr, nnz), _dev(gc16, _F16, "gc16"),
                                        int(bool(accumulate)), _stream()), "samo_wgrad_gather_fp16")


def _wgrad_jobs(jobs, dtype, name: str):
    """A samo_wgrad_job array from (dy, x, idx, seg_ptr, gc) tuples."""
    arr = (WgradJob * max(len(jobs), 1))()
    for j, (dy, x, idx, seg_ptr, gc) in enumerate(jobs):
        nnz = gc.numel()
        dy_ptr, x_ptr, tokens, out_features, in_features, idx_ptr, seg, _ = _wgrad_args(dy, x, idx, seg_ptr, nnz)
        arr[j] = WgradJob(dy_ptr, x_ptr, tokens, out_features, in_features, idx_ptr, seg, nnz,
                          _dev(gc, dtype, "%s of job %d" % (name, j)))
    return arr


def samo_wgrad_gather_batched(jobs, inv_loss_scale: float) -> None:
    """samo_wgrad_gather for every (dy, x, idx, seg_ptr, gc) of jobs (at most SAMO_WGRAD_MAX_JOBS), the
    layers' tiles dealt to the compute units as one list."""
    _check(lib().samo_wgrad_gather_batched(len(jobs), _wgrad_jobs(jobs, torch.float32, "gc"), float(inv_loss_scale),
                                           _stream()), "samo_wgrad_gather_batched")


def samo_wgrad_gather_fp16_batched(jobs, accumulate: bool = False) -> None:
    """samo_wgrad_gather_fp16 for every (dy, x, idx, seg_ptr, gc16) of jobs."""
    _check(lib().samo_wgrad_gather_fp16_batched(len(jobs), _wgrad_jobs(jobs, _F16, "gc16"), int(bool(accumulate)),
                                                _stream()), "samo_wgrad_gather_fp16_batched")


def sgd_cfg(lr: float, momentum: float = 0.9, weight_decay: float = 0.0) -> SgdCfg:
    return SgdCfg(lr, momentum, weight_decay)


def samo_sgd_step(p: torch.Tensor, buf: torch.Tensor, gc: torch.Tensor, cfg: SgdCfg) -> None:
    nnz = p.numel()
    _check(lib().samo_sgd_step(_dev(p, torch.float32, "p"), _dev(buf, torch.float32, "buf", nnz),
                               _dev(gc, torch.float32, "gc", nnz), nnz, ctypes.byref(cfg), _stream()),
           "samo_sgd_step")


def samo_adam_expand_step(gc16: torch.Tensor, w: torch.Tensor, idx: Optional[torch.Tensor],
                          seg_ptr: Optional[torch.Tensor], p: torch.Tensor, m: torch.Tensor, v: torch.Tensor,
                          inv_loss_scale: float, cfg: AdamCfg) -> None:
    n, nnz = w.numel(), p.numel()
    _check(lib().samo_adam_expand_step(_dev(gc16, _F16, "gc16", nnz), _dev(w, _F16, "w"), n,
                                       _dev(idx, torch.int32, "idx", nnz),
                                       _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)), nnz,
                                       _dev(p, torch.float32, "p"), _dev(m, torch.float32, "m", nnz),
                                       _dev(v, torch.float32, "v", nnz), float(inv_loss_scale), ctypes.byref(cfg),
                                       _stream()), "samo_adam_expand_step")


def samo_fused_sgd_step(g: torch.Tensor, w: torch.Tensor, idx: Optional[torch.Tensor],
                        seg_ptr: Optional[torch.Tensor], p: torch.Tensor, buf: torch.Tensor,
                        inv_loss_scale: float, cfg: SgdCfg) -> None:
    n, nnz = w.numel(), p.numel()
    _check(lib().samo_fused_sgd_step(_dev(g, _F16, "g", n), _dev(w, _F16, "w"), n,
                                     _dev(idx, torch.int32, "idx", nnz),
                                     _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)), nnz,
                                     _dev(p, torch.float32, "p"), _dev(buf, torch.float32, "buf", nnz),
                                     float(inv_loss_scale), ctypes.byref(cfg), _stream()), "samo_fused_sgd_step")


def samo_adam_step(p: torch.Tensor, m: torch.Tensor, v: torch.Tensor, gc: torch.Tensor, cfg: AdamCfg) -> None:
    nnz = p.numel()
    _check(lib().samo_adam_step(_dev(p, torch.float32, "p"), _dev(m, torch.float32, "m", nnz),
                                _dev(v, torch.float32, "v", nnz), _dev(gc, torch.float32, "gc", nnz), nnz,
                                ctypes.byref(cfg), _stream()), "samo_adam_step")


def samo_fused_step(g: torch.Tensor, w: torch.Tensor, idx: Optional[torch.Tensor], seg_ptr: Optional[torch.Tensor],
                    p: torch.Tensor, m: torch.Tensor, v: torch.Tensor, inv_loss_scale: float, cfg: AdamCfg) -> None:
    n, nnz = w.numel(), p.numel()
    _check(lib().samo_fused_step(_dev(g, _F16, "g", n), _dev(w, _F16, "w"), n, _dev(idx, torch.int32, "idx", nnz),
                                 _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)), nnz,
                                 _dev(p, torch.float32, "p"), _dev(m, torch.float32, "m", nnz),
                                 _dev(v, torch.float32, "v", nnz), float(inv_loss_scale), ctypes.byref(cfg),
                                 _stream()), "samo_fused_step")


def samo_fused_step_fp32(g32: torch.Tensor, w32: torch.Tensor, idx: Optional[torch.Tensor],
                         seg_ptr: Optional[torch.Tensor], m: torch.Tensor, v: torch.Tensor, grad_factor: float,
                         cfg: AdamCfg) -> None:
    n, nnz = w32.numel(), m.numel()
    _check(lib().samo_fused_step_fp32(_dev(g32, torch.float32, "g32", n), _dev(w32, torch.float32, "w32"), n,
                                      _dev(idx, torch.int32, "idx", nnz),
                                      _dev(seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(n)), nnz,
                                      _dev(m, torch.float32, "m"), _dev(v, torch.float32, "v", nnz),
                                      float(grad_factor), ctypes.byref(cfg), _stream()), "samo_fused_step_fp32")


class Layer(NamedTuple):
    """Device tensors of one layer for the batched entry points (None where unused)."""
    n: int
    idx: Optional[torch.Tensor]
    seg_ptr: Optional[torch.Tensor]
    p: Optional[torch.Tensor]
    m: Optional[torch.Tensor] = None
    v: Optional[torch.Tensor] = None
    w: Optional[torch.Tensor] = None
    g: Optional[torch.Tensor] = None
    gc: Optional[torch.Tensor] = None
    gc16: Optional[torch.Tensor] = None
    w32: Optional[torch.Tensor] = None      # single-precision SAMO: dense fp32 parameters
    g32: Optional[torch.Tensor] = None      # single-precision SAMO: dense fp32 gradient


class GradStats:
    """A device-resident samo_grad_stats plus the reduction workspace of a plan."""

    def __init__(self, plan: "Plan"):
        dev = plan.device
        self.buf = torch.zeros(2, dtype=torch.float64, device=dev)          # 16 bytes: double, int32, int32
        self.workspace = torch.empty(plan.stats_workspace_bytes(), dtype=torch.uint8, device=dev)

    @property
    def ptr(self) -> int:
        return self.buf.data_ptr()

    def read(self):
        """(sum_squares, nonfinite) — synchronises with the device."""
        host = self.buf.cpu()
        return float(host[0]), bool(host[1:2].view(torch.int32)[0].item())

    def guard(self, max_grad_norm: float = 0.0, skip_on_nonfinite: bool = False) -> StepGuard:
        return StepGuard(self.ptr, float(max_grad_norm), int(bool(skip_on_nonfinite)))


class ModelBuffers(list):
    """The list of Layers alloc_model returns, plus `gc16_bucket`: the one contiguous fp16 buffer that
    holds every layer's compressed gradient when it was asked for (None otherwise)."""
    gc16_bucket: Optional[torch.Tensor] = None


def alloc_model(shapes: Sequence[tuple], device, with_gc: bool = False, with_gc16: bool = False,
                align: int = 4096, bucket_gc16: bool = False) -> "ModelBuffers":
    """Device buffers for a whole model in ONE allocation, layer-major.

    shapes: (n, nnz, dense) per layer.  Returns one Layer per entry whose tensors are views of a
    single uint8 arena in the order seg_ptr, idx, p, g, m, v, w[, gc][, gc16] for layer 0, then layer 1, ...
    Keeping a layer's arrays adjacent in the address space is worth ~4 % of the fused step's
    bandwidth on MI355X compared with grouping the arrays by kind across layers (measured on the
    GPT-3 2.7B shape); m and v start at zero, everything else is uninitialised.  Every array starts on
    a multiple of `align` bytes: arrays that a wave walks at the same element offset run about 5 % slower
    when their starts do not agree modulo 1 KiB (measured on the flat Adam step).

    bucket_gc16: the compressed fp16 gradients of all layers are laid out back to back in one flat
    buffer of their own instead (each layer's slice starts on a 16-byte boundary; the padding
    elements are zero and no kernel touches them) — the single message a data-parallel all-reduce
    sends (Section IV-A of the paper); it is returned as `.gc16_bucket`.  Memory plumbing only: no
    arithmetic of the method happens here."""
    def rnd(x):
        return (x + align - 1) // align * align
    with_gc16 = with_gc16 or bucket_gc16
    plan, total, bucket_elems = [], 0, 0
    for n, nnz, dense in shapes:
        if dense and nnz != n:
            raise ValueError("a dense layer has nnz == n")
        seg = 0 if dense else 4 * samo_seg_ptr_len(n)
        sizes = [("seg_ptr", seg, torch.int32), ("idx", 0 if dense else 4 * nnz, torch.int32),
                 ("p", 4 * nnz, torch.float32), ("g", 2 * n, _F16), ("m", 4 * nnz, torch.float32),
                 ("v", 4 * nnz, torch.float32), ("w", 2 * n, _F16)]
        if with_gc:
            sizes.append(("gc", 4 * nnz, torch.float32))
        if with_gc16 and not bucket_gc16:
            sizes.append(("gc16", 2 * nnz, _F16))
        offs = {}
        for name, nb, dt in sizes:
            offs[name] = (total, nb, dt)
            total += rnd(nb)
        plan.append((n, nnz, dense, offs, bucket_elems))
        bucket_elems += (nnz + 7) // 8 * 8                      # 16-byte slices
    arena = torch.empty(max(total, 1), dtype=torch.uint8, device=device)
    bucket = torch.zeros(max(bucket_elems, 1), dtype=_F16, device=device) if bucket_gc16 else None
    layers = ModelBuffers()
    layers.gc16_bucket = bucket
    for n, nnz, dense, offs, at in plan:
        t = {name: arena[o:o + nb].view(dt) for name, (o, nb, dt) in offs.items()}
        t["m"].zero_()
        t["v"].zero_()
        gc16 = bucket[at:at + nnz] if bucket_gc16 else t.get("gc16")
        layers.append(Layer(n, None if dense else t["idx"], None if dense else t["seg_ptr"], t["p"], t["m"], t["v"],
                            t["w"], t["g"], t.get("gc"), gc16))
    return layers


def alloc_model_fp32(shapes: Sequence[tuple], device, align: int = 4096) -> list:
    """The same for single-precision SAMO: per layer seg_ptr, idx, g32, m, v, w32 in one arena
    (no compressed p, no 16-bit buffers); m and v start at zero."""
    def rnd(x):
        return (x + align - 1) // align * align
    plan, total = [], 0
    for n, nnz, dense in shapes:
        if dense and nnz != n:
            raise ValueError("a dense layer has nnz == n")
        sizes = [("seg_ptr", 0 if dense else 4 * samo_seg_ptr_len(n), torch.int32),
                 ("idx", 0 if dense else 4 * nnz, torch.int32), ("g32", 4 * n, torch.float32),
                 ("m", 4 * nnz, torch.float32), ("v", 4 * nnz, torch.float32), ("w32", 4 * n, torch.float32)]
        offs = {}
        for name, nb, dt in sizes:
            offs[name] = (total, nb, dt)
            total += rnd(nb)
        plan.append((n, dense, offs))
    arena = torch.empty(max(total, 1), dtype=torch.uint8, device=device)
    layers = []
    for n, dense, offs in plan:
        t = {name: arena[o:o + nb].view(dt) for name, (o, nb, dt) in offs.items()}
        t["m"].zero_()
        t["v"].zero_()
        layers.append(Layer(n, None if dense else t["idx"], None if dense else t["seg_ptr"], None, t["m"], t["v"],
                            w32=t["w32"], g32=t["g32"]))
    return layers


class Plan:
    """samo_plan: one launch per entry point over all layers of a model.  The plan's device tables
    live in a workspace allocated here through torch (the library itself allocates nothing)."""

    def __init__(self, layers: Sequence[Layer], workspace: Optional[torch.Tensor] = None):
        self._layers = list(layers)          # keeps the tensors alive
        self.device = next(((L.p if L.p is not None else L.m).device for L in self._layers),
                           torch.device("cuda", torch.cuda.current_device()))
        self._descs = (LayerDesc * max(len(self._layers), 1))()
        for d, L in zip(self._descs, self._layers):
            nnz = (L.p if L.p is not None else L.m).numel()      # a single-precision layer has no compressed p
            d.n, d.nnz = int(L.n), nnz
            d.idx = _dev(L.idx, torch.int32, "idx", nnz)
            d.seg_ptr = _dev(L.seg_ptr, torch.int32, "seg_ptr", samo_seg_ptr_len(L.n))
            d.p = _dev(L.p, torch.float32, "p")
            d.m = _dev(L.m, torch.float32, "m", nnz)
            d.v = _dev(L.v, torch.float32, "v", nnz)
            d.w = _dev(L.w, _F16, "w", L.n)
            d.g = _dev(L.g, _F16, "g", L.n)
            d.gc = _dev(L.gc, torch.float32, "gc", nnz)
            d.gc16 = _dev(L.gc16, _F16, "gc16", nnz)
            d.w32 = _dev(L.w32, torch.float32, "w32", L.n)
            d.g32 = _dev(L.g32, torch.float32, "g32", L.n)
        need = ctypes.c_size_t()
        _check(lib().samo_plan_workspace_bytes(self._descs, len(self._layers), ctypes.byref(need)),
               "samo_plan_workspace_bytes")
        self.workspace_bytes = need.value
        if workspace is None:
            workspace = torch.empty(max(need.value, 1), dtype=torch.uint8, device=self.device)
        self.workspace = workspace
        self._plan = PlanDesc()
        self.init()

    def init(self) -> None:
        """samo_plan_init on the current stream: (re)writes the plan's tables from the layers' seg_ptr as
        they are at that point of the stream.  Call again after the index has been rebuilt."""
        _check(lib().samo_plan_init(self._descs, len(self._layers), self.workspace.data_ptr(),
                                    self.workspace.numel(), _stream(), ctypes.byref(self._plan)), "samo_plan_init")

    @property
    def _handle(self):
        return ctypes.byref(self._plan)

    def close(self) -> None:
        """Nothing to release in the library; drops the references to the workspace and the layers."""
        self.workspace = None
        self._layers = []

    def totals(self):
        return self._plan.n_total, self._plan.nnz_total

    @property
    def num_tiles(self) -> int:
        """Workgroups of a tile-kernel launch over this plan (fused step, expansion)."""
        return self._plan.num_tiles

    def stats_workspace_bytes(self) -> int:
        out = ctypes.c_size_t()
        _check(lib().samo_plan_stats_workspace_bytes(self._handle, ctypes.byref(out)), "samo_plan_stats_workspace_bytes")
        return out.value

    @staticmethod
    def _stats_args(stats: Optional[GradStats]):
        if stats is None:
            return None, None, 0
        return stats.ptr, stats.workspace.data_ptr(), stats.workspace.numel()

    @staticmethod
    def _guard_arg(guard: Optional[StepGuard]):
        return ctypes.byref(guard) if guard is not None else None

    def samo_decompress_batched(self) -> None:
        _check(lib().samo_decompress_batched(self._handle, _stream()), "samo_decompress_batched")

    def samo_gather_batched(self, inv_loss_scale: float, stats: Optional[GradStats] = None) -> None:
        _check(lib().samo_gather_batched(self._handle, float(inv_loss_scale), *self._stats_args(stats), _stream()),
               "samo_gather_batched")

    def samo_gather_fp16_batched(self, accumulate: bool, inv_loss_scale: float,
                                 stats: Optional[GradStats] = None) -> None:
        _check(lib().samo_gather_fp16_batched(self._handle, int(bool(accumulate)), float(inv_loss_scale),
                                              *self._stats_args(stats), _stream()), "samo_gather_fp16_batched")

    def samo_grad_stats_batched(self, source: int, inv_loss_scale: float, stats: GradStats) -> None:
        _check(lib().samo_grad_stats_batched(self._handle, int(source), float(inv_loss_scale),
                                             *self._stats_args(stats), _stream()), "samo_grad_stats_batched")

    def samo_grad_stats_batched_static(self, source: int, inv_loss_scale: float, stats: GradStats) -> None:
        """The same with the partials in the library's static scratch array (no workspace, no allocation)."""
        _check(lib().samo_grad_stats_batched_static(self._handle, int(source), float(inv_loss_scale), stats.ptr,
                                                    _stream()), "samo_grad_stats_batched_static")

    def samo_adam_batched(self, cfg: AdamCfg, guard: Optional[StepGuard] = None) -> None:
        _check(lib().samo_adam_batched(self._handle, ctypes.byref(cfg), self._guard_arg(guard), _stream()),
               "samo_adam_batched")

    def samo_fused_step_batched(self, inv_loss_scale: float, cfg: AdamCfg, guard: Optional[StepGuard] = None) -> None:
        _check(lib().samo_fused_step_batched(self._handle, float(inv_loss_scale), ctypes.byref(cfg),
                                             self._guard_arg(guard), _stream()), "samo_fused_step_batched")

    def samo_fused_step_fp32_batched(self, grad_factor: float, cfg: AdamCfg, guard: Optional[StepGuard] = None) -> None:
        _check(lib().samo_fused_step_fp32_batched(self._handle, float(grad_factor), ctypes.byref(cfg),
                                                  self._guard_arg(guard), _stream()), "samo_fused_step_fp32_batched")

    def samo_adam_expand_batched(self, inv_loss_scale: float, cfg: AdamCfg, guard: Optional[StepGuard] = None) -> None:
        _check(lib().samo_adam_expand_batched(self._handle, float(inv_loss_scale), ctypes.byref(cfg),
                                              self._guard_arg(guard), _stream()), "samo_adam_expand_batched")

    def samo_fused_sgd_step_batched(self, inv_loss_scale: float, cfg: SgdCfg,
                                    guard: Optional[StepGuard] = None) -> None:
        _check(lib().samo_fused_sgd_step_batched(self._handle, float(inv_loss_scale), ctypes.byref(cfg),
                                                 self._guard_arg(guard), _stream()), "samo_fused_sgd_step_batched")


def samo_memory_model(n_total: int, nnz_total: int):
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().samo_memory_model(int(n_total), int(nnz_total), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)),
           "samo_memory_model")
    return a.value, b.value, c.value


def samo_mfma_rate_probe(iters: int, sink: torch.Tensor) -> float:
    """Launches the matrix-rate probe with one workgroup per element of sink (float32); returns its flops."""
    flops = ctypes.c_double(0.0)
    _check(lib().samo_mfma_rate_probe(int(iters), _dev(sink, torch.float32, "sink"), sink.numel(), ctypes.byref(flops),
                                      _stream()), "samo_mfma_rate_probe")
    return flops.value


def samo_stream_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst is smaller than src")
    _check(lib().samo_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream()), "samo_stream_copy")
