"""Thin ctypes binding over the C-ABI library (include/isopo.h).

Argument marshalling only: every step of the layer step runs in the library's
kernels.  torch supplies device memory and the stream.  There is no CPU
fallback: if libisopo.so is missing the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libisopo.so")
_lib = None

OK = 0
F32, BF16 = 0, 1
GRAM_AUTO, GRAM_GHOST, GRAM_MATERIALISED = 0, 1, 2
STASH_ROW_MAJOR, STASH_TILE_ORDER = 0, 1
KEEP_ROW_MAJOR, KEEP_FAST = 1, 2          # keep_stash values of layer_gram
VARIANT_FISHER, VARIANT_INTERACTING = 0, 1
REG_ABSOLUTE, REG_REL_TRACE, REG_EMA_TRACE = 0, 1, 2
MAX_SEQ = 1024

_VARIANTS = {"fisher": VARIANT_FISHER, "interacting": VARIANT_INTERACTING}
_PATHS = {"auto": GRAM_AUTO, "ghost": GRAM_GHOST, "materialised": GRAM_MATERIALISED}
_PATH_NAMES = {v: k for k, v in _PATHS.items()}

EXPORTS = ("isopo_layer_gram_plan", "isopo_gram_cost_model", "isopo_contraction_plan", "isopo_layer_gram",
           "isopo_stash_layout_of", "isopo_weighted_grad_stash", "isopo_weighted_grad_stash_bf16", "isopo_seq_grads_stash",
           "isopo_transform_ema", "isopo_seq_grads_limited", "isopo_seq_grads",
           "isopo_stash_gram_workspace", "isopo_stash_gram", "isopo_transform_workspace",
           "isopo_transform", "isopo_transform_noalloc", "isopo_weighted_grad", "isopo_scale_rows",
           "isopo_fisher_samples_workspace", "isopo_fisher_samples",
           "isopo_fisher_samples_group_workspace", "isopo_fisher_samples_group",
           "isopo_fisher_samples_block_workspace", "isopo_fisher_samples_block",
           "isopo_weighted_grad_scratch", "isopo_weighted_grad_prescaled",
           "isopo_gram_norms", "isopo_rescale", "isopo_ntk_eigh_workspace", "isopo_ntk_eigh",
           "isopo_transform_eigh", "isopo_probe_mfma_loop", "isopo_probe_lds_dma", "isopo_probe_contraction_waves", "isopo_status_string", "isopo_version")


class IsopoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class _RescaleParams(ctypes.Structure):
    _fields_ = [("p", ctypes.c_float), ("q", ctypes.c_float), ("r", ctypes.c_float),
                ("reg", ctypes.c_float * 3), ("expectation", ctypes.c_float * 3)]


class _Layer(ctypes.Structure):
    _fields_ = [("X", ctypes.c_void_p), ("Delta", ctypes.c_void_p), ("dtype", ctypes.c_int),
                ("n_tokens", ctypes.c_int64), ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32),
                ("n_seq", ctypes.c_int32), ("seq_offsets_dev", ctypes.c_void_p),
                ("seq_offsets_host", ctypes.c_void_p)]


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libisopo.so (built by `python -m paper_2512_23353_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is not built; run `python -m paper_2512_23353_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, i32, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_float
    lp = ctypes.POINTER(_Layer)
    lib.isopo_layer_gram_plan.argtypes = [lp, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(sz),
                                          ctypes.POINTER(sz)]
    lib.isopo_layer_gram_plan.restype = ctypes.c_int
    lib.isopo_gram_cost_model.argtypes = [lp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.isopo_gram_cost_model.restype = ctypes.c_int
    lib.isopo_contraction_plan.argtypes = [lp, ctypes.c_int, vp]
    lib.isopo_contraction_plan.restype = ctypes.c_int
    lib.isopo_layer_gram.argtypes = [lp, ctypes.c_int, vp, vp, sz, ctypes.c_int, vp]
    lib.isopo_layer_gram.restype = ctypes.c_int
    lib.isopo_seq_grads.argtypes = [lp, vp, vp]
    lib.isopo_seq_grads.restype = ctypes.c_int
    lib.isopo_seq_grads_limited.argtypes = [lp, vp, i32, vp, vp]
    lib.isopo_seq_grads_limited.restype = ctypes.c_int
    lib.isopo_seq_grads_stash.argtypes = [lp, vp, ctypes.c_int, i32, vp, vp]
    lib.isopo_seq_grads_stash.restype = ctypes.c_int
    lib.isopo_stash_gram_workspace.argtypes = [i32]
    lib.isopo_stash_gram_workspace.restype = sz
    lib.isopo_stash_gram.argtypes = [vp, ctypes.c_int, i32, ctypes.c_int64, vp, vp, sz, vp]
    lib.isopo_stash_gram.restype = ctypes.c_int
    lib.isopo_transform_workspace.argtypes = [i32, i32]
    lib.isopo_transform_workspace.restype = sz
    lib.isopo_transform.argtypes = [vp, vp, i32, i32, ctypes.c_int, f32, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.isopo_transform.restype = ctypes.c_int
    lib.isopo_transform_noalloc.argtypes = [vp, vp, i32, i32, ctypes.c_int, f32, ctypes.c_int, vp, vp, vp]
    lib.isopo_transform_noalloc.restype = ctypes.c_int
    lib.isopo_transform_ema.argtypes = [vp, vp, i32, i32, ctypes.c_int, f32, vp, f32, vp, vp, vp, sz, vp]
    lib.isopo_transform_ema.restype = ctypes.c_int
    lib.isopo_weighted_grad.argtypes = [lp, vp, vp, f32, vp, vp]
    lib.isopo_weighted_grad.restype = ctypes.c_int
    lib.isopo_stash_layout_of.argtypes = [lp, vp, vp]
    lib.isopo_stash_layout_of.restype = ctypes.c_int
    lib.isopo_weighted_grad_stash.argtypes = [lp, vp, vp, ctypes.c_int, f32, vp, vp]
    lib.isopo_weighted_grad_stash.restype = ctypes.c_int
    lib.isopo_weighted_grad_stash_bf16.argtypes = [lp, vp, vp, ctypes.c_int, f32, vp, vp]
    lib.isopo_weighted_grad_stash_bf16.restype = ctypes.c_int
    lib.isopo_scale_rows.argtypes = [vp, ctypes.c_int, ctypes.c_int64, i32, vp, i32, vp, vp, vp]
    lib.isopo_scale_rows.restype = ctypes.c_int
    lib.isopo_fisher_samples_workspace.argtypes = [lp, i32]
    lib.isopo_fisher_samples_workspace.restype = sz
    lib.isopo_fisher_samples.argtypes = [lp, vp, i32, vp, f32, ctypes.c_int, vp, f32, vp, vp, vp, sz, vp]
    lib.isopo_fisher_samples.restype = ctypes.c_int
    lib.isopo_fisher_samples_group_workspace.argtypes = [lp, i32, i32]
    lib.isopo_fisher_samples_group_workspace.restype = sz
    lib.isopo_fisher_samples_group.argtypes = [ctypes.POINTER(lp), i32, vp, i32, vp, f32, ctypes.c_int, vp, f32, vp, vp,
                                               vp, sz, vp]
    lib.isopo_fisher_samples_group.restype = ctypes.c_int
    lib.isopo_fisher_samples_block_workspace.argtypes = [lp, i32, i32]
    lib.isopo_fisher_samples_block_workspace.restype = sz
    lib.isopo_fisher_samples_block.argtypes = [ctypes.POINTER(lp), ctypes.POINTER(i32), i32, vp, i32, vp, f32, ctypes.c_int,
                                               vp, f32, vp, vp, vp, sz, vp]
    lib.isopo_fisher_samples_block.restype = ctypes.c_int
    lib.isopo_weighted_grad_scratch.argtypes = [lp]
    lib.isopo_weighted_grad_scratch.restype = sz
    lib.isopo_weighted_grad_prescaled.argtypes = [lp, vp, f32, vp, vp, sz, vp]
    lib.isopo_weighted_grad_prescaled.restype = ctypes.c_int
    lib.isopo_gram_norms.argtypes = [vp, i32, vp, vp, vp]
    lib.isopo_gram_norms.restype = ctypes.c_int
    lib.isopo_rescale.argtypes = [vp, vp, ctypes.c_int64, i32, vp, ctypes.POINTER(_RescaleParams), vp, vp, vp]
    lib.isopo_rescale.restype = ctypes.c_int
    lib.isopo_ntk_eigh_workspace.argtypes = [i32, i32]
    lib.isopo_ntk_eigh_workspace.restype = sz
    lib.isopo_ntk_eigh.argtypes = [vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.isopo_ntk_eigh.restype = ctypes.c_int
    lib.isopo_transform_eigh.argtypes = [vp, vp, i32, i32, vp, ctypes.POINTER(ctypes.c_float), i32, ctypes.c_int, vp, f32,
                                         vp, vp, vp]
    lib.isopo_transform_eigh.restype = ctypes.c_int
    lib.isopo_probe_mfma_loop.argtypes = [i32, vp, vp, i32, vp]
    lib.isopo_probe_mfma_loop.restype = ctypes.c_int
    lib.isopo_probe_lds_dma.argtypes = [vp, sz, i32, i32, i32, i32, vp, vp]
    lib.isopo_probe_lds_dma.restype = ctypes.c_int
    lib.isopo_probe_contraction_waves.argtypes = [lp, i32, vp, vp]
    lib.isopo_probe_contraction_waves.restype = ctypes.c_int
    lib.isopo_status_string.argtypes = [ctypes.c_int]
    lib.isopo_status_string.restype = ctypes.c_char_p
    lib.isopo_version.argtypes = []
    lib.isopo_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().isopo_status_string(int(status)).decode()


def version() -> str:
    return load().isopo_version().decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise IsopoError(status, where)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Layer:
    """One ragged layer problem.  Keeps the host offsets and the device copies
    alive for as long as the C struct is in use."""

    def __init__(self, X: Optional[torch.Tensor], Delta: Optional[torch.Tensor], seq_offsets,
                 seq_offsets_dev: Optional[torch.Tensor] = None, d_in: Optional[int] = None,
                 d_out: Optional[int] = None, dtype: Optional[int] = None, n_tokens: Optional[int] = None):
        self.X, self.Delta = X, Delta
        self.off_host = np.ascontiguousarray(np.asarray(seq_offsets, dtype=np.int32))
        if X is not None:
            if X.dtype != Delta.dtype or X.dim() != 2 or Delta.dim() != 2:
                raise ValueError("X and Delta must be 2-D tensors of one dtype")
            if not (X.is_contiguous() and Delta.is_contiguous()):
                raise ValueError("X and Delta must be contiguous (row-major)")
            if X.dtype not in (torch.float32, torch.bfloat16):
                raise IsopoError(3, "Layer")
            dtype = BF16 if X.dtype == torch.bfloat16 else F32
            d_in, d_out, n_tokens = X.shape[1], Delta.shape[1], X.shape[0]
            if Delta.shape[0] != n_tokens:
                raise ValueError("X and Delta must have the same number of token rows")
            if seq_offsets_dev is None and X.is_cuda:
                seq_offsets_dev = torch.from_numpy(self.off_host).to(X.device)
        self.off_dev = seq_offsets_dev
        self.d_in, self.d_out, self.dtype = int(d_in), int(d_out), int(dtype)
        self.n_seq = int(self.off_host.size - 1)
        self.n_tokens = int(n_tokens)
        self.c = _Layer(_ptr(X), _ptr(Delta), self.dtype, self.n_tokens, self.d_in, self.d_out, self.n_seq,
                        _ptr(self.off_dev), self.off_host.ctypes.data)

    @property
    def device(self):
        return self.X.device

    def ref(self):
        return ctypes.byref(self.c)


def gram_plan(layer: Layer, path="auto") -> Tuple[str, int, int]:
    """(chosen path, ws_full bytes, ws_min bytes).  Host only."""
    chosen, full, mn = ctypes.c_int(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().isopo_layer_gram_plan(layer.ref(), _PATHS[path], ctypes.byref(chosen), ctypes.byref(full),
                                        ctypes.byref(mn)), "isopo_layer_gram_plan")
    return _PATH_NAMES[chosen.value], int(full.value), int(mn.value)


def gram_cost_model(layer: Layer) -> Tuple[float, float]:
    tg, tm = ctypes.c_double(), ctypes.c_double()
    _check(load().isopo_gram_cost_model(layer.ref(), ctypes.byref(tg), ctypes.byref(tm)), "isopo_gram_cost_model")
    return tg.value, tm.value


class ContractionPlanInfo(ctypes.Structure):
    _fields_ = [("tile", ctypes.c_int32), ("workgroups_per_cu", ctypes.c_int32), ("tiles", ctypes.c_int32),
                ("n_chunks", ctypes.c_int32), ("chunk_tokens", ctypes.c_int32), ("xcd_start", ctypes.c_int32 * 9),
                ("workgroups", ctypes.c_int64), ("whole_tiles", ctypes.c_int32)]


def contraction_plan(layer_ref, per_sequence: bool) -> dict:
    """Launch plan of the bf16 contraction (host arithmetic only).  `layer_ref`: an isopo_layer struct
    (Layer.ref(), or one built on the host with null device pointers)."""
    info = ContractionPlanInfo()
    _check(load().isopo_contraction_plan(layer_ref, int(bool(per_sequence)), ctypes.byref(info)),
           "isopo_contraction_plan")
    return {"tile": info.tile, "workgroups_per_cu": info.workgroups_per_cu, "tiles": info.tiles,
            "n_chunks": info.n_chunks, "chunk_tokens": info.chunk_tokens, "xcd_start": list(info.xcd_start),
            "workgroups": info.workgroups, "whole_tiles": info.whole_tiles}


def alloc_workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def layer_gram(layer: Layer, path="auto", K: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, keep_stash=False, stream=None):
    """K [n_seq, n_seq] fp32.  Returns (K, workspace); with keep_stash the stash
    lies at the start of the workspace: True / KEEP_ROW_MAJOR as [n_seq, d_out, d_in],
    KEEP_FAST in the layout stash_layout(layer) reports (for weighted_grad's `layout`)."""
    if K is None:
        K = torch.empty((layer.n_seq, layer.n_seq), dtype=torch.float32, device=layer.device)
    if workspace is None:
        _, full, mn = gram_plan(layer, path)
        workspace = alloc_workspace(full, layer.device)
    _check(load().isopo_layer_gram(layer.ref(), _PATHS[path], K.data_ptr(), workspace.data_ptr(),
                                   workspace.numel(), int(keep_stash), _stream(stream)), "isopo_layer_gram")
    return K, workspace


def stash_nbytes(layer: Layer) -> int:
    return layer.n_seq * layer.d_out * layer.d_in * (2 if layer.dtype == BF16 else 4)


def seq_grads(layer: Layer, stash: Optional[torch.Tensor] = None, stream=None, max_workgroups: int = 0,
              queue: Optional[torch.Tensor] = None, layout: Optional[int] = None) -> torch.Tensor:
    """The stash of per-sequence gradients [n_seq, d_out, d_in] in the input dtype.  max_workgroups > 0:
    at most that many compute units are used (queue: int32/uint32 device tensor of 8 elements, scratch).
    layout = STASH_TILE_ORDER: the same elements in tile order (see stash_layout)."""
    if stash is None:
        stash = torch.empty((layer.n_seq, layer.d_out, layer.d_in), dtype=layer.X.dtype, device=layer.device)
    if layout is not None:
        if max_workgroups and queue is None:
            queue = torch.zeros(8, dtype=torch.int32, device=layer.device)
        _check(load().isopo_seq_grads_stash(layer.ref(), stash.data_ptr(), int(layout), int(max_workgroups),
                                            _ptr(queue) if max_workgroups else None, _stream(stream)),
               "isopo_seq_grads_stash")
    elif max_workgroups:
        if queue is None:
            queue = torch.zeros(8, dtype=torch.int32, device=layer.device)
        _check(load().isopo_seq_grads_limited(layer.ref(), stash.data_ptr(), int(max_workgroups), queue.data_ptr(),
                                              _stream(stream)), "isopo_seq_grads_limited")
    else:
        _check(load().isopo_seq_grads(layer.ref(), stash.data_ptr(), _stream(stream)), "isopo_seq_grads")
    return stash


def stash_gram(stash: torch.Tensor, K: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
               stream=None) -> torch.Tensor:
    """K from a stash [n_seq, d_out, d_in] (or any [n_seq, n_elem] view of it)."""
    n_seq = stash.shape[0]
    n_elem = stash.numel() // n_seq
    if K is None:
        K = torch.empty((n_seq, n_seq), dtype=torch.float32, device=stash.device)
    if workspace is None:
        workspace = alloc_workspace(load().isopo_stash_gram_workspace(n_seq), stash.device)
    dtype = BF16 if stash.dtype == torch.bfloat16 else F32
    _check(load().isopo_stash_gram(stash.data_ptr(), dtype, n_seq, n_elem, K.data_ptr(), workspace.data_ptr(),
                                   workspace.numel(), _stream(stream)), "isopo_stash_gram")
    return K


def transform_workspace(n_seq: int, batch: int = 1) -> int:
    return int(load().isopo_transform_workspace(n_seq, batch))


def transform(K: torch.Tensor, A: torch.Tensor, variant="fisher", lam: float = 0.0, reg_mode: int = REG_ABSOLUTE,
              c: Optional[torch.Tensor] = None, info: Optional[torch.Tensor] = None,
              workspace: Optional[torch.Tensor] = None, stream=None):
    """c from K [batch?, m, m] and A [batch?, m].  Returns (c, info)."""
    m = K.shape[-1]
    batch = 1 if K.dim() == 2 else K.shape[0]
    if K.dtype != torch.float32 or A.dtype != torch.float32 or not K.is_contiguous() or not A.is_contiguous():
        raise ValueError("K and A must be contiguous fp32")
    if c is None:
        c = torch.empty_like(A)
    if info is None:
        info = torch.zeros(batch, dtype=torch.int32, device=K.device)
    need = transform_workspace(m, batch)
    if workspace is None and need:
        workspace = alloc_workspace(need, K.device)
    _check(load().isopo_transform(K.data_ptr(), A.data_ptr(), m, batch, _VARIANTS[variant], float(lam),
                                  int(reg_mode), c.data_ptr(), info.data_ptr(), _ptr(workspace),
                                  0 if workspace is None else workspace.numel(), _stream(stream)), "isopo_transform")
    return c, info


NOALLOC_SCRATCH_BYTES = 16 << 20


def transform_noalloc(K: torch.Tensor, A: torch.Tensor, variant, lam: float, reg_mode: int, c: torch.Tensor,
                      info: Optional[torch.Tensor] = None, stream=None):
    """isopo_transform_noalloc: every buffer comes from the caller (c and info included), nothing is allocated
    here or in the library; the scratch is the library's per-GPU array.  Returns (c, info)."""
    m = K.shape[-1]
    batch = 1 if K.dim() == 2 else K.shape[0]
    if K.dtype != torch.float32 or A.dtype != torch.float32 or not K.is_contiguous() or not A.is_contiguous():
        raise ValueError("K and A must be contiguous fp32")
    _check(load().isopo_transform_noalloc(K.data_ptr(), A.data_ptr(), m, batch, _VARIANTS[variant], float(lam),
                                          int(reg_mode), c.data_ptr(), _ptr(info), _stream(stream)),
           "isopo_transform_noalloc")
    return c, info


def transform_ema(K: torch.Tensor, A: torch.Tensor, variant, factor: float, ema_state: torch.Tensor,
                  ema_decay: float = 0.9, c: Optional[torch.Tensor] = None, info: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None):
    """transform() with reg = factor * trailing mean over minibatches of tr(K)/m; ema_state [batch?, 2]
    fp32 on the device is read and updated.  Returns (c, info)."""
    m = K.shape[-1]
    batch = 1 if K.dim() == 2 else K.shape[0]
    if K.dtype != torch.float32 or A.dtype != torch.float32 or not K.is_contiguous() or not A.is_contiguous():
        raise ValueError("K and A must be contiguous fp32")
    if ema_state.dtype != torch.float32 or ema_state.numel() != 2 * batch or not ema_state.is_contiguous():
        raise ValueError("ema_state must be contiguous fp32 [batch, 2]")
    if c is None:
        c = torch.empty_like(A)
    if info is None:
        info = torch.zeros(batch, dtype=torch.int32, device=K.device)
    need = transform_workspace(m, batch)
    if workspace is None and need:
        workspace = alloc_workspace(need, K.device)
    _check(load().isopo_transform_ema(K.data_ptr(), A.data_ptr(), m, batch, _VARIANTS[variant], float(factor),
                                      ema_state.data_ptr(), float(ema_decay), c.data_ptr(), info.data_ptr(),
                                      _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                      _stream(stream)), "isopo_transform_ema")
    return c, info


def stash_layout(layer: Layer):
    """(layout, tile) of the stash layer_gram(keep_stash=KEEP_FAST) leaves for this layer."""
    layout, tile = ctypes.c_int(0), ctypes.c_int32(0)
    _check(load().isopo_stash_layout_of(layer.ref(), ctypes.byref(layout), ctypes.byref(tile)), "isopo_stash_layout_of")
    return layout.value, tile.value


def weighted_grad(layer: Layer, c: Optional[torch.Tensor], stash: Optional[torch.Tensor] = None, beta: float = 0.0,
                  dW: Optional[torch.Tensor] = None, stream=None, layout: Optional[int] = None) -> torch.Tensor:
    """dW [d_out, d_in] fp32 = beta dW + sum_i c_i G_i (from the stash if given,
    else by contracting X and Delta again).  `layout`: the kept stash's layout, if not row-major."""
    if dW is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs an existing dW")
        dW = torch.empty((layer.d_out, layer.d_in), dtype=torch.float32, device=layer.device)
    if layout is not None:
        _check(load().isopo_weighted_grad_stash(layer.ref(), _ptr(c), _ptr(stash), int(layout), float(beta),
                                                dW.data_ptr(), _stream(stream)), "isopo_weighted_grad_stash")
        return dW
    _check(load().isopo_weighted_grad(layer.ref(), _ptr(c), _ptr(stash), float(beta), dW.data_ptr(),
                                      _stream(stream)), "isopo_weighted_grad")
    return dW


def weighted_grad_stash_bf16(layer: Layer, c: torch.Tensor, stash: torch.Tensor, layout: int = 0, beta: float = 0.0,
                             dW: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """dW [d_out, d_in] bf16 = bf16(beta dW + sum_i c_i G_i) from a kept stash in the given layout."""
    if dW is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs an existing dW")
        dW = torch.empty((layer.d_out, layer.d_in), dtype=torch.bfloat16, device=layer.device)
    if dW.dtype != torch.bfloat16 or not dW.is_contiguous() or tuple(dW.shape) != (layer.d_out, layer.d_in):
        raise ValueError("dW must be a contiguous bf16 [d_out, d_in] tensor")
    _check(load().isopo_weighted_grad_stash_bf16(layer.ref(), _ptr(c), _ptr(stash), int(layout), float(beta),
                                                 dW.data_ptr(), _stream(stream)), "isopo_weighted_grad_stash_bf16")
    return dW


def fisher_samples(layer: Layer, sample_idx: torch.Tensor, A: torch.Tensor, lam: float = 0.0,
                   reg_mode: int = REG_ABSOLUTE, c: Optional[torch.Tensor] = None,
                   fisher_sq: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                   ema_state: Optional[torch.Tensor] = None, ema_decay: float = 0.9):
    """Coefficients of the non-interacting update from the token-position-sample Fisher estimate.
    sample_idx: int32 device tensor of token rows.  Returns (c, F^2)."""
    n_s = int(sample_idx.numel())
    if sample_idx.dtype != torch.int32 or not sample_idx.is_contiguous():
        raise ValueError("sample_idx must be a contiguous int32 tensor")
    if c is None:
        c = torch.empty(layer.n_seq, dtype=torch.float32, device=layer.device)
    if fisher_sq is None:
        fisher_sq = torch.empty(layer.n_seq, dtype=torch.float32, device=layer.device)
    if workspace is None:
        workspace = alloc_workspace(load().isopo_fisher_samples_workspace(layer.ref(), n_s), layer.device)
    _check(load().isopo_fisher_samples(layer.ref(), sample_idx.data_ptr(), n_s, A.data_ptr(), float(lam),
                                       int(reg_mode), _ptr(ema_state), float(ema_decay), c.data_ptr(),
                                       fisher_sq.data_ptr(), workspace.data_ptr(),
                                       workspace.numel(), _stream(stream)), "isopo_fisher_samples")
    return c, fisher_sq


def gram_norms(K: torch.Tensor, stream=None):
    """(F_norm^2, ||G||^2) per sequence from the Gram matrix: (1/m) sum_j K_ij^2 and K_ii."""
    m = K.shape[-1]
    f2 = torch.empty(m, dtype=torch.float32, device=K.device)
    g2 = torch.empty(m, dtype=torch.float32, device=K.device)
    _check(load().isopo_gram_norms(K.data_ptr(), m, f2.data_ptr(), g2.data_ptr(), _stream(stream)), "isopo_gram_norms")
    return f2, g2


def rescale(fisher_sq: torch.Tensor, grad_sq: torch.Tensor, A: torch.Tensor, p: float = -1.0, q: float = 0.0,
            r: float = 0.0, reg=(0.0, 0.0, 0.0), expectation=(None, None, None), c: Optional[torch.Tensor] = None,
            batch_means: Optional[torch.Tensor] = None, stream=None):
    """c_i = A_i reg2(F_i)^p reg2(||G_i||)^q reg2(F_i/||G_i||)^r.  grad_sq may be a 1-d tensor or a
    Gram matrix (its diagonal is read in place).  An expectation of None takes the batch mean."""
    m = int(fisher_sq.numel())
    if grad_sq.dim() == 2:
        stride = grad_sq.shape[-1] + 1
    else:
        stride = 1
    if not grad_sq.is_contiguous() or not fisher_sq.is_contiguous():
        raise ValueError("fisher_sq and grad_sq must be contiguous")
    prm = _RescaleParams(float(p), float(q), float(r), (ctypes.c_float * 3)(*[float(x) for x in reg]),
                         (ctypes.c_float * 3)(*[-1.0 if x is None else float(x) for x in expectation]))
    if c is None:
        c = torch.empty(m, dtype=torch.float32, device=fisher_sq.device)
    _check(load().isopo_rescale(fisher_sq.data_ptr(), grad_sq.data_ptr(), stride, m, A.data_ptr(), ctypes.byref(prm),
                                c.data_ptr(), _ptr(batch_means), _stream(stream)), "isopo_rescale")
    return c


def ntk_eigh(K: torch.Tensor, workspace: Optional[torch.Tensor] = None, stream=None):
    """D (ascending), U (eigenvectors as columns), info from the Gram matrix; fp64 on the device.
    K [m, m] or a batch [b, m, m] (one launch); outputs carry the same leading dimension."""
    if not K.is_contiguous():
        raise ValueError("K must be contiguous")
    m = K.shape[-1]
    batch = K.shape[0] if K.dim() == 3 else 1
    lead = (batch,) if K.dim() == 3 else ()
    D = torch.empty(lead + (m,), dtype=torch.float64, device=K.device)
    U = torch.empty(lead + (m, m), dtype=torch.float64, device=K.device)
    info = torch.zeros(batch, dtype=torch.int32, device=K.device)
    if workspace is None:
        workspace = alloc_workspace(load().isopo_ntk_eigh_workspace(m, batch), K.device)
    _check(load().isopo_ntk_eigh(K.data_ptr(), m, batch, D.data_ptr(), U.data_ptr(), info.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), _stream(stream)), "isopo_ntk_eigh")
    return D, U, info


def transform_eigh(D: torch.Tensor, U: torch.Tensor, A: torch.Tensor, lambdas, reg_mode: int = REG_ABSOLUTE,
                   ema_state: Optional[torch.Tensor] = None, ema_decay: float = 0.9,
                   c: Optional[torch.Tensor] = None, info: Optional[torch.Tensor] = None, stream=None):
    """c [n_lambda, m] = U ((U^T A) / (D + reg_l)); with a batch (D [b, m], U [b, m, m], A [b, m],
    ema_state [b, 2]) c is [b, n_lambda, m].  Returns (c, info)."""
    m = int(D.shape[-1])
    batch = D.shape[0] if D.dim() == 2 else 1
    lead = (batch,) if D.dim() == 2 else ()
    if A.numel() != batch * m:
        raise ValueError("A must hold one advantage per sequence and problem")
    lam = [float(x) for x in lambdas]
    if c is None:
        c = torch.empty(lead + (len(lam), m), dtype=torch.float32, device=D.device)
    if info is None:
        info = torch.zeros(batch, dtype=torch.int32, device=D.device)
    arr = (ctypes.c_float * max(len(lam), 1))(*lam)
    _check(load().isopo_transform_eigh(D.data_ptr(), U.data_ptr(), m, batch, A.data_ptr(), arr, len(lam),
                                       int(reg_mode), _ptr(ema_state), float(ema_decay), c.data_ptr(),
                                       info.data_ptr(), _stream(stream)), "isopo_transform_eigh")
    return c, info


def fisher_samples_group(layers, sample_idx: torch.Tensor, A: torch.Tensor, lam: float = 0.0,
                         reg_mode: int = REG_ABSOLUTE, c: Optional[torch.Tensor] = None,
                         fisher_sq: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                         ema_state: Optional[torch.Tensor] = None, ema_decay: float = 0.9):
    """fisher_samples for layers that share X (same tensor, same offsets): X is read once.
    Returns (c [n_layers, n_seq], F^2 [n_layers, n_seq])."""
    n = len(layers)
    first = layers[0]
    n_s = int(sample_idx.numel())
    if sample_idx.dtype != torch.int32 or not sample_idx.is_contiguous():
        raise ValueError("sample_idx must be a contiguous int32 tensor")
    if c is None:
        c = torch.empty((n, first.n_seq), dtype=torch.float32, device=first.device)
    if fisher_sq is None:
        fisher_sq = torch.empty((n, first.n_seq), dtype=torch.float32, device=first.device)
    if workspace is None:
        workspace = alloc_workspace(load().isopo_fisher_samples_group_workspace(first.ref(), n, n_s), first.device)
    arr = (ctypes.POINTER(_Layer) * n)(*[ctypes.pointer(l.c) for l in layers])
    _check(load().isopo_fisher_samples_group(arr, n, sample_idx.data_ptr(), n_s, A.data_ptr(), float(lam), int(reg_mode),
                                             _ptr(ema_state), float(ema_decay), c.data_ptr(), fisher_sq.data_ptr(),
                                             workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "isopo_fisher_samples_group")
    return c, fisher_sq


def fisher_samples_block(groups, sample_idx: torch.Tensor, A: torch.Tensor, lam: float = 0.0,
                         reg_mode: int = REG_ABSOLUTE, c: Optional[torch.Tensor] = None,
                         fisher_sq: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                         ema_state: Optional[torch.Tensor] = None, ema_decay: float = 0.9):
    """fisher_samples_group for several groups of one microbatch in one launch (`groups`: a list of lists of
    layers, each inner list sharing its X).  Returns (c, F^2), both [total layers, n_seq] in the groups' order."""
    layers = [l for g in groups for l in g]
    n, first = len(layers), layers[0]
    n_s = int(sample_idx.numel())
    if sample_idx.dtype != torch.int32 or not sample_idx.is_contiguous():
        raise ValueError("sample_idx must be a contiguous int32 tensor")
    if c is None:
        c = torch.empty((n, first.n_seq), dtype=torch.float32, device=first.device)
    if fisher_sq is None:
        fisher_sq = torch.empty((n, first.n_seq), dtype=torch.float32, device=first.device)
    if workspace is None:
        workspace = alloc_workspace(load().isopo_fisher_samples_block_workspace(first.ref(), n, n_s), first.device)
    arr = (ctypes.POINTER(_Layer) * n)(*[ctypes.pointer(l.c) for l in layers])
    sizes = (ctypes.c_int32 * len(groups))(*[len(g) for g in groups])
    _check(load().isopo_fisher_samples_block(arr, sizes, len(groups), sample_idx.data_ptr(), n_s, A.data_ptr(), float(lam),
                                             int(reg_mode), _ptr(ema_state), float(ema_decay), c.data_ptr(),
                                             fisher_sq.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "isopo_fisher_samples_block")
    return c, fisher_sq


def scale_rows(src: torch.Tensor, layer: Layer, c: torch.Tensor, dst: Optional[torch.Tensor] = None,
               stream=None) -> torch.Tensor:
    """dst[t, :] = c[seq(t)] * src[t, :] for src = X or Delta of `layer`."""
    if dst is None:
        dst = torch.empty_like(src)
    dtype = BF16 if src.dtype == torch.bfloat16 else F32
    _check(load().isopo_scale_rows(src.data_ptr(), dtype, src.shape[0], src.shape[1], _ptr(layer.off_dev),
                                   layer.n_seq, c.data_ptr(), dst.data_ptr(), _stream(stream)), "isopo_scale_rows")
    return dst


def weighted_grad_prescaled(layer: Layer, c: torch.Tensor, scratch: Optional[torch.Tensor] = None, beta: float = 0.0,
                            dW: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """dW = beta dW + Delta^T diag(c_tok) X without a stash: the narrower of X and Delta is scaled
    into `scratch`, then the unweighted contraction runs on it (one ABI call)."""
    need = int(load().isopo_weighted_grad_scratch(layer.ref()))
    if scratch is None:
        scratch = alloc_workspace(need, layer.device)
    if dW is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs an existing dW")
        dW = torch.empty((layer.d_out, layer.d_in), dtype=torch.float32, device=layer.device)
    _check(load().isopo_weighted_grad_prescaled(layer.ref(), c.data_ptr(), float(beta), dW.data_ptr(),
                                                scratch.data_ptr(), scratch.numel() * scratch.element_size(),
                                                _stream(stream)), "isopo_weighted_grad_prescaled")
    return dW


PROBE_THREADS = 256 * 256


def probe_mfma_loop(shape: int, operands: torch.Tensor, sink: torch.Tensor, iters: int, stream=None) -> None:
    """Diagnostic: `iters` trips of nothing but bf16 MFMAs of the given shape (32 or 16) on register operands."""
    if operands.numel() * operands.element_size() < PROBE_THREADS * 256 or sink.numel() < PROBE_THREADS:
        raise ValueError("operands / sink too small for the probe")
    _check(load().isopo_probe_mfma_loop(int(shape), operands.data_ptr(), sink.data_ptr(), int(iters), _stream(stream)),
           "isopo_probe_mfma_loop")


def probe_lds_dma(buf: torch.Tensor, waves: int, stages: int, workgroups: int, iters: int, sink: torch.Tensor,
                  stream=None) -> None:
    """Diagnostic: `workgroups` workgroups of `waves` waves keep a ring of `stages` 32 KiB LDS stages filled from
    `buf` by DMA loads for `iters` stages each (workgroups * iters * 32768 bytes in all)."""
    if sink.dtype != torch.float32 or sink.numel() < workgroups:
        raise ValueError("sink must hold one float per workgroup")
    _check(load().isopo_probe_lds_dma(buf.data_ptr(), buf.numel() * buf.element_size(), int(waves), int(stages),
                                      int(workgroups), int(iters), sink.data_ptr(), _stream(stream)), "isopo_probe_lds_dma")


def probe_contraction_waves(layer: Layer, waves: int, dW: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Diagnostic: dW = Delta^T X by the 256x256-tile contraction with 4 (the library's own launch) or 8 waves
    per workgroup."""
    if dW is None:
        dW = torch.empty((layer.d_out, layer.d_in), dtype=torch.float32, device=layer.device)
    _check(load().isopo_probe_contraction_waves(layer.ref(), int(waves), dW.data_ptr(), _stream(stream)),
           "isopo_probe_contraction_waves")
    return dW


def layer_step(layer: Layer, A: torch.Tensor, variant="interacting", lam: float = 0.0,
               reg_mode: int = REG_ABSOLUTE, path="auto", beta: float = 0.0, dW: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, stream=None) -> dict:
    """The three calls chained on one stream with no host synchronisation.  The returned workspace holds
    the stash in layout `stash_layout` (None: no stash was kept)."""
    chosen, full, _ = gram_plan(layer, path)
    if workspace is None:
        workspace = alloc_workspace(full, layer.device)
    keep = chosen == "materialised" and workspace.numel() >= full
    K, workspace = layer_gram(layer, path, workspace=workspace, keep_stash=KEEP_FAST if keep else 0, stream=stream)
    c, info = transform(K, A, variant, lam, reg_mode, stream=stream)
    layout = stash_layout(layer)[0] if keep else None
    if keep:
        dW = weighted_grad(layer, c, workspace, beta, dW, stream=stream, layout=layout)
    else:
        dW = weighted_grad(layer, c, None, beta, dW, stream=stream)
    return {"K": K, "c": c, "info": info, "dW": dW, "path": chosen, "workspace": workspace, "stash_layout": layout}
