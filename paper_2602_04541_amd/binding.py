"""Thin ctypes binding of liblychee.so: argument marshalling only.

Function names and argument order follow include/lychee.h.  Tensors are torch tensors used
purely as device-memory handles (`data_ptr()`); the stream is torch's current HIP stream
unless one is given.  If the shared library is missing the import of this module fails
loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblychee.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, EARENA = 0, -1, -2, -3, -4, -5
KERNEL_STREAM, KERNEL_GATHER, KERNEL_THRESHOLD, KERNEL_SELECT, KERNEL_COMBINE = 0, 1, 2, 3, 4
N_KERNEL_CLASSES = 5
OPT_DEFAULTS = 0
OPT_SELECT_LEAD = 10
STATIC_SCRATCH_BYTES = 32 << 20
OPT_WG_PER_CU, OPT_STEP_MODE, OPT_GATHER_BLOCK, OPT_N_WG, OPT_TAIL_PERMILLE, OPT_SELECT_MARGIN = 1, 2, 6, 7, 8, 9
STEP_PHASED, STEP_LAYERWISE = 1, 0
RULE_THRESHOLD, RULE_TOP_P = 1, 2

EXPORTS = [
    "lychee_create", "lychee_destroy", "lychee_check_shape", "lychee_workspace_bytes",
    "lychee_step_workspace_bytes",
    "lychee_decode_attn", "lychee_decode_attn_static", "lychee_decode_attn_deferred", "lychee_select_flush",
    "lychee_dense_decode_attn", "lychee_decode_step",
    "lychee_dense_decode_step", "lychee_decode_step_append", "lychee_append_kv", "lychee_select_stats",
    "lychee_wait_timeouts",
    "lychee_validate_idx", "lychee_set_option", "lychee_timing_enable",
    "lychee_timing_read", "lychee_probe_read", "lychee_probe_copy", "lychee_strerror",
]


class Shape(ctypes.Structure):
    """Mirror of `lychee_shape`."""
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("max_len", ctypes.c_int32), ("k", ctypes.c_int32),
                ("kv_stride_batch", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
                ("kv_stride_tok", ctypes.c_int64), ("keep_ppm", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("prob_rule", ctypes.c_int32),
                ("prob_param", ctypes.c_float)]


class LycheeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("liblychee.so is not built (run `python -m paper_2602_04541_amd.build` "
                          "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    shp = ctypes.POINTER(Shape)
    lib.lychee_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.lychee_destroy.argtypes = [vp]
    lib.lychee_check_shape.argtypes = [shp, vp, ctypes.c_int]
    lib.lychee_workspace_bytes.argtypes = [shp]
    lib.lychee_workspace_bytes.restype = sz
    lib.lychee_step_workspace_bytes.argtypes = [shp, i32]
    lib.lychee_step_workspace_bytes.restype = sz
    lib.lychee_decode_attn.argtypes = [vp, shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lychee_decode_attn_deferred.argtypes = lib.lychee_decode_attn.argtypes
    lib.lychee_decode_attn_static.argtypes = [vp, shp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.lychee_select_flush.argtypes = [vp, vp]
    lib.lychee_dense_decode_attn.argtypes = [vp, shp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lychee_decode_step.argtypes = [vp, shp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lychee_dense_decode_step.argtypes = [vp, shp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lychee_decode_step_append.argtypes = [vp, shp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.lychee_append_kv.argtypes = [vp, shp, vp, vp, vp, vp, vp, vp]
    lib.lychee_select_stats.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), vp]
    lib.lychee_wait_timeouts.argtypes = [vp, ctypes.POINTER(i64), vp]
    lib.lychee_validate_idx.argtypes = [vp, shp, vp, vp, ctypes.POINTER(i64), vp]
    lib.lychee_set_option.argtypes = [vp, i32, i32]
    lib.lychee_timing_enable.argtypes = [vp, ctypes.c_int]
    lib.lychee_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    lib.lychee_probe_read.argtypes = [vp, vp, sz, vp, vp]
    lib.lychee_probe_copy.argtypes = [vp, vp, vp, sz, vp]
    lib.lychee_strerror.argtypes = [ctypes.c_int]
    lib.lychee_strerror.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("lychee_workspace_bytes", "lychee_step_workspace_bytes", "lychee_strerror"):
            getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def strerror(code: int) -> str:
    return _lib.lychee_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != OK:
        raise LycheeError(code, where)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr()
    return int(t)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def make_shape(batch: int, n_q_heads: int, n_kv_heads: int, max_len: int, k: int,
               kv: Optional[torch.Tensor] = None, head_dim: int = 128,
               strides: Optional[Sequence[int]] = None, keep_ppm: int = 0,
               block_size: int = 0, prob_rule: int = 0, prob_param: float = 0.0) -> Shape:
    """A `lychee_shape`; KV strides (elements) come from a [B,H_kv,L_cap,128] tensor or `strides`."""
    if strides is None:
        if kv is not None:
            strides = (kv.stride(0), kv.stride(1), kv.stride(2))
        else:
            strides = (n_kv_heads * max_len * head_dim, max_len * head_dim, head_dim)
    return Shape(batch, n_q_heads, n_kv_heads, head_dim, max_len, k, *[int(s) for s in strides],
                 int(keep_ppm), int(block_size), int(prob_rule), float(prob_param))


def check_shape(shape: Shape, head_type_mask: Optional[np.ndarray] = None,
                has_idx_in: bool = True) -> int:
    """lychee_check_shape: returns the status code (pure host)."""
    m = None
    if head_type_mask is not None:
        m = np.ascontiguousarray(head_type_mask, dtype=np.uint8)
    return _lib.lychee_check_shape(ctypes.byref(shape), None if m is None else m.ctypes.data,
                                   int(has_idx_in))


def workspace_bytes(shape: Shape) -> int:
    return int(_lib.lychee_workspace_bytes(ctypes.byref(shape)))


def step_workspace_bytes(shape: Shape, n_layers: int) -> int:
    return int(_lib.lychee_step_workspace_bytes(ctypes.byref(shape), n_layers))


class Context:
    """Owner of a `lychee_ctx*`."""

    def __init__(self, device: int = 0):
        h = ctypes.c_void_p()
        _check(_lib.lychee_create(ctypes.byref(h), device), "lychee_create")
        self._h = h
        self.device = device

    def close(self) -> None:
        if self._h:
            _lib.lychee_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the path -----------------------------------------------------------------------
    def decode_attn(self, shape: Shape, q, k_cache, v_cache, head_type_mask: np.ndarray, idx_in,
                    out, idx_out, lengths, workspace, stream=None) -> None:
        mask = np.ascontiguousarray(head_type_mask, dtype=np.uint8)
        _check(_lib.lychee_decode_attn(self._h, ctypes.byref(shape), _ptr(q), _ptr(k_cache),
                                       _ptr(v_cache), mask.ctypes.data, _ptr(idx_in), _ptr(out),
                                       _ptr(idx_out), _ptr(lengths), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _stream(stream)), "lychee_decode_attn")

    def decode_attn_static(self, shape: Shape, q, k_cache, v_cache, head_type_mask: np.ndarray, idx_in,
                           out, idx_out, lengths, stream=None) -> None:
        """lychee_decode_attn on the library's own static scratch: no workspace, no allocation."""
        mask = np.ascontiguousarray(head_type_mask, dtype=np.uint8)
        _check(_lib.lychee_decode_attn_static(self._h, ctypes.byref(shape), _ptr(q), _ptr(k_cache),
                                              _ptr(v_cache), mask.ctypes.data, _ptr(idx_in), _ptr(out),
                                              _ptr(idx_out), _ptr(lengths), _stream(stream)),
               "lychee_decode_attn_static")

    def decode_attn_deferred(self, shape: Shape, q, k_cache, v_cache, head_type_mask: np.ndarray,
                             idx_in, out, idx_out, lengths, workspace, stream=None) -> None:
        """The layer call that leaves its selection for the next such call (or select_flush);
        `workspace` holds two layers (alloc_workspace(..., n_layers=2))."""
        mask = np.ascontiguousarray(head_type_mask, dtype=np.uint8)
        _check(_lib.lychee_decode_attn_deferred(self._h, ctypes.byref(shape), _ptr(q), _ptr(k_cache),
                                                _ptr(v_cache), mask.ctypes.data, _ptr(idx_in), _ptr(out),
                                                _ptr(idx_out), _ptr(lengths), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(),
                                                _stream(stream)), "lychee_decode_attn_deferred")

    def select_flush(self, stream=None) -> None:
        _check(_lib.lychee_select_flush(self._h, _stream(stream)), "lychee_select_flush")

    def dense_decode_attn(self, shape: Shape, q, k_cache, v_cache, out, lengths, workspace,
                          stream=None) -> None:
        _check(_lib.lychee_dense_decode_attn(self._h, ctypes.byref(shape), _ptr(q), _ptr(k_cache),
                                             _ptr(v_cache), _ptr(out), _ptr(lengths),
                                             _ptr(workspace),
                                             workspace.numel() * workspace.element_size(),
                                             _stream(stream)), "lychee_dense_decode_attn")

    def decode_step(self, shape: Shape, q: Sequence, k_cache: Sequence, v_cache: Sequence,
                    head_type_masks: np.ndarray, idx_in, out: Sequence, idx_out, lengths,
                    workspace, stream=None) -> None:
        n = len(q)
        arr = ctypes.c_void_p * n
        masks = np.ascontiguousarray(head_type_masks, dtype=np.uint8)
        assert masks.shape == (n, shape.n_q_heads)
        _check(_lib.lychee_decode_step(self._h, ctypes.byref(shape), n,
                                       arr(*[_ptr(t) for t in q]), arr(*[_ptr(t) for t in k_cache]),
                                       arr(*[_ptr(t) for t in v_cache]), masks.ctypes.data,
                                       _ptr(idx_in), arr(*[_ptr(t) for t in out]), _ptr(idx_out),
                                       _ptr(lengths), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(),
                                       _stream(stream)), "lychee_decode_step")

    def decode_step_append(self, shape: Shape, q: Sequence, k_new: Sequence, v_new: Sequence,
                           k_cache: Sequence, v_cache: Sequence, head_type_masks: np.ndarray, idx_in,
                           out: Sequence, idx_out, lengths, workspace, stream=None) -> None:
        n = len(q)
        arr = ctypes.c_void_p * n
        masks = np.ascontiguousarray(head_type_masks, dtype=np.uint8)
        assert masks.shape == (n, shape.n_q_heads)
        _check(_lib.lychee_decode_step_append(
            self._h, ctypes.byref(shape), n, arr(*[_ptr(t) for t in q]), arr(*[_ptr(t) for t in k_new]),
            arr(*[_ptr(t) for t in v_new]), arr(*[_ptr(t) for t in k_cache]),
            arr(*[_ptr(t) for t in v_cache]), masks.ctypes.data, _ptr(idx_in),
            arr(*[_ptr(t) for t in out]), _ptr(idx_out), _ptr(lengths), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)), "lychee_decode_step_append")

    def append_kv(self, shape: Shape, k_new, v_new, k_cache, v_cache, lengths, stream=None) -> None:
        _check(_lib.lychee_append_kv(self._h, ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                     _ptr(v_cache), _ptr(lengths), _stream(stream)), "lychee_append_kv")

    def dense_decode_step(self, shape: Shape, q: Sequence, k_cache: Sequence, v_cache: Sequence,
                          out: Sequence, lengths, workspace, stream=None) -> None:
        n = len(q)
        arr = ctypes.c_void_p * n
        _check(_lib.lychee_dense_decode_step(self._h, ctypes.byref(shape), n,
                                             arr(*[_ptr(t) for t in q]), arr(*[_ptr(t) for t in k_cache]),
                                             arr(*[_ptr(t) for t in v_cache]), arr(*[_ptr(t) for t in out]),
                                             _ptr(lengths), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(),
                                             _stream(stream)), "lychee_dense_decode_step")

    # -- helpers ------------------------------------------------------------------------
    def select_stats(self, stream=None):
        """(too_few, too_many): score rows the select ranked whole since the context was created."""
        a, b = ctypes.c_int64(-1), ctypes.c_int64(-1)
        _check(_lib.lychee_select_stats(self._h, ctypes.byref(a), ctypes.byref(b), _stream(stream)),
               "lychee_select_stats")
        return int(a.value), int(b.value)

    def wait_timeouts(self, stream=None) -> int:
        """Bounded waits inside layer launches that gave up since the context was created."""
        n = ctypes.c_int64(-1)
        _check(_lib.lychee_wait_timeouts(self._h, ctypes.byref(n), _stream(stream)), "lychee_wait_timeouts")
        return int(n.value)

    def validate_idx(self, shape: Shape, idx, lengths, stream=None) -> int:
        n_bad = ctypes.c_int64(-1)
        _check(_lib.lychee_validate_idx(self._h, ctypes.byref(shape), _ptr(idx), _ptr(lengths),
                                        ctypes.byref(n_bad), _stream(stream)), "lychee_validate_idx")
        return int(n_bad.value)

    def set_option(self, option: int, value: int) -> None:
        _check(_lib.lychee_set_option(self._h, option, value), "lychee_set_option")

    def timing_enable(self, on: bool) -> None:
        _check(_lib.lychee_timing_enable(self._h, int(on)), "lychee_timing_enable")

    def timing_read(self):
        ms = (ctypes.c_float * N_KERNEL_CLASSES)()
        n = (ctypes.c_int32 * N_KERNEL_CLASSES)()
        _check(_lib.lychee_timing_read(self._h, ms, n), "lychee_timing_read")
        return list(ms), list(n)

    def probe_read(self, src, nbytes: int, sink, stream=None) -> None:
        _check(_lib.lychee_probe_read(self._h, _ptr(src), nbytes, _ptr(sink), _stream(stream)),
               "lychee_probe_read")

    def probe_copy(self, dst, src, nbytes: int, stream=None) -> None:
        _check(_lib.lychee_probe_copy(self._h, _ptr(dst), _ptr(src), nbytes, _stream(stream)),
               "lychee_probe_copy")


def alloc_workspace(shape: Shape, device="cuda", n_layers: int = 1) -> torch.Tensor:
    """A device buffer of lychee_step_workspace_bytes(shape, n_layers) bytes (torch only
    allocates it); n_layers = 1 is what the single-layer calls need."""
    n = step_workspace_bytes(shape, n_layers)
    if n == 0:
        raise LycheeError(_lib.lychee_check_shape(ctypes.byref(shape), None, 1), "lychee_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)
