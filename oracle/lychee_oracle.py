"""ctypes front end of the fp64 CPU oracle in lychee_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's
cpu-baseline leg; never by the product package.  It marshals numpy arrays and nothing
else; all arithmetic is in the C file.  The C file is compiled with gcc on first use
when no built library is present.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lychee_oracle.c")
_LIB = os.path.join(_HERE, "liblychee_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile lychee_oracle.c into a shared library next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        i32, i64 = ctypes.c_int32, ctypes.c_int64
        lib.lo_scores.argtypes = [u16p, u16p, i64, i32, i32, f64p]
        lib.lo_scores.restype = None
        lib.lo_scores_at.argtypes = [u16p, u16p, i64, i32p, i32, i32, f64p]
        lib.lo_scores_at.restype = None
        lib.lo_softmax_weights.argtypes = [f64p, i32p, i32, f64p]
        lib.lo_softmax_weights.restype = None
        lib.lo_weighted_values.argtypes = [f64p, i32p, i32, u16p, i64, i32, f64p]
        lib.lo_weighted_values.restype = None
        lib.lo_topk.argtypes = [f64p, i32, i32, i32p]
        lib.lo_topk.restype = None
        lib.lo_decode_attn.argtypes = [i32, i32, i32, i32, i32, i32, u16p, u16p, u16p, i64, i64,
                                       i64, u8p, i32p, i32p, f64p, i32p, f64p]
        lib.lo_decode_attn.restype = ctypes.c_int
        lib.lo_decode_attn_rule.argtypes = lib.lo_decode_attn.argtypes + [i32]
        lib.lo_decode_attn_rule.restype = ctypes.c_int
        lib.lo_decode_attn_block.argtypes = lib.lo_decode_attn.argtypes + [i32, i32, i32, ctypes.c_double]
        lib.lo_rule_count.argtypes = [f64p, i32, i32, ctypes.c_double]
        lib.lo_rule_count.restype = i32
        lib.lo_decode_attn_block.restype = ctypes.c_int
        lib.lo_append_kv.argtypes = [i32, i32, i32, u16p, u16p, u16p, u16p, i64, i64, i64, i32p]
        lib.lo_append_kv.restype = ctypes.c_int
        lib.lo_ratio_budget.argtypes = [i32, i32, i32]
        lib.lo_ratio_budget.restype = i32
        lib.lo_topk_n.argtypes = [f64p, i32, i32, i32, i32p]
        lib.lo_topk_n.restype = None
        lib.lo_num_threads.argtypes = []
        lib.lo_num_threads.restype = i32
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().lo_num_threads())


def scores(q_bits: np.ndarray, k_bits: np.ndarray) -> np.ndarray:
    """Scaled logits of one query against every row of a [L, d] key matrix (Eq. 1)."""
    q = _c(q_bits, np.uint16)
    K = _c(k_bits, np.uint16)
    L, d = K.shape
    s = np.empty(L, dtype=np.float64)
    _load().lo_scores(_ptr(q, ctypes.c_uint16), _ptr(K, ctypes.c_uint16), d, L, d,
                      _ptr(s, ctypes.c_double))
    return s


def softmax_weights(s: np.ndarray, pos: np.ndarray) -> np.ndarray:
    s = _c(s, np.float64)
    pos = _c(pos, np.int32)
    w = np.empty(pos.size, dtype=np.float64)
    _load().lo_softmax_weights(_ptr(s, ctypes.c_double), _ptr(pos, ctypes.c_int32), pos.size,
                               _ptr(w, ctypes.c_double))
    return w


def weighted_values(w: np.ndarray, pos: np.ndarray, v_bits: np.ndarray) -> np.ndarray:
    w = _c(w, np.float64)
    pos = _c(pos, np.int32)
    V = _c(v_bits, np.uint16)
    d = V.shape[1]
    o = np.empty(d, dtype=np.float64)
    _load().lo_weighted_values(_ptr(w, ctypes.c_double), _ptr(pos, ctypes.c_int32), pos.size,
                               _ptr(V, ctypes.c_uint16), d, d, _ptr(o, ctypes.c_double))
    return o


def topk(sel: np.ndarray, k: int) -> np.ndarray:
    """Eq. 2 by full sort: the min(k, L) best positions, ascending, padded with -1."""
    sel = _c(sel, np.float64)
    out = np.empty(k, dtype=np.int32)
    _load().lo_topk(_ptr(sel, ctypes.c_double), sel.size, k, _ptr(out, ctypes.c_int32))
    return out


def append_kv(k_new: np.ndarray, v_new: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray,
              lengths: np.ndarray) -> None:
    """Alg. 1's cache append, in place: k_new / v_new [B,Hkv,d] become row lengths[b]-1 of the
    caches k_bits / v_bits [B,Hkv,L_cap,d] (uint16 bf16 bit patterns, writable)."""
    kn, vn = _c(k_new, np.uint16), _c(v_new, np.uint16)
    assert k_bits.dtype == np.uint16 and v_bits.dtype == np.uint16 and k_bits.flags.writeable
    assert k_bits.strides == v_bits.strides
    B, Hkv, d = kn.shape
    sb, sh, st, sd = (x // 2 for x in k_bits.strides)
    assert sd == 1
    lengths = _c(lengths, np.int32)
    rc = _load().lo_append_kv(B, Hkv, d, _ptr(kn, ctypes.c_uint16), _ptr(vn, ctypes.c_uint16),
                              _ptr(k_bits, ctypes.c_uint16), _ptr(v_bits, ctypes.c_uint16), sb, sh, st,
                              _ptr(lengths, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle rejected its arguments (rc=%d)" % rc)


RULE_TOPK, RULE_THRESHOLD, RULE_TOP_P = 0, 1, 2


def rule_count(sel: np.ndarray, rule: int, param: float) -> int:
    """Positions the Threshold (rule 1) or Top-p (rule 2) rule keeps among these pooled logits,
    before the clamp to [1, min(k, L)]."""
    sel = _c(sel, np.float64)
    return int(_load().lo_rule_count(_ptr(sel, ctypes.c_double), sel.size, int(rule), float(param)))


def ratio_budget(L: int, k: int, keep_ppm: int) -> int:
    """Positions the Ratio rule (Sec. 4.4.1) keeps for a sequence of L rows: ceil(L * keep_ppm /
    10^6), at least 1, at most L and the set capacity k; keep_ppm = 0 gives min(k, L)."""
    return int(_load().lo_ratio_budget(int(L), int(k), int(keep_ppm)))


def decode_attn(q_bits: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray, mask: np.ndarray,
                k: int, idx_in: Optional[np.ndarray], lengths: np.ndarray,
                want_sel: bool = False, keep_ppm: int = 0, block: int = 1, rule: int = 0,
                rule_param: float = 0.0) -> Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]:
    """One layer of Alg. 1's per-head loop.  keep_ppm > 0: the Ratio rule of Sec. 4.4.1
    (ratio_budget() entries per sequence, in sets of capacity k) instead of the fixed budget.
    block > 1: the block-granular variant (App. C): set entries are block numbers, k counts
    blocks, a block is scored by its best token.  rule 1 / 2: the Threshold / Top-p rule of
    Sec. 4.4.1 with parameter rule_param, on the softmax of the pooled logits, capped at k.

    q_bits [B,Hq,d], k_bits / v_bits [B,Hkv,L_cap,d] (uint16 bf16 bit patterns, any
    strides numpy can express with a contiguous last axis), mask [Hq] uint8, idx_in
    [B,Hkv,k] int32 or None, lengths [B] int32.
    Returns (out fp64 [B,Hq,d], idx_out int32 [B,Hkv,k], sel fp64 [B,Hkv,L_cap] or None).
    """
    q = _c(q_bits, np.uint16)
    assert k_bits.dtype == np.uint16 and v_bits.dtype == np.uint16
    assert k_bits.shape == v_bits.shape and k_bits.strides == v_bits.strides
    B, Hq, d = q.shape
    _, Hkv, l_cap, _ = k_bits.shape
    sb, sh, st, sd = (x // 2 for x in k_bits.strides)
    assert sd == 1
    mask = _c(mask, np.uint8)
    lengths = _c(lengths, np.int32)
    if idx_in is not None:
        idx_in = _c(idx_in, np.int32)
        assert idx_in.shape == (B, Hkv, k)
    out = np.empty((B, Hq, d), dtype=np.float64)
    idx_out = np.empty((B, Hkv, k), dtype=np.int32)
    sel = np.empty((B, Hkv, l_cap), dtype=np.float64) if want_sel else None
    rc = _load().lo_decode_attn_block(B, Hq, Hkv, d, k, l_cap, _ptr(q, ctypes.c_uint16),
                                     _ptr(k_bits, ctypes.c_uint16), _ptr(v_bits, ctypes.c_uint16),
                                     sb, sh, st, _ptr(mask, ctypes.c_uint8),
                                     _ptr(idx_in, ctypes.c_int32), _ptr(lengths, ctypes.c_int32),
                                     _ptr(out, ctypes.c_double), _ptr(idx_out, ctypes.c_int32),
                                     _ptr(sel, ctypes.c_double), int(keep_ppm), int(block), int(rule),
                                     float(rule_param))
    if rc != 0:
        raise ValueError("oracle rejected its arguments (rc=%d)" % rc)
    return out, idx_out, sel


def dense_attn(q_bits, k_bits, v_bits, lengths) -> np.ndarray:
    """Dense decode attention (every head is Eq. 1 + o = A V): the all-retrieval case."""
    Hq = q_bits.shape[1]
    out, _, _ = decode_attn(q_bits, k_bits, v_bits, np.ones(Hq, np.uint8), 1, None, lengths)
    return out
