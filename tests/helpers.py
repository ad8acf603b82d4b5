"""Small shared test utilities (no method arithmetic beyond what each test states)."""
from __future__ import annotations

import numpy as np


def to_bf16_bits(x) -> np.ndarray:
    """bf16 bit patterns of values that bf16 represents exactly (asserted)."""
    a = np.asarray(x, dtype=np.float32)
    u = a.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value is not exactly representable in bf16"
    return (u >> 16).astype(np.uint16)


def round_to_bf16_bits(x) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    a = np.asarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    return r


def bits_to_f64(bits) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)


def index_sets_match(idx_a: np.ndarray, idx_ref: np.ndarray, sel_ref: np.ndarray, n: int,
                     rel: float = 1e-4):
    """Compare two index sets of one (sequence, KV head).

    Sets must be equal, except that a position may differ where the reference's
    selection score ties with the reference's n-th largest score within `rel`
    relative.  Returns (ok, n_different, message)."""
    a = np.asarray(idx_a)
    r = np.asarray(idx_ref)
    va, vr = a[a >= 0], r[r >= 0]
    if va.size != n or vr.size != n:
        return False, -1, "valid count %d / %d, expected %d" % (va.size, vr.size, n)
    if np.unique(va).size != va.size:
        return False, -1, "duplicate positions"
    if (va.max(initial=0) >= sel_ref.size):
        return False, -1, "position out of range"
    diff = np.setxor1d(va, vr)
    if diff.size == 0:
        return True, 0, ""
    tau = np.sort(sel_ref[vr])[0]           # the n-th largest reference score
    slack = rel * max(abs(tau), 1e-30)
    bad = diff[np.abs(sel_ref[diff] - tau) > slack]
    if bad.size:
        return False, diff.size, "positions %s differ away from a tie (tau=%r, scores %r)" % (
            bad[:8], tau, sel_ref[bad[:8]])
    return True, diff.size, ""
