"""Seeded synthetic inputs for the decode-step hybrid-head attention path.

This module only *draws inputs*: query vectors, a bf16 KV cache with planted
query-aligned key rows, head-type masks and ragged lengths.  It holds none of the
method's arithmetic (no scores, no softmax, no selection) and is the one module the
HIP path's tests/bench and the CPU oracle's tests both read, so that both sides see
the same bf16 bits.

The shapes stand in for the workloads the paper runs (8B-class GQA models, 32 query /
8 KV heads, head dim 128, contexts 4K..128K, token budgets 256..4096, batch 1..8;
Sec. 4.1, Sec. 4.3, App. E.4); no benchmark item, prompt or trained weight is used.

Recipe (every draw is seeded):
  * Q, K, V ~ N(0,1) drawn in fp32 and rounded (RNE) to bf16.
  * per (sequence, KV head) P distinct "planted" positions; the key row there becomes
        a * sqrt(d) * q_hat + noise,   q_hat = q*/||q*||,
    q* = query of the group's lowest-index retrieval head (else the group's first
    head), noise = the N(0,1) row already drawn.  Its scaled logit under q* is about
    a*||q*|| (~34 for a = 3) against an N(0,1) background, so top-k is non-trivial.
  * heavy tail ("zipf"): the rank-r planted row uses a_r = (3*sqrt(d) - alpha*ln r)/||q*||
    so that its attention mass falls off like r**(-alpha).
  * rows at and beyond a sequence's length (ragged batches) hold strongly aligned
    "poison" keys: reading them would change every result.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

HEAD_DIM = 128
BASE_SEED = 20260204 * 10


@dataclass(frozen=True)
class Workload:
    """Shape and recipe parameters of one synthetic configuration."""

    name: str
    config_id: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    max_len: int
    k: int
    n_layers: int = 1
    n_retrieval: int = 0          # retrieval query heads per layer (0 -> explicit list)
    retrieval_heads: tuple = ()   # explicit list, used when n_retrieval == 0
    planted: int = 0
    zipf_alpha: float = 0.0       # > 0: heavy-tailed planted strengths
    len_lo: int = 0               # ragged lengths drawn in [len_lo, len_hi]
    len_hi: int = 0
    first_layer_all_retrieval: bool = False

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


WORKLOADS: Dict[str, Workload] = {
    # single layer, 8 q / 2 kv heads, context 4096, heads 0 and 4 retrieval, k = 256
    "c1": Workload("c1", 1, 1, 8, 2, 4096, 256, retrieval_heads=(0, 4), planted=32),
    # Llama-3-8B-shaped layer, context 32768, one retrieval head per pair of KV groups
    "c2": Workload("c2", 2, 1, 32, 8, 32768, 2048, n_retrieval=4, planted=512),
    # Qwen3-8B-shaped decode step: 36 layers at 128K, 3 retrieval heads per layer
    "c3": Workload("c3", 3, 1, 32, 8, 131072, 4096, n_layers=36, n_retrieval=3,
                   planted=1024, zipf_alpha=1.2, first_layer_all_retrieval=True),
    # batched ragged decode
    "c4": Workload("c4", 4, 8, 32, 8, 98304, 2048, n_retrieval=4, planted=256,
                   len_lo=16384, len_hi=98304),
    # single 128K layer used by the k / retrieval-fraction / tie sweep
    "c5": Workload("c5", 5, 1, 32, 8, 131072, 4096, n_retrieval=4, planted=1024,
                   zipf_alpha=1.2),
}


def kernel_study(batch: int, context: int, sparse_groups: int) -> Workload:
    """The shape of the paper's kernel-level study (Sec. 4.3.2): one layer, 8 KV heads (4 query
    heads each), `sparse_groups` of the 8 KV groups entirely sparse with 90 % block sparsity
    (block size 64: a tenth of the blocks is attended), the other groups entirely dense.
    `k` counts blocks.  Only the shape is the paper's; values and block choices are synthetic."""
    n_blocks = (context + 63) // 64
    heads = tuple(h for h in range(32) if h // 4 < 8 - sparse_groups)
    return Workload("ks_b%d_L%d_s%d" % (batch, context, sparse_groups), 6, batch, 32, 8, context,
                    max(1, n_blocks // 10), retrieval_heads=heads, planted=0)


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (smaller test variants)."""
    d = dict(w.__dict__)
    d.update(changes)
    return Workload(**d)


def _np_rng(w: Workload, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=BASE_SEED + w.config_id,
                                                counter=[layer, stream, 0, 0]))


def head_type_mask(w: Workload, layer: int = 0) -> np.ndarray:
    """uint8 [n_q_heads]: 1 = retrieval head, 0 = sparse head, for one layer."""
    m = np.zeros(w.n_q_heads, dtype=np.uint8)
    if w.first_layer_all_retrieval and layer == 0:
        m[:] = 1
        return m
    if w.n_retrieval == 0:
        m[list(w.retrieval_heads)] = 1
        return m
    rng = _np_rng(w, layer, 1)
    if w.n_retrieval * 2 * w.group == w.n_q_heads:
        # one retrieval head inside each pair of adjacent KV groups
        span = 2 * w.group
        for p in range(w.n_retrieval):
            m[p * span + int(rng.integers(0, span))] = 1
    else:
        m[rng.choice(w.n_q_heads, size=w.n_retrieval, replace=False)] = 1
    return m


def lengths(w: Workload) -> np.ndarray:
    """int32 [batch] context lengths (the current token included)."""
    if w.len_hi > 0:
        rng = _np_rng(w, 0, 2)
        out = rng.integers(w.len_lo, w.len_hi + 1, size=w.batch).astype(np.int32)
        return np.minimum(out, w.max_len).astype(np.int32)
    return np.full(w.batch, w.max_len, dtype=np.int32)


@dataclass
class LayerInputs:
    """One layer's inputs. Tensors live on `device`; small arrays on the host."""

    workload: Workload
    layer: int
    q: torch.Tensor            # bf16 [B, Hq, 128]
    k_cache: torch.Tensor      # bf16 [B, Hkv, L_cap, 128]
    v_cache: torch.Tensor      # bf16 [B, Hkv, L_cap, 128]
    mask: np.ndarray           # uint8 [Hq]
    lengths: np.ndarray        # int32 [B]
    planted_pos: np.ndarray    # int64 [B, Hkv, P]
    extra: dict = field(default_factory=dict)


def _randn_bf16(shape, gen: torch.Generator, device) -> torch.Tensor:
    """N(0,1) in fp32 rounded to bf16, drawn slab by slab to bound the fp32 temporary."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    n = flat.numel()
    step = 1 << 26
    for s in range(0, n, step):
        e = min(n, s + step)
        flat[s:e] = torch.randn(e - s, generator=gen, device=device,
                                dtype=torch.float32).to(torch.bfloat16)
    return out


def make_layer(w: Workload, layer: int = 0, device="cpu",
               mask: Optional[np.ndarray] = None,
               lens: Optional[np.ndarray] = None,
               l_cap: Optional[int] = None) -> LayerInputs:
    """Draw one layer's q / K / V, plant the aligned key rows and return everything."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(BASE_SEED + w.config_id + 1000 * layer)
    if mask is None:
        mask = head_type_mask(w, layer)
    if lens is None:
        lens = lengths(w)
    lens = np.asarray(lens, dtype=np.int32)
    if l_cap is None:
        l_cap = int(w.max_len)
    B, Hq, Hkv, G, d = w.batch, w.n_q_heads, w.n_kv_heads, w.group, HEAD_DIM

    q = _randn_bf16((B, Hq, d), gen, device)
    k_cache = _randn_bf16((B, Hkv, l_cap, d), gen, device)
    v_cache = _randn_bf16((B, Hkv, l_cap, d), gen, device)

    P = int(w.planted)
    planted = np.zeros((B, Hkv, P), dtype=np.int64)
    rng = _np_rng(w, layer, 3)
    root_d = math.sqrt(d)
    for b in range(B):
        L = int(lens[b])
        for g in range(Hkv):
            heads = [h for h in range(g * G, (g + 1) * G) if mask[h]]
            h_star = heads[0] if heads else g * G
            qs = q[b, h_star].float()
            qn = float(qs.norm())
            q_hat = qs / qn
            if P > 0:
                pp = min(P, L)
                pos = rng.choice(L, size=pp, replace=False).astype(np.int64)
                planted[b, g, :pp] = pos
                planted[b, g, pp:] = pos[0] if pp else 0
                if w.zipf_alpha > 0:
                    r = torch.arange(1, pp + 1, dtype=torch.float32, device=device)
                    a = (3.0 * root_d - w.zipf_alpha * torch.log(r)) / qn
                else:
                    a = torch.full((pp,), 3.0, dtype=torch.float32, device=device)
                pos_t = torch.from_numpy(pos).to(device)
                rows = k_cache[b, g, pos_t].float() + (a * root_d)[:, None] * q_hat[None, :]
                k_cache[b, g, pos_t] = rows.to(torch.bfloat16)
            if L < l_cap:
                # poison: strongly aligned keys past the end of the sequence
                n_poison = min(64, l_cap - L)
                k_cache[b, g, L:L + n_poison] = (5.0 * root_d * q_hat).to(torch.bfloat16)
                v_cache[b, g, L:L + n_poison] = 100.0
    return LayerInputs(w, layer, q, k_cache, v_cache, mask.astype(np.uint8), lens, planted)


def plant_ties(inp: LayerInputs, n_copies: int, sources: np.ndarray,
               stream: int = 7) -> np.ndarray:
    """Overwrite `n_copies` key rows per (b, g) with copies of the rows at `sources`
    ([B, Hkv, n_src] positions), leaving V untouched so that a wrong tie-break changes
    the output.  Returns the overwritten positions [B, Hkv, n_copies]."""
    w = inp.workload
    rng = _np_rng(w, inp.layer, stream)
    B, Hkv = w.batch, w.n_kv_heads
    dst_all = np.zeros((B, Hkv, n_copies), dtype=np.int64)
    for b in range(B):
        L = int(inp.lengths[b])
        for g in range(Hkv):
            src = np.asarray(sources[b, g], dtype=np.int64)
            free = np.setdiff1d(np.arange(L, dtype=np.int64), src)
            dst = rng.choice(free, size=min(n_copies, free.size), replace=False)
            which = src[rng.integers(0, src.size, size=dst.size)]
            dev = inp.k_cache.device
            inp.k_cache[b, g, torch.from_numpy(dst).to(dev)] = \
                inp.k_cache[b, g, torch.from_numpy(which).to(dev)]
            dst_all[b, g, :dst.size] = dst
            dst_all[b, g, dst.size:] = dst[0]
    return dst_all


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """The raw bf16 bit patterns of a tensor as a host uint16 array (same shape)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def algorithmic_bytes(w: Workload, mask: np.ndarray, lens: np.ndarray, score_bytes: int = 0) -> int:
    """HBM bytes one hybrid layer call must move: K+V rows streamed for groups holding a
    retrieval head, K+V rows gathered for groups holding a sparse head, the index sets and
    q / out.  `score_bytes` adds that many bytes per streamed row for an implementation that
    materialises the selection scores (8 = fp32 written once and read once); the library
    does not, so its figures use 0."""
    G, Hkv, d = w.group, w.n_kv_heads, HEAD_DIM
    row = 2 * d * 2
    n_r = sum(1 for g in range(Hkv) if mask[g * G:(g + 1) * G].any())
    n_s = sum(1 for g in range(Hkv) if (mask[g * G:(g + 1) * G] == 0).any())
    total = 0
    for L in lens:
        L = int(L)
        total += n_r * L * row + n_s * min(w.k, L) * row + n_r * L * score_bytes
        total += Hkv * w.k * 4 * 2
    total += w.batch * w.n_q_heads * d * 2 * 2
    return total


def dense_bytes(w: Workload, lens: np.ndarray) -> int:
    """HBM bytes of dense decode attention on the same shape (all K+V rows, q, out)."""
    row = 2 * HEAD_DIM * 2
    return int(sum(int(L) for L in lens)) * w.n_kv_heads * row \
        + w.batch * w.n_q_heads * HEAD_DIM * 2 * 2
