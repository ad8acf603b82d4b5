"""Shared plumbing of the GPU parity tests: upload, call the C ABI, download, compare with
the CPU oracle.  No attention arithmetic lives here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from oracle import lychee_oracle as lo
from paper_2602_04541_amd import workloads as wl
from tests.helpers import index_sets_match

ABS_TOL = 2e-2   # the stated bar for bf16 outputs: |gpu - ref| <= 2e-2 + 1e-2 * |ref|
REL_TOL = 1e-2
TIE_REL = 1e-4   # an index may differ only where the oracle's scores tie within 1e-4 relative


def binding():
    from paper_2602_04541_amd import binding as lb
    return lb


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def previous_layer_sets(inp: wl.LayerInputs, k: int, seed: int = 99, block: int = 1) -> np.ndarray:
    """Realistic inherited sets: the oracle's top-k of an all-retrieval previous layer with
    an independently drawn query on the same cache."""
    w = inp.workload
    g = torch.Generator()
    g.manual_seed(wl.BASE_SEED + 7919 * seed + w.config_id)
    q_prev = torch.randn(inp.q.shape, generator=g, dtype=torch.float32).to(torch.bfloat16)
    _, idx, _ = lo.decode_attn(wl.bf16_bits(q_prev), wl.bf16_bits(inp.k_cache),
                               wl.bf16_bits(inp.v_cache), np.ones(w.n_q_heads, np.uint8), k, None,
                               inp.lengths, block=block)
    return idx


class DeviceLayer:
    """Device copies of one layer's inputs plus output buffers."""

    def __init__(self, inp: wl.LayerInputs, k: int, idx_in: Optional[np.ndarray], device="cuda",
                 keep_ppm: int = 0, block: int = 1):
        lb = binding()
        w = inp.workload
        self.inp, self.k = inp, k
        self.q = inp.q.to(device)
        self.k_cache = inp.k_cache.to(device)
        self.v_cache = inp.v_cache.to(device)
        self.lengths = torch.from_numpy(inp.lengths.astype(np.int32)).to(device)
        self.idx_in = None if idx_in is None else torch.from_numpy(idx_in.astype(np.int32)).to(device)
        self.out = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=torch.bfloat16,
                              device=device)
        self.idx_out = torch.full((w.batch, w.n_kv_heads, k), -7, dtype=torch.int32, device=device)
        self.shape = lb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, self.k_cache.shape[2], k,
                                   kv=self.k_cache, keep_ppm=keep_ppm, block_size=block)
        self.workspace = lb.alloc_workspace(self.shape, device)
        # poison the workspace: results must not depend on what it held
        self.workspace.fill_(0xFF)


def run_hybrid(ctx, dl: DeviceLayer, mask: np.ndarray):
    ctx.decode_attn(dl.shape, dl.q, dl.k_cache, dl.v_cache, mask, dl.idx_in, dl.out, dl.idx_out,
                    dl.lengths, dl.workspace)
    torch.cuda.synchronize()
    return bf16_tensor_to_f64(dl.out), dl.idx_out.cpu().numpy()


def run_dense(ctx, dl: DeviceLayer):
    ctx.dense_decode_attn(dl.shape, dl.q, dl.k_cache, dl.v_cache, dl.out, dl.lengths, dl.workspace)
    torch.cuda.synchronize()
    return bf16_tensor_to_f64(dl.out)


def oracle_layer(inp: wl.LayerInputs, mask, k, idx_in, keep_ppm: int = 0, block: int = 1):
    return lo.decode_attn(wl.bf16_bits(inp.q), wl.bf16_bits(inp.k_cache), wl.bf16_bits(inp.v_cache),
                          np.asarray(mask, np.uint8), k, idx_in, inp.lengths, want_sel=True,
                          keep_ppm=keep_ppm, block=block)


def unit_scores(sel_row: np.ndarray, L: int, block: int) -> np.ndarray:
    """What the sets rank: a position's pooled score, or a block's best one."""
    if block == 1:
        return sel_row[:L]
    return np.maximum.reduceat(sel_row[:L], np.arange(0, L, block))


def assert_outputs_close(got: np.ndarray, ref: np.ndarray, what=""):
    err = np.abs(got - ref)
    bound = ABS_TOL + REL_TOL * np.abs(ref)
    if not (err <= bound).all():
        bad = np.argwhere(err > bound)[0]
        raise AssertionError("%s: output differs at %s: got %r, oracle %r (max abs err %.4g)" % (
            what, tuple(bad), got[tuple(bad)], ref[tuple(bad)], err.max()))
    return float(err.max())


def assert_sets_match(idx_gpu, idx_ref, sel_ref, mask, inp: wl.LayerInputs, k, idx_in, what="",
                      keep_ppm: int = 0, block: int = 1):
    """Per (sequence, KV head): retrieval groups match the oracle's set (differences only at
    oracle ties), are ascending and -1 padded; other groups are a verbatim copy of idx_in.
    Returns the number of positions that differed inside the tie allowance."""
    w = inp.workload
    G = w.group
    n_diff = 0
    for b in range(w.batch):
        L = -(-int(inp.lengths[b]) // block)       # units: positions, or blocks
        n = lo.ratio_budget(L, k, keep_ppm)
        for g in range(w.n_kv_heads):
            got = idx_gpu[b, g]
            if np.asarray(mask[g * G:(g + 1) * G]).any():
                valid = got[:n]
                assert (got[n:] == -1).all(), "%s: padding b=%d g=%d" % (what, b, g)
                assert (np.diff(valid) > 0).all(), "%s: not ascending b=%d g=%d" % (what, b, g)
                assert valid.min() >= 0 and valid.max() < L
                ok, nd, msg = index_sets_match(got, idx_ref[b, g],
                                               unit_scores(sel_ref[b, g], int(inp.lengths[b]), block), n, TIE_REL)
                assert ok, "%s: b=%d g=%d: %s" % (what, b, g, msg)
                n_diff += nd
            else:
                assert (got == idx_in[b, g]).all(), "%s: pass-through b=%d g=%d" % (what, b, g)
    return n_diff


def check_layer(ctx, inp: wl.LayerInputs, mask, k, idx_in, what="", exact_sets=False, keep_ppm: int = 0,
                block: int = 1):
    """Run one hybrid layer call on the GPU and compare everything with the oracle."""
    dl = DeviceLayer(inp, k, idx_in, keep_ppm=keep_ppm, block=block)
    out_gpu, idx_gpu = run_hybrid(ctx, dl, np.asarray(mask, np.uint8))
    out_ref, idx_ref, sel_ref = oracle_layer(inp, mask, k, idx_in, keep_ppm, block)
    assert_outputs_close(out_gpu, out_ref, what)
    n_diff = assert_sets_match(idx_gpu, idx_ref, sel_ref, mask, inp, k, idx_in, what, keep_ppm, block)
    if exact_sets:
        assert n_diff == 0, "%s: %d positions differ from the oracle's sets" % (what, n_diff)
    return dl, out_gpu, idx_gpu, out_ref, idx_ref, sel_ref


def check_prob_rule_layer(ctx, inp: wl.LayerInputs, mask, k, rule, param, what="", idx_in=None):
    """One all-in-one check of a Threshold (rule 1) / Top-p (rule 2) layer call: outputs as usual;
    every selected set must be the oracle's top set of its own size, and its size must be the
    oracle's, or differ only by positions whose probability (cumulative probability) lies within
    fp32 rounding of the parameter.  Returns the sizes [B][H_kv] (0 for groups that keep theirs)."""
    lb = binding()
    w = inp.workload
    dl = DeviceLayer(inp, k, idx_in)
    dl.shape = lb.make_shape(w.batch, w.n_q_heads, w.n_kv_heads, dl.k_cache.shape[2], k, kv=dl.k_cache,
                             prob_rule=rule, prob_param=param)
    out_gpu, idx_gpu = run_hybrid(ctx, dl, np.asarray(mask, np.uint8))
    out_ref, idx_ref, sel_ref = lo.decode_attn(wl.bf16_bits(inp.q), wl.bf16_bits(inp.k_cache),
                                               wl.bf16_bits(inp.v_cache), np.asarray(mask, np.uint8), k, idx_in,
                                               inp.lengths, want_sel=True, rule=rule, rule_param=param)
    assert_outputs_close(out_gpu, out_ref, what)
    sizes = np.zeros((w.batch, w.n_kv_heads), np.int64)
    G = w.group
    for b in range(w.batch):
        L = int(inp.lengths[b])
        for g in range(w.n_kv_heads):
            if not np.asarray(mask[g * G:(g + 1) * G]).any():
                continue
            got = idx_gpu[b, g]
            n_g = int((got >= 0).sum())
            n_o = int((idx_ref[b, g] >= 0).sum())
            sizes[b, g] = n_g
            assert 1 <= n_g <= min(k, L) and (got[n_g:] == -1).all() and (np.diff(got[:n_g]) > 0).all()
            sel = sel_ref[b, g, :L]
            ref_same_size = lo.topk(sel, n_g)                    # the oracle's top set of the GPU's size
            ok, _, msg = index_sets_match(got[:n_g], ref_same_size, sel, n_g, TIE_REL)
            assert ok, "%s: b=%d g=%d: %s" % (what, b, g, msg)
            if n_g == n_o:
                continue
            # sizes differ: only by positions at the very edge of the rule
            order = np.array(sorted(range(L), key=lambda t: (-sel[t], t)))
            m = sel.max()
            prob = np.exp(sel - m) / np.exp(sel - m).sum()
            lo_n, hi_n = min(n_g, n_o), max(n_g, n_o)
            between = order[lo_n:hi_n]
            if rule == 1:
                assert (np.abs(np.log(prob[between]) - np.log(param)) <= 1e-3).all(), \
                    "%s: b=%d g=%d: sizes %d / %d differ away from the threshold" % (what, b, g, n_g, n_o)
            else:
                cum = np.cumsum(prob[order])
                # the smaller set already holds the mass, to within fp32 rounding of it
                assert abs(cum[lo_n - 1] - param) <= 1e-4 * param, \
                    "%s: b=%d g=%d: sizes %d / %d differ away from the mass %r" % (what, b, g, n_g, n_o, param)
    return sizes
