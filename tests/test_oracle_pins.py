"""Pins of the CPU oracle against what the paper's equations and plain mathematics fix.

None of these tests re-types the oracle's own formula in the oracle's own style and
calls it a check: each compares against brute force in pure Python, a library routine
(torch fp64 softmax / matmul), a closed form, or an invariant of Eq. 1-3.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import lychee_oracle as lo
from paper_2602_04541_amd import workloads as wl
from tests.helpers import bits_to_f64, round_to_bf16_bits, to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_form_cases.json")


def _rand_bits(rng, shape, scale=1.0):
    return round_to_bf16_bits(rng.standard_normal(shape).astype(np.float32) * scale)


def _tiny(rng, B=2, Hq=4, Hkv=2, L=13, d=6, l_cap=None):
    l_cap = l_cap or L
    q = _rand_bits(rng, (B, Hq, d))
    K = _rand_bits(rng, (B, Hkv, l_cap, d))
    V = _rand_bits(rng, (B, Hkv, l_cap, d))
    return q, K, V


# --------------------------------------------------------------------------- golden
@pytest.mark.parametrize("case", json.load(open(GOLDEN))["cases"], ids=lambda c: c["name"])
def test_closed_form_cases(case):
    d, k = case["d"], case["k"]
    q = to_bf16_bits(case["q"])[None]                      # [1, Hq, d]
    K = to_bf16_bits(case["K"])[None, None]                # [1, 1, L, d]
    V = to_bf16_bits(case["V"])[None, None]
    L = K.shape[2]
    idx_in = None if case["idx_in"] is None else np.asarray(case["idx_in"], np.int32)[None, None]
    out, idx_out, _ = lo.decode_attn(q, K, V, np.asarray(case["mask"], np.uint8), k, idx_in,
                                     np.asarray([L], np.int32))
    np.testing.assert_allclose(out[0], np.asarray(case["expect_out"]), rtol=0, atol=1e-14)
    assert idx_out[0, 0].tolist() == case["expect_idx_out"]


def test_tie_case_with_larger_budget():
    # same logits (1,3,3,2,3): k = 4 keeps {1,2,3,4}; k = 7 > L pads with -1
    s = np.array([1.0, 3.0, 3.0, 2.0, 3.0])
    assert lo.topk(s, 4).tolist() == [1, 2, 3, 4]
    assert lo.topk(s, 3).tolist() == [1, 2, 4]
    assert lo.topk(s, 7).tolist() == [0, 1, 2, 3, 4, -1, -1]


# ---------------------------------------------------------------- brute force, Eq. 1
def test_scores_against_pure_python_loops():
    rng = np.random.default_rng(1)
    L, d = 7, 5                                            # non-square: a transposed read fails
    q = _rand_bits(rng, (d,))
    K = _rand_bits(rng, (L, d))
    qf, Kf = bits_to_f64(q).tolist(), bits_to_f64(K).tolist()
    want = [math.fsum(qf[i] * Kf[t][i] for i in range(d)) / math.sqrt(d) for t in range(L)]
    np.testing.assert_allclose(lo.scores(q, K), want, rtol=1e-14, atol=1e-15)


def test_softmax_weights_properties():
    rng = np.random.default_rng(2)
    s = rng.standard_normal(50) * 5
    pos = rng.permutation(50)[:20].astype(np.int32)
    w = lo.softmax_weights(s, pos)
    assert abs(w.sum() - 1.0) < 1e-12 and (w > 0).all()
    # strictly monotone in the logit; ratio of two weights is exp of the logit gap
    order = np.argsort(s[pos])
    assert (np.diff(w[order]) >= 0).all()
    np.testing.assert_allclose(w[3] / w[7], math.exp(s[pos[3]] - s[pos[7]]), rtol=1e-12)
    # shift invariance of softmax
    np.testing.assert_allclose(lo.softmax_weights(s + 123.0, pos), w, rtol=1e-10)
    # huge logits do not overflow
    big = np.array([1000.0, 999.0, -1000.0])
    wb = lo.softmax_weights(big, np.arange(3, dtype=np.int32))
    np.testing.assert_allclose(wb, [1 / (1 + math.exp(-1)), math.exp(-1) / (1 + math.exp(-1)), 0.0],
                               atol=1e-15)


def test_weighted_values_against_pure_python_loops():
    rng = np.random.default_rng(3)
    L, d = 9, 4
    V = _rand_bits(rng, (L, d))
    pos = np.array([8, 0, 3], np.int32)
    w = np.array([0.2, 0.5, 0.3])
    Vf = bits_to_f64(V).tolist()
    want = [math.fsum(w[j] * Vf[pos[j]][i] for j in range(3)) for i in range(d)]
    np.testing.assert_allclose(lo.weighted_values(w, pos, V), want, rtol=1e-14)


# ------------------------------------------------------------- library routine, Eq. 1
@pytest.mark.parametrize("B,Hq,Hkv,L,d", [(2, 8, 2, 37, 16), (1, 6, 6, 5, 128), (3, 4, 1, 64, 8)])
def test_all_retrieval_equals_library_gqa_attention(B, Hq, Hkv, L, d):
    rng = np.random.default_rng(4)
    q, K, V = _tiny(rng, B, Hq, Hkv, L, d)
    out = lo.dense_attn(q, K, V, np.full(B, L, np.int32))
    G = Hq // Hkv
    qt = torch.from_numpy(bits_to_f64(q))
    Kt = torch.from_numpy(bits_to_f64(K)).repeat_interleave(G, dim=1)
    Vt = torch.from_numpy(bits_to_f64(V)).repeat_interleave(G, dim=1)
    att = torch.softmax(torch.matmul(Kt, qt[..., None])[..., 0] / math.sqrt(d), dim=-1)
    want = torch.matmul(att[:, :, None, :], Vt)[:, :, 0, :].numpy()
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)


def test_outputs_are_convex_combinations_of_value_rows():
    rng = np.random.default_rng(5)
    q, K, V = _tiny(rng, 1, 4, 2, 21, 8)
    out = lo.dense_attn(q, K, V, np.array([21], np.int32))
    Vf = bits_to_f64(V)
    for h in range(4):
        g = h // 2
        assert (out[0, h] <= Vf[0, g].max(0) + 1e-12).all()
        assert (out[0, h] >= Vf[0, g].min(0) - 1e-12).all()


# ------------------------------------------------------------------ Eq. 3 special cases
def test_sparse_with_full_set_equals_dense():
    rng = np.random.default_rng(6)
    B, Hq, Hkv, L, d = 2, 4, 2, 19, 8
    q, K, V = _tiny(rng, B, Hq, Hkv, L, d)
    lens = np.full(B, L, np.int32)
    full = np.tile(np.arange(L, dtype=np.int32), (B, Hkv, 1))
    sparse, idx_out, _ = lo.decode_attn(q, K, V, np.zeros(Hq, np.uint8), L, full, lens)
    dense = lo.dense_attn(q, K, V, lens)
    np.testing.assert_allclose(sparse, dense, rtol=1e-13, atol=1e-14)
    assert (idx_out == full).all()


def test_sparse_ignores_rows_outside_the_set_and_the_order_of_the_set():
    rng = np.random.default_rng(7)
    B, Hq, Hkv, L, d, k = 1, 4, 2, 31, 8, 6
    q, K, V = _tiny(rng, B, Hq, Hkv, L, d)
    lens = np.full(B, L, np.int32)
    idx = np.stack([np.sort(rng.permutation(L)[:k]) for _ in range(Hkv)])[None].astype(np.int32)
    mask = np.zeros(Hq, np.uint8)
    base, _, _ = lo.decode_attn(q, K, V, mask, k, idx, lens)
    K2, V2 = K.copy(), V.copy()
    for g in range(Hkv):
        outside = np.setdiff1d(np.arange(L), idx[0, g])
        K2[0, g, outside] = _rand_bits(rng, (outside.size, d), 50.0)
        V2[0, g, outside] = _rand_bits(rng, (outside.size, d), 50.0)
    again, _, _ = lo.decode_attn(q, K2, V2, mask, k, idx, lens)
    assert (again == base).all()
    shuffled = idx[:, :, rng.permutation(k)]
    perm, idx_out, _ = lo.decode_attn(q, K, V, mask, k, shuffled, lens)
    np.testing.assert_allclose(perm, base, rtol=1e-12, atol=1e-14)
    assert (idx_out == shuffled).all()                      # handed on bit for bit
    # -1 padding is skipped: a padded set gives what the short set gives
    padded = np.concatenate([idx, np.full((1, Hkv, 3), -1, np.int32)], axis=2)
    pad_out, _, _ = lo.decode_attn(q, K, V, mask, k + 3, padded, lens)
    assert (pad_out == base).all()


def test_sparse_against_library_on_the_gathered_rows():
    rng = np.random.default_rng(8)
    L, d, k = 40, 16, 9
    q, K, V = _tiny(rng, 1, 1, 1, L, d)
    idx = np.sort(rng.permutation(L)[:k]).astype(np.int32)
    out, _, _ = lo.decode_attn(q, K, V, np.zeros(1, np.uint8), k, idx[None, None],
                               np.array([L], np.int32))
    Ks = torch.from_numpy(bits_to_f64(K[0, 0, idx]))
    Vs = torch.from_numpy(bits_to_f64(V[0, 0, idx]))
    qt = torch.from_numpy(bits_to_f64(q[0, 0]))
    want = (torch.softmax(Ks @ qt / math.sqrt(d), 0) @ Vs).numpy()
    np.testing.assert_allclose(out[0, 0], want, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------------ Eq. 2, top-k
def test_topk_against_python_sorted_for_every_k_with_ties():
    rng = np.random.default_rng(9)
    for L in (1, 2, 17, 64):
        s = np.round(rng.standard_normal(L) * 2) / 2       # many exact ties
        for k in range(1, L + 3):
            ranked = sorted(range(L), key=lambda t: (-s[t], t))
            want = sorted(ranked[:min(k, L)]) + [-1] * max(0, k - L)
            assert lo.topk(s, k).tolist() == want


def test_selection_uses_the_mean_logit_of_the_groups_retrieval_heads():
    """App. F pooling, by linearity: top-k of (mean of the retrieval q's) . K."""
    rng = np.random.default_rng(10)
    B, Hq, Hkv, L, d, k = 1, 8, 2, 50, 16, 7
    q, K, V = _tiny(rng, B, Hq, Hkv, L, d)
    mask = np.array([1, 0, 1, 1, 0, 0, 0, 1], np.uint8)     # group 0: heads 0,2,3; group 1: head 7
    idx_in = np.tile(np.arange(k, dtype=np.int32), (B, Hkv, 1))
    _, idx_out, sel = lo.decode_attn(q, K, V, mask, k, idx_in, np.array([L], np.int32),
                                     want_sel=True)
    qf, Kf = bits_to_f64(q), bits_to_f64(K)
    for g, heads in ((0, [0, 2, 3]), (1, [7])):
        pooled_q = qf[0, heads].mean(0)
        pooled_logit = Kf[0, g] @ pooled_q / math.sqrt(d)
        np.testing.assert_allclose(sel[0, g], pooled_logit, rtol=1e-12, atol=1e-13)
        want = np.sort(np.argsort(-pooled_logit, kind="stable")[:k])
        assert idx_out[0, g].tolist() == want.tolist()


def test_sets_pass_through_groups_without_a_retrieval_head():
    rng = np.random.default_rng(11)
    B, Hq, Hkv, L, d, k = 2, 6, 3, 20, 8, 5
    q, K, V = _tiny(rng, B, Hq, Hkv, L, d)
    mask = np.array([0, 0, 1, 0, 0, 0], np.uint8)           # only group 1 selects
    idx_in = rng.integers(0, L, size=(B, Hkv, k)).astype(np.int32)
    idx_in[0, 0, 3:] = -1
    _, idx_out, _ = lo.decode_attn(q, K, V, mask, k, idx_in, np.full(B, L, np.int32))
    assert (idx_out[:, 0] == idx_in[:, 0]).all() and (idx_out[:, 2] == idx_in[:, 2]).all()
    assert not (idx_out[:, 1] == idx_in[:, 1]).all()


# ----------------------------------------------------------- lengths, strides, workloads
def test_ragged_lengths_equal_the_truncated_problem_and_strides_are_honoured():
    rng = np.random.default_rng(12)
    B, Hq, Hkv, L, d, k, cap = 2, 4, 2, 11, 8, 4, 16
    q, K, V = _tiny(rng, B, Hq, Hkv, L, d, l_cap=cap)
    lens = np.array([11, 6], np.int32)
    mask = np.array([1, 0, 0, 1], np.uint8)
    idx_in = np.tile(np.arange(k, dtype=np.int32), (B, Hkv, 1))
    out, idx_out, _ = lo.decode_attn(q, K, V, mask, k, idx_in, lens)
    for b in range(B):
        Lb = int(lens[b])
        o1, i1, _ = lo.decode_attn(q[b:b + 1], np.ascontiguousarray(K[b:b + 1, :, :Lb]),
                                   np.ascontiguousarray(V[b:b + 1, :, :Lb]), mask, k,
                                   idx_in[b:b + 1], lens[b:b + 1])
        assert (o1 == out[b:b + 1]).all() and (i1 == idx_out[b:b + 1]).all()
    # the same cache embedded in a wider buffer (token stride 2d, padded heads)
    wide_k = np.zeros((B, Hkv + 1, cap, 2 * d), np.uint16)
    wide_v = np.zeros_like(wide_k)
    wide_k[:, :Hkv, :, :d], wide_v[:, :Hkv, :, :d] = K, V
    o2, i2, _ = lo.decode_attn(q, wide_k[:, :Hkv, :, :d], wide_v[:, :Hkv, :, :d], mask, k,
                               idx_in, lens)
    assert (o2 == out).all() and (i2 == idx_out).all()


def test_planted_rows_are_selected_on_the_small_workload():
    w = wl.WORKLOADS["c1"]
    inp = wl.make_layer(w)
    q, K, V = (wl.bf16_bits(t) for t in (inp.q, inp.k_cache, inp.v_cache))
    prev = np.tile(np.arange(w.k, dtype=np.int32), (1, w.n_kv_heads, 1))
    out, idx_out, sel = lo.decode_attn(q, K, V, inp.mask, w.k, prev, inp.lengths, want_sel=True)
    for g in range(w.n_kv_heads):
        assert np.isin(inp.planted_pos[0, g], idx_out[0, g]).all()
        assert (np.diff(idx_out[0, g]) > 0).all()
        # planted logits sit near 3*||q*|| and far above the N(0,1) background
        assert sel[0, g, inp.planted_pos[0, g]].min() > 20.0
    assert np.isfinite(out).all()


def test_oracle_rejects_bad_arguments():
    rng = np.random.default_rng(13)
    q, K, V = _tiny(rng, 1, 4, 2, 8, 4)
    with pytest.raises(ValueError):                          # sparse heads but no set
        lo.decode_attn(q, K, V, np.zeros(4, np.uint8), 2, None, np.array([8], np.int32))
    with pytest.raises(ValueError):                          # length beyond the cache
        lo.decode_attn(q, K, V, np.ones(4, np.uint8), 2, None, np.array([9], np.int32))
    with pytest.raises(ValueError):                          # index beyond the length
        lo.decode_attn(q, K, V, np.zeros(4, np.uint8), 2,
                       np.full((1, 2, 2), 7, np.int32), np.array([5], np.int32))


# ------------------------------------------------------------------ the Ratio rule (Sec. 4.4.1)
def test_ratio_budget_is_the_rounded_up_share_clamped_to_the_set_capacity():
    from fractions import Fraction
    import math
    for L in (1, 2, 7, 64, 1000, 4097, 131072):
        for ppm in (1, 100000, 300000, 333333, 500000, 999999, 1000000):
            want = max(1, math.ceil(Fraction(L * ppm, 1000000)))     # exact rational arithmetic
            for k in (1, 5, L, 2 * L):
                assert lo.ratio_budget(L, k, ppm) == min(want, k, L), (L, ppm, k)
    # theta = 70 % of the tokens dropped (App. E.2's sparsity table) keeps 30 % of them
    assert lo.ratio_budget(100000, 10 ** 6, 300000) == 30000
    assert lo.ratio_budget(10, 4, 0) == 4 and lo.ratio_budget(3, 4, 0) == 3   # rule off: min(k, L)


def test_ratio_rule_selects_the_top_share_per_sequence_and_nests():
    rng = np.random.default_rng(11)
    B, Hq, Hkv, d, cap = 3, 4, 2, 128, 40
    lens = np.array([37, 80, 5], np.int32)
    q = round_to_bf16_bits(rng.standard_normal((B, Hq, d)))
    K = round_to_bf16_bits(rng.standard_normal((B, Hkv, 80, d)))
    K[:, :, 10] = K[:, :, 3]                       # an exact tie inside every head
    V = round_to_bf16_bits(rng.standard_normal((B, Hkv, 80, d)))
    mask = np.ones(Hq, np.uint8)
    prev = None
    for ppm in (100000, 250000, 500000, 1000000):
        out, idx, sel = lo.decode_attn(q, K, V, mask, cap, None, lens, want_sel=True, keep_ppm=ppm)
        out0, _, _ = lo.decode_attn(q, K, V, mask, cap, None, lens)
        assert (out == out0).all()                 # the rule changes the sets, not this layer's output
        for b in range(B):
            L = int(lens[b])
            n = min(cap, L, max(1, -(-L * ppm // 1000000)))
            for g in range(Hkv):
                order = sorted(range(L), key=lambda t: (-sel[b, g, t], t))      # brute force
                want = sorted(order[:n])
                got = idx[b, g]
                assert list(got[:n]) == want and (got[n:] == -1).all(), (ppm, b, g)
                if prev is not None:               # a larger share keeps everything a smaller one kept
                    assert set(prev[b, g][prev[b, g] >= 0]) <= set(got[got >= 0])
        prev = idx


def test_ratio_rule_with_the_share_that_gives_k_equals_topk():
    rng = np.random.default_rng(12)
    q = round_to_bf16_bits(rng.standard_normal((1, 2, 128)))
    K = round_to_bf16_bits(rng.standard_normal((1, 1, 200, 128)))
    V = round_to_bf16_bits(rng.standard_normal((1, 1, 200, 128)))
    lens = np.array([200], np.int32)
    mask = np.ones(2, np.uint8)
    _, idx_k, _ = lo.decode_attn(q, K, V, mask, 50, None, lens)
    _, idx_r, _ = lo.decode_attn(q, K, V, mask, 64, None, lens, keep_ppm=250000)   # 25 % of 200 = 50
    assert (idx_r[0, 0, :50] == idx_k[0, 0]).all() and (idx_r[0, 0, 50:] == -1).all()


# ------------------------------------------------------------------ block-granular sets (App. C)
def _block_case(seed, B=2, Hq=4, Hkv=2, L_cap=300, lens=(300, 170)):
    rng = np.random.default_rng(seed)
    q = round_to_bf16_bits(rng.standard_normal((B, Hq, 128)))
    K = round_to_bf16_bits(rng.standard_normal((B, Hkv, L_cap, 128)))
    V = round_to_bf16_bits(rng.standard_normal((B, Hkv, L_cap, 128)))
    return q, K, V, np.array(lens, np.int32)


@pytest.mark.parametrize("block", [4, 64])
def test_block_sets_rank_blocks_by_their_best_token(block):
    q, K, V, lens = _block_case(21)
    K[:, :, 7] = K[:, :, 150]                      # a tie between the best tokens of two blocks
    mask = np.ones(4, np.uint8)
    for kb in (1, 2, 3, 100):
        _, idx, sel = lo.decode_attn(q, K, V, mask, kb, None, lens, want_sel=True, block=block)
        for b in range(2):
            L = int(lens[b])
            units = -(-L // block)
            n = min(kb, units)
            for g in range(2):
                score = [max(sel[b, g, u * block:min((u + 1) * block, L)]) for u in range(units)]
                order = sorted(range(units), key=lambda u: (-score[u], u))    # brute force
                assert list(idx[b, g][:n]) == sorted(order[:n]) and (idx[b, g][n:] == -1).all()
                best_token = int(np.argmax(sel[b, g, :L]))
                assert best_token // block in idx[b, g][:n]   # the best token's block is always kept


def test_block_sparse_attention_equals_token_sparse_attention_on_the_same_positions():
    block = 16
    q, K, V, lens = _block_case(22, lens=(300, 171))          # 171: the last block is ragged
    K[:, :, 171:] = 1000.0                                     # rows past a length must never be read
    mask = np.array([0, 1, 0, 0], np.uint8)
    idx_blocks = np.full((2, 2, 5), -1, np.int32)
    idx_blocks[0, :, :4] = [0, 3, 9, 18]                       # 18 is the last block of 300 rows
    idx_blocks[1, :, :3] = [10, 2, 5]                          # 10 is the ragged last block of 171 rows
    out_b, idx_b, _ = lo.decode_attn(q, K, V, mask, 5, idx_blocks, lens, block=block)
    idx_tok = np.full((2, 2, 5 * block), -1, np.int32)
    for b in range(2):
        for g in range(2):
            pos = [t for e in idx_blocks[b, g] if e >= 0 for t in range(e * block, min((e + 1) * block, int(lens[b])))]
            idx_tok[b, g, :len(pos)] = pos
    out_t, _, _ = lo.decode_attn(q, K, V, mask, 5 * block, idx_tok, lens, block=1)
    sparse_heads = [0, 2, 3]
    assert (out_b[:, sparse_heads] == out_t[:, sparse_heads]).all()
    assert (idx_b[:, 1] == idx_blocks[:, 1]).all()            # group 1 holds no retrieval head: handed on


def test_block_of_one_is_the_token_method_and_ratio_counts_blocks():
    q, K, V, lens = _block_case(23)
    mask = np.ones(4, np.uint8)
    a = lo.decode_attn(q, K, V, mask, 40, None, lens)
    b = lo.decode_attn(q, K, V, mask, 40, None, lens, block=1)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()
    _, idx, _ = lo.decode_attn(q, K, V, mask, 40, None, lens, keep_ppm=250000, block=8)
    assert ((idx[0] >= 0).sum(axis=1) == 10).all()            # 300 rows = 38 blocks of 8; a quarter, rounded up
    assert ((idx[1] >= 0).sum(axis=1) == 6).all()             # 170 rows = 22 blocks; ceil(5.5) = 6


# ------------------------------------------------------------------ the cache append of Alg. 1
def test_append_puts_the_new_rows_at_the_last_position_of_every_head_and_nowhere_else():
    rng = np.random.default_rng(31)
    B, Hkv, L_cap, d = 3, 2, 20, 128
    lens = np.array([20, 1, 7], np.int32)
    K = round_to_bf16_bits(rng.standard_normal((B, Hkv, L_cap, d)))
    V = round_to_bf16_bits(rng.standard_normal((B, Hkv, L_cap, d)))
    kn = round_to_bf16_bits(rng.standard_normal((B, Hkv, d)))
    vn = round_to_bf16_bits(rng.standard_normal((B, Hkv, d)))
    K2, V2 = K.copy(), V.copy()
    lo.append_kv(kn, vn, K2, V2, lens)
    want_k, want_v = K.copy(), V.copy()
    for b in range(B):
        want_k[b, :, lens[b] - 1] = kn[b]          # numpy indexing, not the oracle's loop
        want_v[b, :, lens[b] - 1] = vn[b]
    assert (K2 == want_k).all() and (V2 == want_v).all()
    # token-major storage: same logical result through other strides
    Kt = np.ascontiguousarray(K.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    Vt = np.ascontiguousarray(V.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    lo.append_kv(kn, vn, Kt, Vt, lens)
    assert (Kt == want_k).all() and (Vt == want_v).all()


# ------------------------------------------------------------------ Top-p and Threshold (Sec. 4.4.1)
def test_threshold_and_top_p_counts_against_a_library_softmax():
    from scipy.special import softmax
    rng = np.random.default_rng(41)
    for L in (1, 5, 64, 1000):
        sel = rng.standard_normal(L) * 3.0
        if L > 10:
            sel[7] = sel[3]                                   # a tie
        p = softmax(sel)                                      # library routine
        order = sorted(range(L), key=lambda t: (-sel[t], t))
        for tau in (1e-1, 1e-2, 1e-3, 1e-6):
            assert lo.rule_count(sel, lo.RULE_THRESHOLD, tau) == int((p > tau).sum())
        for pp in (0.2, 0.5, 0.9, 0.99, 0.999):
            cum, n = 0.0, 0
            while n < L and cum < pp:
                cum += p[order[n]]
                n += 1
            assert lo.rule_count(sel, lo.RULE_TOP_P, pp) == n
    # closed forms: L equal logits have probability 1/L each
    flat = np.zeros(10)
    assert lo.rule_count(flat, lo.RULE_THRESHOLD, 0.09) == 10 and lo.rule_count(flat, lo.RULE_THRESHOLD, 0.11) == 0
    assert lo.rule_count(flat, lo.RULE_TOP_P, 0.25) == 3 and lo.rule_count(flat, lo.RULE_TOP_P, 1.0) == 10
    # one dominant logit: probability ~ 1 - 9 e^-30
    spike = np.zeros(10)
    spike[4] = 30.0
    assert lo.rule_count(spike, lo.RULE_TOP_P, 0.999) == 1 and lo.rule_count(spike, lo.RULE_THRESHOLD, 0.5) == 1


def test_threshold_and_top_p_sets_are_top_sets_capped_at_k_and_never_empty():
    rng = np.random.default_rng(42)
    q = round_to_bf16_bits(rng.standard_normal((2, 4, 128)) * 2.0)
    K = round_to_bf16_bits(rng.standard_normal((2, 2, 300, 128)))
    V = round_to_bf16_bits(rng.standard_normal((2, 2, 300, 128)))
    lens = np.array([300, 120], np.int32)
    mask = np.ones(4, np.uint8)
    for rule, params in ((lo.RULE_THRESHOLD, (0.5, 1e-2, 1e-3, 1e-9)), (lo.RULE_TOP_P, (0.01, 0.5, 0.9, 1.0))):
        sizes = []
        for param in params:
            _, idx, sel = lo.decode_attn(q, K, V, mask, 64, None, lens, want_sel=True, rule=rule, rule_param=param)
            for b in range(2):
                L = int(lens[b])
                for g in range(2):
                    n = int((idx[b, g] >= 0).sum())
                    want = min(64, L, max(1, lo.rule_count(sel[b, g, :L], rule, param)))
                    assert n == want
                    order = sorted(range(L), key=lambda t: (-sel[b, g, t], t))
                    assert list(idx[b, g][:n]) == sorted(order[:n]) and (idx[b, g][n:] == -1).all()
            sizes.append((idx >= 0).sum())
        # looser parameters keep more: tau falls / p rises along params
        assert sizes == sorted(sizes)
    _, idx_cap, _ = lo.decode_attn(q, K, V, mask, 64, None, lens, rule=lo.RULE_TOP_P, rule_param=1.0)
    _, idx_k, _ = lo.decode_attn(q, K, V, mask, 64, None, lens)
    assert (idx_cap == idx_k).all()                          # p = 1 wants everything: the cap is Top-k
