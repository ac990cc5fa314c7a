"""Pins for the fp64 CPU oracle: each step is checked against something other
than itself -- a closed form, an invariant, a reduction to a library routine
(torch's CPU scaled_dot_product_attention in fp64), a brute force written here
in numpy, or a number the paper prints.  No GPU needed."""
import math
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def sdpa64(q, k, v, scale):
    """Library cross-check: torch CPU SDPA in float64 on [n, h, d] arrays."""
    tq, tk, tv = (torch.from_numpy(np.asarray(a, dtype=np.float64)).permute(1, 0, 2) for a in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)
    return o.permute(1, 0, 2).numpy()


def masked_dense_bruteforce(q, k, v, idx, block, scale):
    """Second, independently written route for the selection branch: build the
    full n x n boolean mask from the block index sets, then masked softmax."""
    n, heads, d = q.shape
    n_blk = (n + block - 1) // block
    out = np.zeros((n, heads, d))
    lse = np.zeros((heads, n))
    blk_of = np.arange(n) // block
    for h in range(heads):
        allowed_blocks = np.zeros((n_blk, n_blk), dtype=bool)
        for i in range(n_blk):
            allowed_blocks[i, idx[h, i]] = True
        mask = allowed_blocks[blk_of][:, blk_of]                      # [n, n]
        logits = scale * (q[:, h].astype(np.float64) @ k[:, h].astype(np.float64).T)
        logits = np.where(mask, logits, -np.inf)
        mx = logits.max(axis=1, keepdims=True)
        e = np.exp(logits - mx)
        den = e.sum(axis=1, keepdims=True)
        out[:, h] = (e / den) @ v[:, h].astype(np.float64)
        lse[h] = (mx + np.log(den))[:, 0]
    return out, lse


def flat_tokens(oracle, x_rows, n_tok, block):
    rows = np.arange((n_tok + block - 1) // block)
    tok, vals = oracle.rows_to_tokens(x_rows, rows, n_tok, block)
    assert np.array_equal(tok, np.arange(n_tok))
    return vals


# ----------------------------------------------------------------- pooling --

def test_pool_block1_is_identity(oracle):
    x = rnd((37, 3, 8), 1)
    xc = oracle.pool(x, 1)
    assert np.array_equal(xc, x.astype(np.float64).transpose(1, 0, 2))


def test_pool_hand_case_with_tail(oracle):
    # n = 5, block = 2: blocks {0,1}, {2,3}, {4}; the tail is averaged over 1 token.
    x = np.arange(5 * 1 * 2, dtype=np.float32).reshape(5, 1, 2)      # token t = (2t, 2t+1)
    xc = oracle.pool(x, 2)
    expect = np.array([[[1.0, 2.0], [5.0, 6.0], [8.0, 9.0]]])
    assert np.array_equal(xc, expect)


def test_pool_constant_and_sum_identity(oracle):
    x = np.full((130, 2, 4), 0.375, dtype=np.float32)
    assert np.array_equal(oracle.pool(x, 64), np.full((2, 3, 4), 0.375))
    y = rnd((130, 2, 4), 2)
    yc = oracle.pool(y, 64)
    lens = np.array([64, 64, 2], dtype=np.float64)
    total = (yc * lens[None, :, None]).sum(axis=1)
    assert np.allclose(total, y.astype(np.float64).sum(axis=0), rtol=0, atol=1e-12)


def test_pool_heads_not_mixed(oracle):
    x = rnd((64, 3, 4), 3)
    x2 = x.copy()
    x2[:, 1] += 7.0
    a, b = oracle.pool(x, 16), oracle.pool(x2, 16)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2])
    assert np.allclose(b[1] - a[1], 7.0, atol=1e-6)


# ------------------------------------------------------------------ scores --

def test_scores_equal_mean_of_token_dots(oracle):
    # Linearity of eq. 4: S[i, j] = mean over (t in i, u in j) of q_t . k_u, tails included.
    n, h, d, b = 29, 2, 5, 4
    q, k = rnd((n, h, d), 4), rnd((n, h, d), 5)
    s = oracle.scores(oracle.pool(q, b), oracle.pool(k, b))
    n_blk = (n + b - 1) // b
    for hh in range(h):
        full = q[:, hh].astype(np.float64) @ k[:, hh].astype(np.float64).T
        for i in range(n_blk):
            for j in range(n_blk):
                ref = full[i * b:(i + 1) * b, j * b:(j + 1) * b].mean()
                assert abs(s[hh, i, j] - ref) < 1e-12


def test_scores_not_symmetric_and_rows_subset(oracle):
    # A transposed operand (k.q instead of q.k) or a wrong row gather must fail here.
    n, h, d, b = 40, 1, 3, 4
    q, k = rnd((n, h, d), 6), rnd((n, h, d), 7)
    qc, kc = oracle.pool(q, b), oracle.pool(k, b)
    s = oracle.scores(qc, kc)
    assert np.allclose(s[0], qc[0] @ kc[0].T, atol=1e-13)
    assert not np.allclose(s[0], s[0].T)
    rows = np.array([7, 2, 9])
    assert np.array_equal(oracle.scores(qc, kc, rows), s[:, rows])


# ----------------------------------------------------- compressed attention --

def test_compressed_block1_equals_dense_sdpa(oracle):
    n, h, d = 50, 2, 8
    q, k, v = rnd((n, h, d), 8), rnd((n, h, d), 9), rnd((n, h, d), 10)
    scale = 0.3
    qc, kc, vc = (oracle.pool(a, 1) for a in (q, k, v))
    oc = oracle.compressed_attn(oracle.scores(qc, kc), vc, scale)          # [h, n, d]
    ref = sdpa64(q, k, v, scale)                                            # [n, h, d]
    assert np.allclose(oc.transpose(1, 0, 2), ref, rtol=0, atol=1e-13)


def test_compressed_constant_value_and_uniform_keys(oracle):
    h, nb, d = 2, 9, 4
    s = np.random.default_rng(11).standard_normal((h, nb, nb))
    vc = np.full((h, nb, d), -2.5)
    assert np.allclose(oracle.compressed_attn(s, vc, 0.7), -2.5, atol=1e-14)      # rows sum to 1
    vc2 = np.random.default_rng(12).standard_normal((h, nb, d))
    flat = oracle.compressed_attn(np.zeros((h, nb, nb)), vc2, 0.7)                # equal keys
    assert np.allclose(flat, np.broadcast_to(vc2.mean(axis=1, keepdims=True), flat.shape), atol=1e-14)


def test_compressed_two_key_closed_form(oracle):
    # One query block, two pooled keys: out = (e^{a s0} v0 + e^{a s1} v1) / (e^{a s0} + e^{a s1}).
    s = np.array([[[0.4, -1.1], [2.0, 0.5]]])
    vc = np.array([[[1.0, 10.0], [3.0, -4.0]]])
    a = 0.25
    out = oracle.compressed_attn(s, vc, a)
    for i in range(2):
        w0, w1 = math.exp(a * s[0, i, 0]), math.exp(a * s[0, i, 1])
        ref = (w0 * vc[0, 0] + w1 * vc[0, 1]) / (w0 + w1)
        assert np.allclose(out[0, i], ref, atol=1e-15)


def test_compressed_no_overflow_on_large_logits(oracle):
    s = np.array([[[900.0, 899.0, -900.0]]])
    vc = np.array([[[1.0], [2.0], [3.0]]])
    out = oracle.compressed_attn(s, vc, 1.0)
    ref = (1.0 + 2.0 * math.exp(-1.0)) / (1.0 + math.exp(-1.0))
    assert np.isfinite(out).all() and abs(out[0, 0, 0] - ref) < 1e-14


# -------------------------------------------------------------------- TopK --

def test_topk_bruteforce_sort(oracle):
    rng = np.random.default_rng(13)
    s = rng.standard_normal((3, 17, 41))
    for k in (1, 5, 40, 41):
        idx = oracle.topk(s, k)
        for h in range(3):
            for r in range(17):
                order = sorted(range(41), key=lambda j: (-s[h, r, j], j))[:k]
                assert list(idx[h, r]) == sorted(order)


def test_topk_ties_prefer_smaller_index_and_ascending_output(oracle):
    s = np.array([[[1.0, 3.0, 3.0, 0.0, 3.0, 3.0, 2.0]]])
    assert list(oracle.topk(s, 2)[0, 0]) == [1, 2]
    assert list(oracle.topk(s, 3)[0, 0]) == [1, 2, 4]
    assert list(oracle.topk(s, 5)[0, 0]) == [1, 2, 4, 5, 6]
    assert list(oracle.topk(np.zeros((1, 1, 6)), 4)[0, 0]) == [0, 1, 2, 3]
    assert list(oracle.topk(s, 7)[0, 0]) == list(range(7))


def test_topk_planted_blocks_and_scale_invariance(oracle):
    # Block-constant K with orthogonal block means a_j e_j; a query block whose mean is
    # sum_j w_j e_j scores w_j a_j against block j, so the winners are known in advance.
    n_blk, b, d = 8, 4, 8
    a = np.array([1.0, 2.0, 0.5, 1.75, 1.0, 3.0, 0.25, 1.0])       # all exactly representable
    k = np.zeros((n_blk * b, 1, d), dtype=np.float32)
    for j in range(n_blk):
        k[j * b:(j + 1) * b, 0, j] = a[j]
    w = np.array([0.875, 0.125, 1.0, 0.5, -2.0, 0.25, 3.0, 0.0625])
    q = np.tile(w.astype(np.float32), (n_blk * b, 1)).reshape(n_blk * b, 1, d)
    planted = w * a                     # [0.875, 0.25, 0.5, 0.875, -2, 0.75, 0.75, 0.0625]
    qc, kc = oracle.pool(q, b), oracle.pool(k, b)
    s = oracle.scores(qc, kc)
    assert np.array_equal(s[0, 0], planted)
    assert list(oracle.topk(s, 2)[0, 5]) == [0, 3]             # 0.875 twice
    assert list(oracle.topk(s, 1)[0, 5]) == [0]                # exact tie -> smaller index
    assert list(oracle.topk(s, 3)[0, 5]) == [0, 3, 5]          # 0.75 at j = 5 and 6 -> j = 5
    idx = oracle.topk(s, 4)
    assert np.array_equal(idx, oracle.topk(oracle.scores(oracle.pool(q * 8, b), kc), 4))


def test_topk_with_forced_bruteforce_and_edges(oracle):
    # Sec. 3.3: fixed blocks join every row's set and leave the TopK competition.
    rng = np.random.default_rng(14)
    s = rng.standard_normal((2, 9, 23))
    for forced, k in (([0, 1, 2], 4), ([5], 1), ([0, 11, 22], 20), ([3, 4, 9, 10], 30), ([], 6)):
        idx = oracle.topk_with_forced(s, k, forced)
        k_dyn = min(k, 23 - len(forced))
        assert idx.shape == (2, 9, len(forced) + k_dyn)
        for h in range(2):
            for r in range(9):
                rest = [j for j in range(23) if j not in forced]
                best = sorted(rest, key=lambda j: (-s[h, r, j], j))[:k_dyn]
                assert list(idx[h, r]) == sorted(best + list(forced))
    assert np.array_equal(oracle.topk_with_forced(s, 6, []), oracle.topk(s, 6))
    every = list(range(23))
    assert np.array_equal(oracle.topk_with_forced(s, 4, every)[1, 3], every)      # k_dyn = 0
    # a forced block that would have won anyway frees its slot for the runner-up
    t = np.array([[[9.0, 1.0, 8.0, 7.0, 2.0]]])
    assert list(oracle.topk(t, 2)[0, 0]) == [0, 2]
    assert list(oracle.topk_with_forced(t, 2, [0])[0, 0]) == [0, 2, 3]
    assert list(oracle.topk_with_forced(t, 2, [4])[0, 0]) == [0, 2, 4]
    # ties among the free blocks still go to the smaller index
    u = np.array([[[5.0, 5.0, 5.0, 5.0, 5.0]]])
    assert list(oracle.topk_with_forced(u, 2, [1])[0, 0]) == [0, 1, 2]
    with pytest.raises(AssertionError):
        oracle.topk_with_forced(s, 2, [4, 4])
    with pytest.raises(AssertionError):
        oracle.topk_with_forced(s, 2, [7, 3])


# ------------------------------------------------------ selection attention --

@pytest.mark.parametrize("n,block", [(48, 8), (45, 8), (50, 16)])
def test_select_all_blocks_equals_dense_sdpa(oracle, n, block):
    h, d = 2, 8
    q, k, v = rnd((n, h, d), 14), rnd((n, h, d), 15), rnd((n, h, d), 16)
    n_blk = (n + block - 1) // block
    idx = np.broadcast_to(np.arange(n_blk, dtype=np.int32), (h, n_blk, n_blk))
    o_rows, lse_rows = oracle.select_attn(q, k, v, block, idx, 0.35)
    o = flat_tokens(oracle, o_rows, n, block)
    ref = sdpa64(q, k, v, 0.35)
    assert np.allclose(o, ref, rtol=0, atol=1e-13)
    dense, dlse = oracle.dense_attn(q, k, v, 0.35, want_lse=True)
    assert np.allclose(dense, ref, rtol=0, atol=1e-13)
    lse = flat_tokens(oracle, lse_rows.transpose(1, 2, 0), n, block)          # [n, h]
    assert np.allclose(lse, dlse.T, atol=1e-12)
    logits = 0.35 * np.einsum("thd,uhd->htu", q.astype(np.float64), k.astype(np.float64))
    assert np.allclose(np.exp(lse.T), np.exp(logits).sum(axis=2), rtol=1e-12)


@pytest.mark.parametrize("n,block,kk", [(40, 8, 2), (37, 8, 3), (64, 16, 1), (23, 4, 4)])
def test_select_matches_masked_dense_bruteforce(oracle, n, block, kk):
    h, d = 3, 6
    q, k, v = rnd((n, h, d), 17), rnd((n, h, d), 18), rnd((n, h, d), 19)
    n_blk = (n + block - 1) // block
    rng = np.random.default_rng(20)
    idx = np.stack([[np.sort(rng.choice(n_blk, kk, replace=False)) for _ in range(n_blk)]
                    for _ in range(h)]).astype(np.int32)
    o_rows, lse_rows = oracle.select_attn(q, k, v, block, idx, 0.5)
    o = flat_tokens(oracle, o_rows, n, block)
    lse = flat_tokens(oracle, lse_rows.transpose(1, 2, 0), n, block)
    ref, ref_lse = masked_dense_bruteforce(q, k, v, idx, block, 0.5)
    assert np.allclose(o, ref, rtol=0, atol=1e-13)
    assert np.allclose(lse.T, ref_lse, rtol=0, atol=1e-12)


def test_select_two_key_closed_form_and_v_not_k(oracle):
    # One query, block = 1, two selected keys: hand-computed softmax average.
    q = np.array([[[1.0, 2.0]], [[0.0, 0.0]], [[0.0, 0.0]]], dtype=np.float32)
    k = np.array([[[9.0, 9.0]], [[1.0, 0.0]], [[0.0, 1.0]]], dtype=np.float32)
    v = np.array([[[5.0, 5.0]], [[1.0, -1.0]], [[4.0, 2.0]]], dtype=np.float32)
    idx = np.array([[[1, 2], [1, 2], [1, 2]]], dtype=np.int32)
    o, lse = oracle.select_attn(q, k, v, 1, idx, 0.5)
    w1, w2 = math.exp(0.5 * 1.0), math.exp(0.5 * 2.0)
    assert np.allclose(o[0, 0, 0], (w1 * v[1, 0] + w2 * v[2, 0]) / (w1 + w2), atol=1e-15)
    assert abs(lse[0, 0, 0] - math.log(w1 + w2)) < 1e-15
    assert np.allclose(o[1, 0, 0], (v[1, 0] + v[2, 0]) / 2, atol=1e-15)          # zero query


def test_select_permuting_tokens_inside_a_key_block_changes_nothing(oracle):
    n, h, d, b = 32, 2, 4, 8
    q, k, v = rnd((n, h, d), 21), rnd((n, h, d), 22), rnd((n, h, d), 23)
    idx = np.array([[[1, 3]] * 4] * h, dtype=np.int32)
    o1, l1 = oracle.select_attn(q, k, v, b, idx, 0.5)
    perm = np.arange(n)
    perm[8:16] = perm[8:16][::-1]
    o2, l2 = oracle.select_attn(q, k[perm], v[perm], b, idx, 0.5)
    assert np.allclose(o1, o2, atol=1e-14) and np.allclose(l1, l2, atol=1e-14)
    o3, _ = oracle.select_attn(q, k[perm], v, b, idx, 0.5)                     # K moved without V
    assert not np.allclose(o1, o3, atol=1e-6)


def test_select_rows_subset_and_tail_rows(oracle):
    n, h, d, b = 27, 2, 4, 8                       # 4 blocks, tail of 3 tokens
    q, k, v = rnd((n, h, d), 24), rnd((n, h, d), 25), rnd((n, h, d), 26)
    idx = np.array([[[0, 3], [1, 2], [2, 3], [0, 3]]] * h, dtype=np.int32)
    full, full_lse = oracle.select_attn(q, k, v, b, idx, 0.5)
    rows = np.array([3, 1])
    sub, sub_lse = oracle.select_attn(q, k, v, b, idx[:, rows], 0.5, rows=rows)
    assert np.array_equal(sub, full[rows]) and np.array_equal(sub_lse, full_lse[:, rows])
    assert np.all(full[3, 3:] == 0.0)              # rows past n_tok are zero-filled
    ref, _ = masked_dense_bruteforce(q, k, v, idx, b, 0.5)
    assert np.allclose(full[3, :3], ref[24:27], atol=1e-13)   # tail keys beyond n_tok are absent


# ------------------------------------------------------------------- merge --

def test_merge_gate_forms(oracle):
    n, h, d, b = 20, 2, 4, 8
    n_blk = 3
    oc = np.random.default_rng(27).standard_normal((h, n_blk, d))
    osel = np.random.default_rng(28).standard_normal((n_blk, b, h, d))
    up = np.broadcast_to(oc.transpose(1, 0, 2)[:, None], (n_blk, b, h, d))      # eq. 5
    valid = (np.arange(n_blk)[:, None] * b + np.arange(b)[None, :]) < n
    out = oracle.merge(oc, osel, None, n, b)
    assert np.allclose(out[valid], 0.5 * (up + osel)[valid], atol=1e-15)
    assert np.all(out[~valid] == 0)
    big = np.full((n, h, d), 80.0, dtype=np.float32)
    assert np.allclose(oracle.merge(oc, osel, big, n, b)[valid], up[valid], atol=1e-12)
    assert np.allclose(oracle.merge(oc, osel, -big, n, b)[valid], osel[valid], atol=1e-12)
    g_log = rnd((n, h, d), 29)
    out_g = flat_tokens(oracle, oracle.merge(oc, osel, g_log, n, b), n, b)
    g = 1.0 / (1.0 + np.exp(-g_log.astype(np.float64)))
    ref = g * flat_tokens(oracle, up, n, b) + (1 - g) * flat_tokens(oracle, osel, n, b)
    assert np.allclose(out_g, ref, atol=1e-15)


# ------------------------------------------------------------- end to end --

def test_forward_constant_v_gives_constant_out(oracle):
    n, h, d = 100, 2, 8
    q, k = rnd((n, h, d), 30), rnd((n, h, d), 31)
    v = np.ones((n, h, d), dtype=np.float32)
    res = oracle.gsa_forward(q, k, v, 16, 3, gate=rnd((n, h, d), 32))
    out = flat_tokens(oracle, res["out"], n, 16)
    assert np.allclose(out, 1.0, atol=1e-14)


def test_forward_full_topk_and_block1_reduce_to_dense(oracle):
    n, h, d = 60, 2, 8
    q, k, v = rnd((n, h, d), 33), rnd((n, h, d), 34), rnd((n, h, d), 35)
    dense = sdpa64(q, k, v, 1 / math.sqrt(d))
    res = oracle.gsa_forward(q, k, v, 8, 1000)                   # topk clamped to n_blk
    assert res["k"] == 8
    assert np.allclose(flat_tokens(oracle, res["o_sel"], n, 8), dense, atol=1e-13)
    res1 = oracle.gsa_forward(q, k, v, 1, 60)
    assert np.allclose(res1["o_comp"].transpose(1, 0, 2), dense, atol=1e-13)
    assert np.allclose(flat_tokens(oracle, res1["out"], n, 1), dense, atol=1e-13)


# ---- variant: unpooled queries in the compression branch ("queries against the pooled keys") ----

def test_token_queries_block1_is_dense_attention(oracle):
    """Block size 1: pooled keys/values are the keys/values themselves, so every token's compressed
    output is plain softmax attention (library cross-check), and with all blocks selected the merged
    output is dense attention too."""
    n, h, d = 50, 2, 8
    q, k, v = rnd((n, h, d), 60), rnd((n, h, d), 61), rnd((n, h, d), 62)
    scale = 1 / math.sqrt(d)
    dense = sdpa64(q, k, v, scale)
    kc, vc = oracle.pool(k, 1), oracle.pool(v, 1)
    assert np.allclose(oracle.compressed_attn_tokens(q, kc, vc, scale), dense, atol=1e-13)
    res = oracle.gsa_forward(q, k, v, 1, n, token_queries=True, gate=rnd((n, h, d), 63))
    assert np.allclose(flat_tokens(oracle, res["out"], n, 1), dense, atol=1e-13)


def test_token_queries_bruteforce_loops(oracle):
    """Tiny case against pure-Python loops written from the definition."""
    n, h, d, block = 11, 2, 4, 4
    q, k, v = rnd((n, h, d), 64), rnd((n, h, d), 65), rnd((n, h, d), 66)
    scale = 0.37
    kc, vc = oracle.pool(k, block), oracle.pool(v, block)
    got = oracle.compressed_attn_tokens(q, kc, vc, scale)
    n_blk = kc.shape[1]
    for t in range(n):
        for hh in range(h):
            logit = [scale * sum(float(q[t, hh, c]) * kc[hh, j, c] for c in range(d)) for j in range(n_blk)]
            mx = max(logit)
            w = [math.exp(x - mx) for x in logit]
            for c in range(d):
                want = sum(w[j] * vc[hh, j, c] for j in range(n_blk)) / sum(w)
                assert abs(got[t, hh, c] - want) < 1e-13


def test_token_queries_equal_pooled_queries_when_a_block_shares_one_query(oracle):
    """If all tokens of a block carry the same query, pooling the queries changes nothing: the two
    variants must agree, compressed outputs and merged outputs alike (ragged last block included)."""
    n, h, d, block = 45, 2, 8, 8
    n_blk = (n + block - 1) // block
    qb = rnd((n_blk, h, d), 67)
    q = np.repeat(qb, block, axis=0)[:n].copy()
    k, v, gate = rnd((n, h, d), 68), rnd((n, h, d), 69), rnd((n, h, d), 70)
    a = oracle.gsa_forward(q, k, v, block, 3, gate=gate)
    b = oracle.gsa_forward(q, k, v, block, 3, gate=gate, token_queries=True)
    assert np.array_equal(a["idx"], b["idx"])
    up = np.repeat(a["o_comp"].transpose(1, 0, 2)[:, None], block, axis=1)       # [n_blk, block, h, d]
    valid = (np.arange(n_blk * block) < n).reshape(n_blk, block)
    assert np.allclose(b["o_comp_tok"][valid], up[valid], atol=1e-13)
    assert np.allclose(b["out"][valid], a["out"][valid], atol=1e-13)


def test_token_queries_invariants(oracle):
    """Constant values give that constant; permuting the pooled keys and values together changes
    nothing; the gate at +-80 returns one branch or the other; rows beyond n_tok are zero."""
    n, h, d, block = 37, 2, 8, 8
    q, k, v = rnd((n, h, d), 71), rnd((n, h, d), 72), rnd((n, h, d), 73)
    kc, vc = oracle.pool(k, block), oracle.pool(v, block)
    ones = np.full_like(vc, 3.5)
    assert np.allclose(oracle.compressed_attn_tokens(q, kc, ones, 0.2), 3.5, atol=1e-13)
    perm = np.random.default_rng(0).permutation(kc.shape[1])
    assert np.allclose(oracle.compressed_attn_tokens(q, kc[:, perm], vc[:, perm], 0.2),
                       oracle.compressed_attn_tokens(q, kc, vc, 0.2), atol=1e-13)
    hi = oracle.gsa_forward(q, k, v, block, 2, gate=np.full((n, h, d), 80.0, np.float32), token_queries=True)
    lo = oracle.gsa_forward(q, k, v, block, 2, gate=np.full((n, h, d), -80.0, np.float32), token_queries=True)
    assert np.allclose(hi["out"], hi["o_comp_tok"], atol=1e-13)
    valid = (np.arange(hi["out"].shape[0] * block) < n).reshape(-1, block)
    assert np.allclose(lo["out"][valid], lo["o_sel"][valid], atol=1e-13)
    assert np.all(hi["out"][~valid] == 0.0)
    rows = np.array([4, 1])
    part = oracle.gsa_forward(q, k, v, block, 2, token_queries=True, rows=rows)
    full = oracle.gsa_forward(q, k, v, block, 2, token_queries=True)
    assert np.allclose(part["out"], full["out"][rows], atol=1e-13)


def test_forward_agrees_with_bruteforce_route(oracle):
    # Two independently written CPU routes on one small problem (ragged tail, 3 heads).
    n, h, d, b, kk = 77, 3, 8, 8, 3
    q, k, v = rnd((n, h, d), 36), rnd((n, h, d), 37), rnd((n, h, d), 38)
    gate = rnd((n, h, d), 39)
    res = oracle.gsa_forward(q, k, v, b, kk, gate=gate)
    n_blk = 10
    q64, k64, v64 = (a.astype(np.float64) for a in (q, k, v))
    lens = np.minimum(b, n - np.arange(n_blk) * b)
    pad = n_blk * b - n

    def means(x):
        xp = np.concatenate([x, np.zeros((pad,) + x.shape[1:])]).reshape(n_blk, b, h, -1)
        return xp.sum(axis=1) / lens[:, None, None]                       # [n_blk, h, d]

    qc, kc, vc = means(q64), means(k64), means(v64)
    scale = 1 / math.sqrt(d)
    out_ref = np.zeros((n, h, d))
    idx_ref = np.zeros((h, n_blk, kk), dtype=np.int32)
    for hh in range(h):
        s = qc[:, hh] @ kc[:, hh].T
        p = np.exp(scale * s - (scale * s).max(axis=1, keepdims=True))
        ocomp = (p / p.sum(axis=1, keepdims=True)) @ vc[:, hh]
        for i in range(n_blk):
            idx_ref[hh, i] = sorted(sorted(range(n_blk), key=lambda j: (-s[i, j], j))[:kk])
        osel, _ = masked_dense_bruteforce(q[:, hh:hh + 1], k[:, hh:hh + 1], v[:, hh:hh + 1],
                                          idx_ref[hh:hh + 1], b, scale)
        g = 1 / (1 + np.exp(-gate[:, hh].astype(np.float64)))
        out_ref[:, hh] = g * ocomp[np.arange(n) // b] + (1 - g) * osel[:, 0]
    assert np.array_equal(res["idx"], idx_ref)
    assert np.allclose(flat_tokens(oracle, res["out"], n, b), out_ref, rtol=0, atol=1e-13)


def test_forward_with_forced_blocks(oracle):
    n, h, d, b = 90, 2, 8, 8                                   # 12 blocks, ragged tail
    q, k, v = rnd((n, h, d), 40), rnd((n, h, d), 41), rnd((n, h, d), 42)
    scale = 1 / math.sqrt(d)
    forced = [0, 1, 7]
    res = oracle.gsa_forward(q, k, v, b, 3, forced=forced)
    plain = oracle.gsa_forward(q, k, v, b, 3)
    assert res["idx"].shape == (h, 12, 6)
    assert np.all(np.isin(forced, res["idx"]).reshape(-1))
    for hh in range(h):
        for r in range(12):
            assert set(forced) <= set(res["idx"][hh, r])
    # the compressed branch does not depend on the selection set
    assert np.array_equal(res["o_comp"], plain["o_comp"])
    # selection branch = masked dense attention over the united set
    osel, _ = masked_dense_bruteforce(q, k, v, res["idx"], b, scale)
    assert np.allclose(flat_tokens(oracle, res["o_sel"], n, b), osel, rtol=0, atol=1e-13)
    # forcing every block is dense attention
    full = oracle.gsa_forward(q, k, v, b, 1, forced=list(range(12)))
    assert np.allclose(flat_tokens(oracle, full["o_sel"], n, b), sdpa64(q, k, v, scale), atol=1e-13)
    # forcing exactly the blocks TopK picks anyway for one row adds the next-best ones there
    row = plain["idx"][0, 4]
    again = oracle.gsa_forward(q, k, v, b, 3, forced=list(row))
    assert set(row) < set(again["idx"][0, 4]) and again["idx"].shape[2] == 6


def test_layer_special_tokens_dense_and_concat_order(oracle):
    # Eq. 2 for the special rows, eqs. 3-8 among the image rows, results back in place.
    T, s_, views, h, d, b = 13, 2, 3, 2, 8, 4                  # 11 image tokens per view: blocks straddle views
    n = T * views
    q, k, v = rnd((n, h, d), 50), rnd((n, h, d), 51), rnd((n, h, d), 52)
    gate = rnd((n, h, d), 53)
    scale = 1 / math.sqrt(d)
    res = oracle.gsa_layer(q, k, v, b, 3, T, s_, gate=gate)
    spec = [t for t in range(n) if t % T < s_]
    img = [t for t in range(n) if t % T >= s_]
    assert list(res["spec_rows"]) == spec and list(res["img_rows"]) == img
    dense = sdpa64(q, k, v, scale)                               # every row over every key
    assert np.allclose(res["out"][spec], dense[spec], atol=1e-13)
    # image rows: the plain path on the image tokens alone (special keys never enter it)
    alone = oracle.gsa_forward(q[img], k[img], v[img], b, 3, gate=gate[img])
    assert np.array_equal(res["img"]["idx"], alone["idx"])
    assert np.allclose(res["out"][img], flat_tokens(oracle, alone["out"], len(img), b), atol=0)
    # topk >= n_blk: the selection branch is dense attention among the image tokens only
    full = oracle.gsa_layer(q, k, v, b, 100, T, s_)
    o_sel = flat_tokens(oracle, full["img"]["o_sel"], len(img), b)
    assert np.allclose(o_sel, sdpa64(q[img], k[img], v[img], scale), atol=1e-13)
    assert not np.allclose(o_sel, dense[img], atol=1e-3)        # ... so it differs from attention over all keys
    # no special tokens: the layer is the plain path
    plain = oracle.gsa_layer(q, k, v, b, 3, T, 0, gate=gate)
    ref = oracle.gsa_forward(q, k, v, b, 3, gate=gate)
    assert plain["spec_rows"].size == 0
    assert np.array_equal(plain["out"], flat_tokens(oracle, ref["out"], n, b))


def test_layer_row_bookkeeping_closed_form(oracle):
    # q = k = 0: every softmax is uniform and every TopK is an all-way tie (first k blocks win), so
    # with v[t] = t the outputs are means of known row numbers: any slip in the special / image
    # bookkeeping changes them.
    T, s_, views, b, kk = 7, 2, 4, 3, 2
    n = T * views
    z = np.zeros((n, 1, 4), dtype=np.float32)
    v = np.tile(np.arange(n, dtype=np.float32)[:, None, None], (1, 1, 4))
    res = oracle.gsa_layer(z, z, v, b, kk, T, s_)
    img = [t for t in range(n) if t % T >= s_]                   # 20 image rows -> 7 blocks of 3 (tail 2)
    assert np.array_equal(res["img"]["idx"][0], np.tile([0, 1], (7, 1)))
    o_sel = np.mean(img[:kk * b])                                # rows 2..6 and 9: first two image blocks
    blk_means = [np.mean(img[j * b:(j + 1) * b]) for j in range(7)]
    o_comp = np.mean(blk_means)                                  # uniform over the 7 pooled values
    for t in range(n):
        want = np.mean(np.arange(n)) if t % T < s_ else 0.5 * o_comp + 0.5 * o_sel
        assert np.allclose(res["out"][t], want, atol=1e-12), t


def test_window_blocks_tile_every_grid_cell_once(oracle):
    blocks = oracle.window_blocks(3, 2 + 5 * 7, 2, 5, 7, 4)     # 5 x 7 grid, 4 x 4 windows: 2 x 2 windows per view
    assert len(blocks) == 3 * 4
    assert [len(b) for b in blocks[:4]] == [16, 12, 4, 3]        # full, right edge, bottom edge, corner
    rows = np.concatenate(blocks)
    want = [t for t in range(3 * 37) if t % 37 >= 2]
    assert sorted(rows) == want and len(set(rows)) == len(rows)
    # top-left window of view 1: rows 37 + 2 + y * 7 + x, y, x < 4
    assert list(blocks[4]) == [39 + y * 7 + x for y in range(4) for x in range(4)]
    # right-edge window keeps row-major order over its 3 columns
    assert list(blocks[1][:4]) == [2 + 4, 2 + 5, 2 + 6, 2 + 7 + 4]
    # a window that divides the grid gives equal blocks
    assert {len(b) for b in oracle.window_blocks(2, 16, 0, 4, 4, 2)} == {4}


def test_forward_blocks_agrees_with_the_blocked_route(oracle):
    # The explicit-rows route (numpy, no blocking) and the C route on the same equal-length blocks.
    n, h, d, b, kk = 70, 2, 8, 8, 3                               # ragged tail of 6
    q, k, v = rnd((n, h, d), 60), rnd((n, h, d), 61), rnd((n, h, d), 62)
    gate = rnd((n, h, d), 63)
    blocks = [np.arange(j * b, min((j + 1) * b, n)) for j in range(9)]
    for forced in (None, [0, 4]):
        a = oracle.gsa_forward_blocks(q, k, v, blocks, kk, gate=gate, forced=forced)
        c = oracle.gsa_forward(q, k, v, b, kk, gate=gate, forced=forced)
        assert np.array_equal(a["idx"], c["idx"])
        assert np.allclose(a["o_comp"], c["o_comp"], atol=1e-13)
        assert np.allclose(a["out"], flat_tokens(oracle, c["out"], n, b), atol=1e-13)
        assert np.allclose(a["o_sel"], flat_tokens(oracle, c["o_sel"], n, b), atol=1e-13)
        assert np.allclose(a["lse"].T, flat_tokens(oracle, c["lse"].transpose(1, 2, 0), n, b), atol=1e-13)


def test_forward_blocks_on_windows_closed_form(oracle):
    # q = k = 0, v[t] = t: all softmaxes uniform, TopK takes the first blocks; on a 3 x 5 grid with
    # 2 x 2 windows the first two windows of view 0 hold rows {0, 1, 5, 6} and {2, 3, 7, 8}.
    blocks = oracle.window_blocks(2, 15, 0, 3, 5, 2)
    z = np.zeros((30, 1, 4), dtype=np.float32)
    v = np.tile(np.arange(30, dtype=np.float32)[:, None, None], (1, 1, 4))
    res = oracle.gsa_forward_blocks(z, z, v, blocks, 2)
    o_sel = np.mean([0, 1, 5, 6, 2, 3, 7, 8])
    o_comp = np.mean([np.mean(b) for b in blocks])
    assert np.allclose(res["out"], 0.5 * o_comp + 0.5 * o_sel, atol=1e-12)
    assert np.array_equal(res["idx"][0], np.tile([0, 1], (len(blocks), 1)))


def test_paper_sparse_ratios(oracle):
    """Table 2 prints 94 % (pi3 variant) and 84 % (VGGT variant, reference view always
    attended) at 10 views and top-32; counted on the selection stage both follow from
    one per-view block count B_v: 1 - 32/(10 B_v) and 1 - (32 + B_v)/(10 B_v).  Check
    that the number of key blocks the oracle's TopK hands to the selection stage gives
    those ratios."""
    rows = [ln.split() for ln in open(os.path.join(HERE, "golden", "sparse_ratio_table2.txt"))
            if ln.strip() and not ln.startswith("#")]
    table = {r[0]: (int(r[1]), int(r[2]), int(r[3]), int(r[4])) for r in rows}
    views, topk, _, pct_pi3 = table["pi3"]
    _, _, _, pct_vggt = table["vggt"]
    b_v = topk / (views * (1 - pct_pi3 / 100.0))                 # 53.33 blocks per view
    assert abs((1 - (topk + b_v) / (views * b_v)) * 100 - pct_vggt) < 0.5
    n_blk = round(views * b_v)
    s = np.random.default_rng(40).standard_normal((1, 4, n_blk))
    idx = oracle.topk(s, topk)
    kept = np.array([len(set(r)) for r in idx[0]])
    assert np.all(kept == topk)
    assert round((1 - kept[0] / n_blk) * 100) == pct_pi3
    assert round((1 - (kept[0] + n_blk / views) / n_blk) * 100) == pct_vggt
