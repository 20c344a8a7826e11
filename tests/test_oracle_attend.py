"""Pins for the oracle's attention over the compacted cache (Sec. 3 first paragraph).

attend_cache is a textbook definition, so the pins are a library routine, closed forms, a brute-force
loop, and the identities that fix the meaning of the reported log-sum-exp.
"""
import math

import numpy as np
import torch

from oracle import laserkv_oracle as O


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_matches_library_attention_with_grouped_heads():
    h_q, h_kv, n_q, d, cap, n = 6, 2, 5, 16, 40, 33
    q, k, v = _rand((h_q, n_q, d), 1), _rand((h_kv, cap, d), 2), _rand((h_kv, cap, d), 3)
    out, lse = O.attend_cache(q, k, v, n)
    g = h_q // h_kv
    tq = torch.from_numpy(q)[None]
    tk = torch.from_numpy(k[:, :n]).repeat_interleave(g, dim=0)[None]   # query head h*G+g reads KV head h
    tv = torch.from_numpy(v[:, :n]).repeat_interleave(g, dim=0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    ref_lse = torch.logsumexp(torch.einsum("hqd,hkd->hqk", tq[0], tk[0]) / math.sqrt(d), dim=-1).numpy()
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)


def test_brute_force_loops():
    h_q, h_kv, n_q, d, n = 4, 2, 2, 3, 5
    q, k, v = _rand((h_q, n_q, d), 4), _rand((h_kv, n + 2, d), 5), _rand((h_kv, n + 2, d), 6)
    out, lse = O.attend_cache(q, k, v, n)
    for hq in range(h_q):
        h = hq // 2
        for j in range(n_q):
            l = [sum(q[hq, j, x] * k[h, i, x] for x in range(d)) / math.sqrt(d) for i in range(n)]
            z = sum(math.exp(t) for t in l)
            assert abs(lse[hq, j] - math.log(z)) < 1e-12
            for x in range(d):
                want = sum(math.exp(l[i]) / z * v[h, i, x] for i in range(n))
                assert abs(out[hq, j, x] - want) < 1e-12


def test_equal_keys_give_the_mean_value_and_a_closed_form_lse():
    h_q, h_kv, d, n = 2, 1, 8, 7
    q = _rand((h_q, 3, d), 7)
    k1 = _rand((d,), 8)
    k = np.tile(k1, (h_kv, n + 3, 1))
    v = _rand((h_kv, n + 3, d), 9)
    out, lse = O.attend_cache(q, k, v, n)
    np.testing.assert_allclose(out, np.broadcast_to(v[0, :n].mean(axis=0), out.shape), rtol=1e-12)
    np.testing.assert_allclose(lse, q @ k1 / math.sqrt(d) + math.log(n), rtol=1e-12)


def test_rows_past_the_length_are_never_read():
    q, k, v = _rand((2, 2, 4), 10), _rand((1, 9, 4), 11), _rand((1, 9, 4), 12)
    a = O.attend_cache(q, k, v, 6)
    k[:, 6:] = np.nan
    v[:, 6:] = np.nan
    b = O.attend_cache(q, k, v, 6)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    out, lse = O.attend_cache(q, k, v, 0)
    assert not out.any() and np.all(np.isneginf(lse))


def test_two_segments_merge_through_their_lse():
    """Attention over rows [0, n) is the lse-weighted mean of attention over [0, m) and [m, n)."""
    q, k, v = _rand((4, 3, 8), 13), _rand((2, 20, 8), 14), _rand((2, 20, 8), 15)
    full, lse = O.attend_cache(q, k, v, 20)
    a, la = O.attend_cache(q, k, v, 9)
    b, lb = O.attend_cache(q, k[:, 9:], v[:, 9:], 11)
    wa, wb = np.exp(la - lse), np.exp(lb - lse)
    np.testing.assert_allclose(wa + wb, 1.0, rtol=1e-12)
    np.testing.assert_allclose(full, a * wa[..., None] + b * wb[..., None], rtol=1e-11, atol=1e-13)


def test_identity_values_return_the_probabilities_the_score_step_pools():
    """With V = I the output rows are the softmax probabilities; pooled over the window rows and the
    GQA group they are Alg. 1 step 3's S_exact of the same keys without a mask."""
    h_q, h_kv, w, d, n = 4, 2, 3, 8, 8
    q, k = _rand((h_q, w, d), 16), _rand((h_kv, n, d), 17)
    v = np.tile(np.eye(n), (h_kv, 1, 1))
    out, _ = O.attend_cache(q, k, v, n)
    pooled = out.reshape(h_kv, h_q // h_kv * w, n).mean(axis=1)
    np.testing.assert_allclose(pooled, O.exact_scores(q, k, causal=False), rtol=1e-12)


def test_lse_of_the_cache_is_what_the_score_step_takes_as_outside_normaliser():
    """Scores of a block with the cache's keys handed over as look-back keys = scores with only their lse."""
    h_q, h_kv, w, d, s_t, n = 4, 2, 4, 8, 12, 10
    q, kb = _rand((h_q, w, d), 18), _rand((h_kv, s_t, d), 19)
    ck, cv = _rand((h_kv, n + 4, d), 20), _rand((h_kv, n + 4, d), 21)
    _, lse = O.attend_cache(q, ck, cv, n)
    a = O.exact_scores(q, kb, k_ctx=ck[:, :n], block_pos0=100)
    b = O.exact_scores(q, kb, block_pos0=100, row_lse=lse)
    np.testing.assert_allclose(a, b, rtol=1e-12)


# ---- attend_block: the block's prefill attention over [cache | block keys, causal] ----

def test_block_attention_matches_library_attention_with_an_explicit_mask():
    h_q, h_kv, n_q, d, n, s_t = 6, 2, 7, 16, 11, 9
    q, ck, cv = _rand((h_q, n_q, d), 30), _rand((h_kv, n + 3, d), 31), _rand((h_kv, n + 3, d), 32)
    kb, vb = _rand((h_kv, s_t, d), 33), _rand((h_kv, s_t, d), 34)
    block_pos0, q_pos0 = 100, 101          # query j sits at 101 + j: sees block keys 0 .. j + 1
    out, lse = O.attend_block(q, ck, cv, n, kb, vb, block_pos0=block_pos0, q_pos0=q_pos0)
    g = h_q // h_kv
    tq = torch.from_numpy(q)[None]
    tk = torch.from_numpy(np.concatenate([ck[:, :n], kb], axis=1)).repeat_interleave(g, dim=0)[None]
    tv = torch.from_numpy(np.concatenate([cv[:, :n], vb], axis=1)).repeat_interleave(g, dim=0)[None]
    mask = torch.ones(n_q, n + s_t, dtype=torch.bool)
    for j in range(n_q):
        for i in range(s_t):
            mask[j, n + i] = block_pos0 + i <= q_pos0 + j
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    logits = (torch.einsum("hqd,hkd->hqk", tq[0], tk[0]) / math.sqrt(d)).masked_fill(~mask, float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(logits, dim=-1).numpy(), rtol=1e-12, atol=1e-13)


def test_block_attention_hand_worked():
    """d = 1, one head, both queries q = 1, so a logit is the key itself.  Cache: key 0 (value 5).  Block: keys
    ln 2 and ln 4 (values 1 and 3) at positions 10 and 11: exp(logit) is 1, 2, 4.
    Query 0 (position 10) sees the cache row and block key 0: weights 1, 2 -> out (5 + 2) / 3, lse ln 3.
    Query 1 (position 11) sees all three: weights 1, 2, 4 -> out (5 + 2 + 12) / 7, lse ln 7."""
    q = np.array([[[1.0], [1.0]]])
    ck, cv = np.array([[[0.0], [99.0]]]), np.array([[[5.0], [-99.0]]])       # second cache row is past the length
    kb, vb = np.array([[[math.log(2.0)], [math.log(4.0)]]]), np.array([[[1.0], [3.0]]])
    out, lse = O.attend_block(q, ck, cv, 1, kb, vb, block_pos0=10, q_pos0=10)
    np.testing.assert_allclose(out[0, :, 0], [7.0 / 3.0, 19.0 / 7.0], rtol=1e-14)
    np.testing.assert_allclose(lse[0], [math.log(3.0), math.log(7.0)], rtol=1e-14)
    # the default window is the block's last n_q tokens: the same here
    out2, lse2 = O.attend_block(q, ck, cv, 1, kb, vb, block_pos0=10)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)
    # without the mask both queries see everything
    out3, lse3 = O.attend_block(q, ck, cv, 1, kb, vb, block_pos0=10, q_pos0=10, causal=False)
    np.testing.assert_allclose(out3[0, :, 0], [19.0 / 7.0] * 2, rtol=1e-14)
    np.testing.assert_allclose(lse3[0], [math.log(7.0)] * 2, rtol=1e-14)


def test_block_attention_reduces_to_cache_attention_and_merges_through_the_lse():
    h_q, h_kv, n_q, d, n, s_t = 4, 2, 3, 8, 10, 6
    q, ck, cv = _rand((h_q, n_q, d), 35), _rand((h_kv, n, d), 36), _rand((h_kv, n, d), 37)
    kb, vb = _rand((h_kv, s_t, d), 38), _rand((h_kv, s_t, d), 39)
    # no block keys: attention over the cache
    a = O.attend_block(q, ck, cv, n, kb[:, :0], vb[:, :0], block_pos0=50, q_pos0=50)
    b = O.attend_cache(q, ck, cv, n)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-13)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-13)
    # without a mask the block keys are just more cache rows
    c = O.attend_block(q, ck, cv, n, kb, vb, causal=False)
    e = O.attend_cache(q, np.concatenate([ck, kb], axis=1), np.concatenate([cv, vb], axis=1), n + s_t)
    np.testing.assert_allclose(c[0], e[0], rtol=1e-12)
    np.testing.assert_allclose(c[1], e[1], rtol=1e-12)
    # cache part and causal block part merge through their log-sum-exps
    full, lse = O.attend_block(q, ck, cv, n, kb, vb, block_pos0=50, q_pos0=52)
    blk, lb = O.attend_block(q, ck, cv, 0, kb, vb, block_pos0=50, q_pos0=52)
    wa, wb = np.exp(b[1] - lse), np.exp(lb - lse)
    np.testing.assert_allclose(wa + wb, 1.0, rtol=1e-12)
    np.testing.assert_allclose(full, b[0] * wa[..., None] + blk * wb[..., None], rtol=1e-11, atol=1e-13)


def test_block_attention_never_looks_ahead():
    """Changing a block key or value at position p leaves every query before p untouched; queries before the
    block see the cache only, and see nothing when the cache is empty."""
    h_q, h_kv, n_q, d, n, s_t = 2, 1, 6, 4, 5, 6
    q, ck, cv = _rand((h_q, n_q, d), 40), _rand((h_kv, n, d), 41), _rand((h_kv, n, d), 42)
    kb, vb = _rand((h_kv, s_t, d), 43), _rand((h_kv, s_t, d), 44)
    base = O.attend_block(q, ck, cv, n, kb, vb, block_pos0=20, q_pos0=18)     # queries at 18 .. 23, keys at 20 .. 25
    kb2, vb2 = kb.copy(), vb.copy()
    kb2[:, 3:] += 7.0
    vb2[:, 3:] -= 3.0                                                         # keys at 23, 24, 25 change
    other = O.attend_block(q, ck, cv, n, kb2, vb2, block_pos0=20, q_pos0=18)
    np.testing.assert_array_equal(base[0][:, :5], other[0][:, :5])            # queries at 18 .. 22
    np.testing.assert_array_equal(base[1][:, :5], other[1][:, :5])
    assert np.all(base[0][:, 5] != other[0][:, 5])
    cache_only = O.attend_cache(q, ck, cv, n)
    np.testing.assert_allclose(base[0][:, :2], cache_only[0][:, :2], rtol=1e-13)   # queries at 18, 19
    np.testing.assert_allclose(base[1][:, :2], cache_only[1][:, :2], rtol=1e-13)
    empty = O.attend_block(q, ck, cv, 0, kb, vb, block_pos0=20, q_pos0=18)
    assert not empty[0][:, :2].any() and np.all(np.isneginf(empty[1][:, :2])) and np.isfinite(empty[1][:, 2:]).all()


def test_block_attention_lse_is_the_complete_normaliser_of_the_score_step():
    """For the window rows, the block attention's lse over [cache | block] is what exact_scores takes as the
    complete row statistic: scores equal those computed with the cache rows handed over as look-back keys."""
    h_q, h_kv, w, d, s_t, n = 4, 2, 4, 8, 12, 10
    q, kb, vb = _rand((h_q, w, d), 45), _rand((h_kv, s_t, d), 46), _rand((h_kv, s_t, d), 47)
    ck, cv = _rand((h_kv, n + 4, d), 48), _rand((h_kv, n + 4, d), 49)
    _, lse = O.attend_block(q, ck, cv, n, kb, vb, block_pos0=100)
    a = O.exact_scores(q, kb, k_ctx=ck[:, :n], block_pos0=100)
    b = O.exact_scores(q, kb, block_pos0=100, row_lse_complete=lse)
    np.testing.assert_allclose(a, b, rtol=1e-12)
