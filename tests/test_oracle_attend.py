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
