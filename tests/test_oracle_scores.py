"""Pins for the oracle's exact-score step (Sec. 3.3 "Precision"; Alg. 1 step 3)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import laserkv_oracle as O


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_matches_library_softmax_single_head():
    # T = 0, no mask, G = 1: softmax(Q K^T / sqrt(d)) averaged over the window rows.
    q = _rand((1, 5, 16), 0)
    k = _rand((1, 23, 16), 1)
    got = O.exact_scores(q, k, None, causal=False)
    ref = torch.softmax(torch.from_numpy(q[0]) @ torch.from_numpy(k[0]).T / 4.0, dim=-1).mean(0).numpy()
    np.testing.assert_allclose(got[0], ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("hq,hkv,w,s,t,d,offset", [(4, 2, 6, 20, 0, 8, None), (8, 2, 5, 17, 7, 16, None),
                                                   (6, 3, 4, 12, 3, 32, 4), (2, 2, 3, 9, 2, 8, 100)])
def test_matches_library_attention_with_gqa_mask_and_lookback(hq, hkv, w, s, t, d, offset):
    # Library pin: scaled_dot_product_attention with V = identity returns the probability rows.
    # Its enable_gqa path pairs query head h*G+g with KV head h, and its boolean mask is the
    # causal rule "key position <= query position"; look-back keys are always visible.
    q = _rand((hq, w, d), 10)
    k = _rand((hkv, s, d), 11)
    kc = _rand((hkv, t, d), 12) if t else None
    pos0 = 1000
    q_pos0 = pos0 + s - w if offset is None else pos0 + offset
    got = O.exact_scores(q, k, kc, block_pos0=pos0, q_pos0=q_pos0, causal=True)
    keys = np.concatenate([kc, k], axis=1) if t else k
    n_keys = t + s
    mask = torch.ones(w, n_keys, dtype=torch.bool)
    for j in range(w):
        for i in range(s):
            mask[j, t + i] = (pos0 + i) <= (q_pos0 + j)
    eye = torch.eye(n_keys, dtype=torch.float64).expand(hkv, n_keys, n_keys)
    probs = F.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(keys)[None],
                                           eye[None], attn_mask=mask, enable_gqa=True)[0]   # [hq, w, n_keys]
    g = hq // hkv
    ref = probs.reshape(hkv, g * w, n_keys).mean(1)[:, t:].numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


def test_equal_keys_closed_form_with_causal_mask():
    # All keys equal => every row is uniform over its visible keys.
    hq, hkv, w, s, t, d = 4, 2, 4, 10, 3, 8
    q = _rand((hq, w, d), 3)
    kvec = _rand((d,), 4)
    k = np.broadcast_to(kvec, (hkv, s, d)).copy()
    kc = np.broadcast_to(kvec, (hkv, t, d)).copy()
    got = O.exact_scores(q, k, kc, block_pos0=0, causal=True)     # window = last w block tokens
    expect = np.zeros(s)
    for j in range(w):
        qpos = s - w + j
        n_vis = t + qpos + 1
        for i in range(qpos + 1):
            expect[i] += 1.0 / n_vis
    expect /= w
    for h in range(hkv):
        np.testing.assert_allclose(got[h], expect, rtol=0, atol=1e-14)


def test_mass_conservation_and_lookback_mass():
    q = _rand((4, 8, 16), 5)
    k = _rand((2, 40, 16), 6)
    kc = _rand((2, 9, 16), 7)
    no_ctx = O.exact_scores(q, k, None)
    np.testing.assert_allclose(no_ctx.sum(1), 1.0, atol=1e-13)       # T = 0: the block holds all the mass
    with_ctx = O.exact_scores(q, k, kc)
    assert np.all(with_ctx.sum(1) < 1.0) and np.all(with_ctx >= 0)   # look-back keys take some of it
    assert np.all(with_ctx <= no_ctx + 1e-15)


def test_row_shift_invariance():
    # Adding the same vector u to every key shifts each logit row by a constant.
    q = _rand((4, 8, 16), 8)
    k = _rand((2, 30, 16), 9)
    kc = _rand((2, 5, 16), 10)
    u = _rand((16,), 11) * 3
    a = O.exact_scores(q, k, kc)
    b = O.exact_scores(q, k + u, kc + u)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-15)


def test_masked_keys_score_zero_and_future_window():
    q = _rand((2, 4, 8), 12)
    k = _rand((1, 16, 8), 13)
    s = O.exact_scores(q, k, None, block_pos0=0, q_pos0=5, causal=True)   # queries at positions 5..8
    assert np.all(s[0, 9:] == 0.0) and np.all(s[0, :9] > 0)
    later = O.exact_scores(q, k, None, block_pos0=0, q_pos0=100, causal=True)
    free = O.exact_scores(q, k, None, causal=False)
    np.testing.assert_allclose(later, free, atol=1e-15)                   # prompt-style window: mask never fires


def test_large_logits_are_stable():
    q = _rand((1, 3, 8), 14) * 300
    k = _rand((1, 12, 8), 15) * 300
    s = O.exact_scores(q, k, None, causal=False)
    assert np.isfinite(s).all() and abs(s.sum() - 1) < 1e-12


def test_row_lse_equals_extra_context_keys():
    """Keys summarised by their log-sum-exp must weigh in exactly as if they had been passed as
    look-back keys (which enter the normaliser only)."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(77)
    h_q, h_kv, w, s_t, d, t_in, t_out = 4, 2, 5, 40, 16, 6, 23
    q = rng.standard_normal((h_q, w, d)) * 1.5
    k = rng.standard_normal((h_kv, s_t, d))
    ctx_in = rng.standard_normal((h_kv, t_in, d))
    ctx_out = rng.standard_normal((h_kv, t_out, d)) * 2.0
    g = h_q // h_kv
    row_lse = np.stack([logsumexp(q[hq] @ ctx_out[hq // g].T / np.sqrt(d), axis=1) for hq in range(h_q)])
    a = O.exact_scores(q, k, ctx_in, block_pos0=100, causal=True, row_lse=row_lse)
    b = O.exact_scores(q, k, np.concatenate([ctx_out, ctx_in], axis=1), block_pos0=100, causal=True)
    assert np.allclose(a, b, rtol=1e-12, atol=0)
    # and without look-back keys of its own
    a = O.exact_scores(q, k, None, block_pos0=0, causal=False, row_lse=row_lse)
    b = O.exact_scores(q, k, ctx_out, block_pos0=0, causal=False)
    assert np.allclose(a, b, rtol=1e-12, atol=0)
    # a vanishing outside mass changes nothing; a dominating one takes (almost) all of the probability
    base = O.exact_scores(q, k, None, block_pos0=0)
    assert np.allclose(O.exact_scores(q, k, None, block_pos0=0, row_lse=np.full((h_q, w), -1e4)), base, rtol=1e-13, atol=0)
    assert O.exact_scores(q, k, None, block_pos0=0, row_lse=np.full((h_q, w), 60.0)).sum() < 1e-10


def test_complete_row_lse_reproduces_the_plain_path_and_library_attention():
    """Sec. 3.3 "Precision": the exact score is the attention the model computes.  With every window row's
    complete log-sum-exp (over the keys it sees in the block, the look-back keys and any further context)
    the scores must equal the plain path's, and equal library attention weights taken with that normaliser."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(91)
    h_q, h_kv, w, s_t, d, t_in, t_far = 6, 2, 4, 33, 8, 5, 17
    g = h_q // h_kv
    q = rng.standard_normal((h_q, w, d)) * 1.3
    k = rng.standard_normal((h_kv, s_t, d))
    ctx_in = rng.standard_normal((h_kv, t_in, d))
    far = rng.standard_normal((h_kv, t_far, d)) * 1.7       # the rest of the cache: never passed to the call
    pos0, qpos0 = 200, 200 + s_t - w
    vis = (pos0 + np.arange(s_t))[None, :] <= (qpos0 + np.arange(w))[:, None]
    lse = np.zeros((h_q, w))
    for hq in range(h_q):
        h = hq // g
        l_blk = np.where(vis, q[hq] @ k[h].T / np.sqrt(d), -np.inf)
        l_all = np.concatenate([q[hq] @ far[h].T / np.sqrt(d), q[hq] @ ctx_in[h].T / np.sqrt(d), l_blk], axis=1)
        lse[hq] = logsumexp(l_all, axis=1)
    got = O.exact_scores(q, k, None, block_pos0=pos0, row_lse_complete=lse)
    plain = O.exact_scores(q, k, np.concatenate([far, ctx_in], axis=1), block_pos0=pos0)
    np.testing.assert_allclose(got, plain, rtol=1e-12, atol=0)
    # look-back keys and an outside log-sum-exp passed along are ignored: the normaliser is already complete
    same = O.exact_scores(q, k, ctx_in, block_pos0=pos0, row_lse=np.zeros((h_q, w)), row_lse_complete=lse)
    np.testing.assert_array_equal(got, same)
    # library attention over [far | look-back | block] with V = one-hot of the block keys gives the same weights
    t = t_far + t_in
    for h in range(h_kv):
        keys = torch.from_numpy(np.concatenate([far[h], ctx_in[h], k[h]], axis=0))
        mask = torch.from_numpy(np.concatenate([np.ones((w, t), dtype=bool), vis], axis=1))
        v_onehot = torch.zeros(t + s_t, s_t, dtype=torch.float64)
        v_onehot[t:] = torch.eye(s_t, dtype=torch.float64)
        acc = np.zeros(s_t)
        for gi in range(g):
            out = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q[h * g + gi])[None], keys[None], v_onehot[None],
                                                                   attn_mask=mask[None])
            acc += out[0].sum(0).numpy()
        np.testing.assert_allclose(got[h], acc / (g * w), rtol=1e-10, atol=0)
    # a normaliser that misses keys (too small) inflates the scores: the total mass exceeds what the block holds
    assert O.exact_scores(q, k, None, block_pos0=pos0, row_lse_complete=lse - 1.0).sum() > got.sum() * 2.7
