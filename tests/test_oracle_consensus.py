"""Pins for the oracle's global-consensus variant (Alg. 1 step 3 summed over all layers and heads)."""
import numpy as np
import pytest

from oracle import laserkv_oracle as O


def make_layers(rng, n_layers, h_q, h_kv, w, s_t, d, L, K, t_ctx=0, shared_planes=False):
    planes = rng.standard_normal((L * K, d))
    out = []
    for _ in range(n_layers):
        out.append(dict(q_win=rng.standard_normal((h_q, w, d)), k_blk=rng.standard_normal((h_kv, s_t, d)),
                        k_ctx=rng.standard_normal((h_kv, t_ctx, d)) if t_ctx else None,
                        planes=planes if shared_planes else rng.standard_normal((L * K, d))))
    return out


def test_one_layer_one_head_is_the_per_head_path():
    rng = np.random.default_rng(1)
    lay = make_layers(rng, 1, 2, 1, 6, 70, 16, 4, 3, t_ctx=5)
    parts = (8, 8, 20, 9)
    c = O.consensus_block(lay, 4, 3, *parts, block_pos0=70)
    st = O.select_block(lay[0]["q_win"], lay[0]["k_blk"], lay[0]["k_ctx"], lay[0]["planes"], 4, 3, *parts, block_pos0=70)
    assert np.array_equal(c["keep"], st["keep"][0])
    assert np.allclose(c["score"], st["s_exact"][0], rtol=0, atol=0)
    assert np.array_equal(c["count"], st["cnt"][0])


def test_sum_is_written_out_term_by_term():
    """Brute force: the summed score / count of every token from explicit loops over layers, heads,
    group members, window queries and tables."""
    rng = np.random.default_rng(2)
    n_layers, h_q, h_kv, w, s_t, d, L, K = 2, 4, 2, 3, 11, 8, 3, 2
    lay = make_layers(rng, n_layers, h_q, h_kv, w, s_t, d, L, K)
    c = O.consensus_block(lay, L, K, 2, 2, 3, 2, block_pos0=0, causal=True)
    g = h_q // h_kv
    score = np.zeros(s_t)
    count = np.zeros(s_t, dtype=np.int64)
    for la in lay:
        for h in range(h_kv):
            for gi in range(g):
                for j in range(w):
                    q = la["q_win"][h * g + gi, j]
                    logits = np.array([q @ la["k_blk"][h, i] / np.sqrt(d) for i in range(s_t)])
                    vis = np.array([i <= s_t - w + j for i in range(s_t)])
                    e = np.where(vis, np.exp(logits - logits[vis].max()), 0.0)
                    score += e / e.sum() / (g * w)
                    for r in range(L):
                        code_q = sum(int(la["planes"][r * K + b] @ q >= 0) << b for b in range(K))
                        for i in range(s_t):
                            code_k = sum(int(la["planes"][r * K + b] @ la["k_blk"][h, i] >= 0) << b for b in range(K))
                            count[i] += int(code_q == code_k)
    assert np.allclose(c["score"], score, rtol=1e-12, atol=1e-15)
    assert np.array_equal(c["count"], count)
    # total probability mass: one unit per (layer, KV head) when there are no look-back keys
    assert abs(c["score"].sum() - n_layers * h_kv) < 1e-9


def test_order_of_layers_and_heads_does_not_matter():
    rng = np.random.default_rng(3)
    lay = make_layers(rng, 3, 4, 2, 4, 60, 16, 4, 4, t_ctx=6)
    parts = (7, 7, 18, 6)
    a = O.consensus_block(lay, 4, 4, *parts, block_pos0=60)
    perm = [lay[2], lay[0], lay[1]]
    for la in perm:  # swap the two KV heads (and their query groups) inside each layer
        la["k_blk"] = la["k_blk"][::-1].copy()
        la["k_ctx"] = la["k_ctx"][::-1].copy()
        la["q_win"] = np.concatenate([la["q_win"][2:], la["q_win"][:2]])
    b = O.consensus_block(perm, 4, 4, *parts, block_pos0=60)
    assert np.allclose(a["score"], b["score"], rtol=1e-13, atol=0)
    assert np.array_equal(a["count"], b["count"])
    assert np.array_equal(a["keep"], b["keep"])


def test_one_head_can_carry_a_token_for_everyone():
    """A token that only one head of one layer attends to strongly is kept for all of them, while the
    per-head rule keeps it for that head alone (the point of aggregating over layers and heads)."""
    rng = np.random.default_rng(4)
    d, s_t, w = 32, 200, 8
    lay = make_layers(rng, 2, 2, 2, w, s_t, d, 4, 6)
    pos = 77
    lay[1]["k_blk"][1, pos] = 3.0 * lay[1]["q_win"][1, 2]      # layer 1, KV head 1 (G = 1): a needle
    parts = (10, 10, 6, 0)                                      # exact stage only, few slots
    c = O.consensus_block(lay, 4, 6, *parts, block_pos0=0)
    assert pos in c["keep"]
    kept_by = [(li, h) for li, la in enumerate(lay)
               for h in range(2)
               if pos in O.select_block(la["q_win"], la["k_blk"], None, la["planes"], 4, 6, *parts)["keep"][h]]
    assert kept_by == [(1, 1)]


def test_kept_set_invariants_and_end_points():
    rng = np.random.default_rng(5)
    lay = make_layers(rng, 2, 4, 2, 5, 90, 16, 5, 3)
    c = O.consensus_block(lay, 5, 3, 9, 9, 0, 30, block_pos0=0)      # alpha = 0: counts only
    cand = np.arange(9, 81)
    order = cand[np.lexsort((cand, -c["count"][cand]))][:30]
    assert np.array_equal(np.sort(order), c["k_lsh_set"])
    c = O.consensus_block(lay, 5, 3, 9, 9, 30, 0, block_pos0=0)      # alpha = 1: scores only
    order = cand[np.lexsort((cand, -c["score"][cand]))][:30]
    assert np.array_equal(np.sort(order), c["k_exact_set"])
    assert len(c["keep"]) == 48 and np.all(np.diff(c["keep"]) > 0)
    assert set(range(9)) <= set(c["keep"]) and set(range(81, 90)) <= set(c["keep"])
